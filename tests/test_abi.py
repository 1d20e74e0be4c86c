"""The C-ABI library loads, exports every symbol the header declares, and validates arguments
on the host (no GPU work is launched by any call in this file)."""
import ctypes as C
import os
import re

import pytest

from paper_2407_09105_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2407_09105_amd import build
        build.build()
    return binding.lib()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "varlen_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(va_[a-z_0-9]+)\s*\(", text)))


def test_exports_match_header(L):
    declared = _declared_symbols()
    assert set(declared) == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_plan_bytes(L):
    assert L.va_plan_bytes(0, 16) == 0 and L.va_plan_bytes(1, 0) == 0 and L.va_plan_bytes(-1, 4) == 0
    assert L.va_plan_bytes(65536, 65536) == 0          # N >= 2^31
    b = L.va_plan_bytes(1, 8192)
    assert b >= 4 * (8193 + 3 * 8192 + 8 + 2 * 32) and b % 256 == 0
    assert L.va_plan_bytes(8, 8192) > b


def test_bind_validation(L):
    seg = binding.VaSegments()
    need = L.va_plan_bytes(2, 100)
    fake = 0x10000  # never dereferenced: bind is host pointer arithmetic only
    assert L.va_segments_bind(None, need, 2, 100, C.byref(seg)) == 1
    assert L.va_segments_bind(fake, need, 0, 100, C.byref(seg)) == 2
    assert L.va_segments_bind(fake, need - 1, 2, 100, C.byref(seg)) == 4
    assert L.va_segments_bind(fake + 8, need, 2, 100, C.byref(seg)) == 4      # misaligned
    assert L.va_segments_bind(fake, need, 2, 100, C.byref(seg)) == 0
    ptrs = [getattr(seg, f) for f, _ in binding.VaSegments._fields_]
    assert all(fake <= p < fake + need for p in ptrs) and len(set(ptrs)) == len(ptrs)
    assert seg.cu_seqlens == fake and seg.seg_id - seg.cu_seqlens >= 4 * 201


def _bound(L, rows=1, T=16):
    seg = binding.VaSegments()
    assert L.va_segments_bind(0x10000, L.va_plan_bytes(rows, T), rows, T, C.byref(seg)) == 0
    return seg


def test_pack_validation(L):
    seg = _bound(L)
    p = 0x20000
    assert L.va_pack_to_cu_seqlens(None, binding.VA_I64, 1, 16, C.byref(seg), None) == 1
    assert L.va_pack_to_cu_seqlens(p, binding.VA_I64, 1, 16, None, None) == 1
    assert L.va_pack_to_cu_seqlens(p, binding.VA_I64, 0, 16, C.byref(seg), None) == 2
    assert L.va_pack_to_cu_seqlens(p, 7, 1, 16, C.byref(seg), None) == 3
    assert L.va_pack_to_cu_seqlens(p, binding.VA_I64, 1, 16, C.byref(binding.VaSegments()), None) == 1


def test_collate_validation(L):
    p = 0x10000  # never dereferenced: every call below fails validation
    f = L.va_collate_padding_free
    ok = [p, None, binding.VA_I64, p, 4, 16, 40, 0, p, p, p, p, None]

    def with_(i, v):
        a = list(ok)
        a[i] = v
        return a

    assert f(*with_(4, -1)) == 2            # n_examples < 0
    assert f(*with_(5, 0)) == 2             # padded_len <= 0
    assert f(*with_(6, -1)) == 2            # n_out < 0
    a = with_(4, 1 << 20)
    a[5] = 1 << 12
    assert f(*a) == 2                       # n_examples * padded_len >= 2^31
    assert f(*with_(2, 5)) == 3             # unknown id type
    assert f(*with_(0, None)) == 1 and f(*with_(3, None)) == 1
    assert f(*with_(8, None)) == 1 and f(*with_(9, None)) == 1 and f(*with_(10, None)) == 1
    assert f(*with_(11, None)) == 1


def test_rope_validation(L):
    p = 0x10000  # never dereferenced: every call below fails validation
    f = L.va_rope_apply
    ok = [p, p, binding.VA_BF16, p, binding.VA_I64, 64, 4, 128, 0.0, 0, None]

    def with_(i, v):
        a = list(ok)
        a[i] = v
        return a

    assert f(*with_(5, -1)) == 2 and f(*with_(6, 0)) == 2
    assert f(*with_(7, 0)) == 2 and f(*with_(7, 127)) == 2      # head_dim must be even
    assert f(*with_(7, 258)) == 3
    assert f(*with_(2, 9)) == 3 and f(*with_(4, 9)) == 3
    assert f(*with_(0, None)) == 1 and f(*with_(1, None)) == 1 and f(*with_(3, None)) == 1


def test_attn_validation(L):
    seg = _bound(L)
    p = 0x20000
    fwd = lambda *a: L.va_varlen_attn_fwd(*a)
    ok = [p, p, p, p, p, C.byref(seg), 1, 16, 2, 2, 16, binding.VA_F32, 0.0, None, 0, None]

    def with_(i, val):
        a = list(ok)
        a[i] = val
        return a

    assert fwd(*with_(0, None)) == 1
    assert fwd(*with_(4, None)) == 1
    assert fwd(*with_(5, None)) == 1
    assert fwd(*with_(8, 3)) == 2          # Hq % Hkv != 0
    assert fwd(*with_(9, 0)) == 2
    assert fwd(*with_(10, 512)) == 3       # head_dim > 256
    assert fwd(*with_(11, 9)) == 3         # unknown dtype
    assert fwd(*with_(6, 0)) == 2

    okb = [p] * 9 + [binding.VA_F32, C.byref(seg), 1, 16, 2, 2, 16, binding.VA_F32, 0.0, p, 1 << 20, None]
    bwd = lambda *a: L.va_varlen_attn_bwd(*a)

    def withb(i, val):
        a = list(okb)
        a[i] = val
        return a

    assert bwd(*withb(6, None)) == 1
    assert bwd(*withb(9, 5)) == 3
    # gradient type: fp32, or the inputs' own 16-bit type (bf16 also with fp32 inputs)
    for dt, gdt, bad in ((binding.VA_BF16, binding.VA_F16, True), (binding.VA_F16, binding.VA_BF16, True),
                         (binding.VA_F32, binding.VA_F16, True)):
        a = withb(9, gdt)
        a[16] = dt
        assert (bwd(*a) == 3) == bad
    # MFMA path: 32-bit byte offsets inside one packed row
    big = with_(7, 1 << 20)                                # tokens_per_row 2^20 ...
    big[8], big[9], big[10], big[11] = 64, 64, 128, binding.VA_BF16   # ... x 64 heads x 256 B >= 2^32
    assert fwd(*big) == 3
    big[8], big[9] = 8, 8                                  # 2^20 x 8 x 256 B = 2^31: fine for validation
    big[5] = None
    assert fwd(*big) == 1                                  # (rejected later, for the missing segments)
    assert bwd(*withb(18, None)) == 1                      # workspace required
    assert bwd(*withb(19, 16)) == 4                        # workspace too small
    assert L.va_attn_workspace_bytes(16, 2, 2, 16, 1) >= 16 * 2 * 4
    assert L.va_attn_workspace_bytes(16, 2, 2, 16, 0) == 0
    assert L.va_attn_workspace_bytes(0, 2, 2, 16, 1) == 0


def test_noalloc_backward_validation(L):
    """The backward that allocates nothing validates on the host before it touches the GPU: bad
    arguments and sizes beyond its device array are refused with nothing looked up or launched."""
    seg = _bound(L)
    p = 0x20000
    f = L.va_varlen_attn_bwd_noalloc
    ok = [p] * 9 + [binding.VA_F32, C.byref(seg), 1, 16, 2, 2, 16, binding.VA_F32, 0.0, None]

    def with_(i, val):
        a = list(ok)
        a[i] = val
        return a

    assert f(*with_(0, None)) == 1 and f(*with_(8, None)) == 1 and f(*with_(10, None)) == 1
    assert f(*with_(13, 3)) == 2                           # Hq % Hkv != 0
    assert f(*with_(9, 5)) == 3                            # unknown gradient type
    big = list(ok)
    big[11], big[12], big[13], big[14] = 8, 8192, 256, 256  # D = 65536 tokens x 256 heads x 4 B = 64 MiB
    assert 8 * 8192 * 256 * 4 > binding.NOALLOC_SCRATCH_BYTES
    assert f(*big) == 4                                    # beyond the library's array


def test_probe_library_is_separate_and_validates():
    """The measurement aids live in their own library: the attention library exports none of them, the
    probe library exports what its header declares and rejects what it cannot run before launching."""
    from paper_2407_09105_amd import probes
    text = open(os.path.join(ROOT, "paper_2407_09105_amd", "probes", "va_probes.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert sorted(set(re.findall(r"\b(vap_[a-z_0-9]+)\s*\(", text))) == sorted(probes.EXPORTS)
    P = probes.lib()
    assert not hasattr(binding.lib(), "va_probe_mfma") and not hasattr(binding.lib(), "vap_probe_mfma")
    p = C.c_void_p(0x1000)
    assert P.vap_probe_mfma(None, 10, None, None) == 1
    assert P.vap_probe_mfma(p, 0, None, None) == 2
    assert P.vap_probe_mix(None, 16, 24, p, None, 10, None, None) == 1
    assert P.vap_probe_mix(p, 16, 24, None, None, 10, None, None) == 1
    assert P.vap_probe_mix(p, 16, 24, p, None, 0, None, None) == 2
    assert P.vap_probe_mix(p, 5, 24, p, None, 10, None, None) == 3      # not an instantiated mix
    assert P.vap_probe_mix(p, 8, 24, p, None, 10, None, None) == 3


def test_strings(L):
    assert L.va_status_string(0) == b"ok"
    assert all(L.va_status_string(i) for i in range(7))
    assert b"gfx950" in L.va_version()
