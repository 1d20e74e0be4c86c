"""Pins for the oracle's rotary embedding (the second consumer of the restarting position ids)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_09105_amd import workloads as wl


def test_two_dim_closed_form():
    # d = 2: one pair, frequency base^0 = 1: a plane rotation by `pos` radians, counter-clockwise
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -3.0]]])
    pos = np.array([1, 2, 5])
    y = oracle.rope(x, pos, base=123.0)
    assert np.allclose(y[0, 0], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    assert np.allclose(y[1, 0], [-np.sin(2.0), np.cos(2.0)], atol=1e-15)
    assert np.allclose(y[2, 0], [2 * np.cos(5.0) + 3 * np.sin(5.0), -3 * np.cos(5.0) + 2 * np.sin(5.0)], atol=1e-14)


def test_frequency_ladder_and_pairing():
    # d = 4, base = 10000: pair 0 = (x0, x2) turns by pos, pair 1 = (x1, x3) by pos / 100
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    y = oracle.rope(x, np.array([100]), base=10000.0)
    assert np.allclose(y[0, 0], [np.cos(100.0), np.cos(1.0), np.sin(100.0), np.sin(1.0)], atol=1e-12)
    # d = 8, base = 16: frequencies 1, 1/2, 1/4, 1/8
    x = np.zeros((1, 1, 8)); x[0, 0, :4] = 1.0
    y = oracle.rope(x, np.array([8]), base=16.0)
    ang = 8.0 / np.array([1.0, 2.0, 4.0, 8.0])
    assert np.allclose(y[0, 0, :4], np.cos(ang), atol=1e-14) and np.allclose(y[0, 0, 4:], np.sin(ang), atol=1e-14)


def test_position_zero_is_identity_and_norms_are_kept():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((50, 3, 16))
    pos = rng.integers(0, 5000, size=50)
    pos[::7] = 0
    y = oracle.rope(x, pos)
    assert np.array_equal(y[::7], x[::7])
    pair_norm = lambda z: z[..., :8] ** 2 + z[..., 8:] ** 2
    assert np.allclose(pair_norm(y), pair_norm(x), rtol=1e-12)


def test_complex_multiplication_library_form():
    # the same map written with a library's complex arithmetic: (x1 + i x2) * exp(i a)
    rng = np.random.default_rng(1)
    N, H, d = 40, 2, 32
    x = rng.standard_normal((N, H, d))
    pos = rng.integers(0, 20000, size=N)
    inv_freq = torch.tensor(10000.0, dtype=torch.float64) ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.from_numpy(pos).to(torch.float64)[:, None] * inv_freq[None, :]
    z = torch.complex(torch.from_numpy(x[..., : d // 2]), torch.from_numpy(x[..., d // 2:]))
    zr = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    ref = torch.cat([zr.real, zr.imag], dim=-1).numpy()
    assert np.allclose(oracle.rope(x, pos), ref, rtol=1e-12, atol=1e-12)


def test_inverse_and_relative_position():
    rng = np.random.default_rng(2)
    N, H, d = 30, 2, 16
    q, k = rng.standard_normal((N, H, d)), rng.standard_normal((N, H, d))
    pos = rng.integers(0, 3000, size=N)
    assert np.allclose(oracle.rope(oracle.rope(q, pos), pos, inverse=True), q, atol=1e-12)
    # inverse is the transpose: <R x, y> == <x, R^T y>
    y = rng.standard_normal((N, H, d))
    assert np.allclose((oracle.rope(q, pos) * y).sum(), (q * oracle.rope(y, pos, inverse=True)).sum(), rtol=1e-12)
    # scores depend on the position difference only: shifting all positions changes nothing
    s0 = np.einsum("ihc,jhc->hij", oracle.rope(q, pos), oracle.rope(k, pos))
    s1 = np.einsum("ihc,jhc->hij", oracle.rope(q, pos + 977), oracle.rope(k, pos + 977))
    assert np.allclose(s0, s1, atol=1e-9)


def test_packed_example_is_encoded_as_if_alone():
    # ids restart at 0 in every example, so its rotary phases -- and its attention output -- are
    # those of the example processed on its own (what packing with position ids promises)
    w = wl.make_custom([[5, 9, 2]], hq=2, hkv=1, d=8, dtype="f32", seed=3)
    pos = w.position_ids
    seg = oracle.pack(pos)
    qr, kr = oracle.rope(w.q, pos), oracle.rope(w.k, pos)
    O, _ = oracle.fwd(qr, kr, w.v, seg["cu_seqlens"])
    a, b = 5, 14
    alone_pos = np.arange(9)
    Oa, _ = oracle.fwd(oracle.rope(w.q[a:b], alone_pos), oracle.rope(w.k[a:b], alone_pos), w.v[a:b],
                       np.array([0, 9], dtype=np.int32))
    assert np.array_equal(O[a:b], Oa)
    # without the restart (ids 0..15) the rotated tensors differ
    assert not np.allclose(oracle.rope(w.q, np.arange(16))[a:b], qr[a:b])
