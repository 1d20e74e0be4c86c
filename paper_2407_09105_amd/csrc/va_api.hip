// C ABI of the library: argument validation and dispatch.  See include/varlen_attn.h.
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "va_internal.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct PlanLayout {
  size_t cu, seg_id, seg_start, seg_end, meta, q_order, kv_order, scratch, total;
};

bool plan_layout(int32_t rows, int32_t T, PlanLayout *L) {
  if (rows <= 0 || T <= 0) return false;
  const long long N = (long long)rows * T;
  if (N >= (1ll << 31) - 1) return false;
  const size_t n = (size_t)N;
  const size_t ntiles = (size_t)rows * (size_t)va::ceil_div(T, va::kTile);
  const size_t nchunks = (n + va::kScanChunk - 1) / va::kScanChunk;
  size_t off = 0;
  L->cu = off;        off += align_up((n + 1) * 4);
  L->seg_id = off;    off += align_up(n * 4);
  L->seg_start = off; off += align_up(n * 4);
  L->seg_end = off;   off += align_up(n * 4);
  L->meta = off;      off += align_up(8 * 4);
  L->q_order = off;   off += align_up(ntiles * 4);
  L->kv_order = off;  off += align_up(ntiles * 4);
  L->scratch = off;   off += align_up((8 * nchunks + 4 * ntiles) * 4);
  L->total = off;
  return true;
}

// The MFMA kernels take bf16 / fp16 tensors whose head_dim is a multiple of 8: the forward up to
// 256, the backward kernels up to kMfmaDqMaxD / kMfmaDkdvMaxD; everything else runs on the plain kernels.
constexpr int kMfmaFwdMaxD = 256, kMfmaDqMaxD = 256, kMfmaDkdvMaxD = 256;
bool use_mfma(va_dtype dt, int d, int max_d) {
  static const bool force_generic = [] {
    const char *e = std::getenv("VA_FORCE_GENERIC");
    return e && e[0] == '1';
  }();
  return (dt == VA_BF16 || dt == VA_F16) && d <= max_d && d % 8 == 0 && !force_generic;
}

va_status check_common(const va_segments *seg, int32_t rows, int32_t T, int32_t hq, int32_t hkv,
                       int32_t d, va_dtype dt) {
  if (!seg) return VA_ERR_NULL;
  if (!seg->cu_seqlens || !seg->seg_id || !seg->seg_start || !seg->seg_end || !seg->meta ||
      !seg->q_tile_order || !seg->kv_tile_order)
    return VA_ERR_NULL;
  if (rows <= 0 || T <= 0 || hq <= 0 || hkv <= 0 || d <= 0) return VA_ERR_SHAPE;
  if ((long long)rows * T >= (1ll << 31) - 1) return VA_ERR_SHAPE;
  if (hq % hkv != 0) return VA_ERR_SHAPE;
  if (dt != VA_F32 && dt != VA_BF16 && dt != VA_F16) return VA_ERR_UNSUPPORTED;
  if (d > 256) return VA_ERR_UNSUPPORTED;
  if (hq > 65535) return VA_ERR_UNSUPPORTED;  // a grid dimension of the D kernel
  // the MFMA kernels address one packed row's K/V (or Q/dO) through 32-bit byte offsets
  if (use_mfma(dt, d, kMfmaFwdMaxD) && ((long long)T + 256) * hq * d * 2 >= 0xffffff00ll) return VA_ERR_UNSUPPORTED;  // largest buffer size
  return VA_OK;
}

}  // namespace

extern "C" {

size_t va_plan_bytes(int32_t rows, int32_t tokens_per_row) {
  PlanLayout L;
  return plan_layout(rows, tokens_per_row, &L) ? L.total : 0;
}

va_status va_segments_bind(void *plan, size_t plan_bytes, int32_t rows, int32_t tokens_per_row,
                           va_segments *seg) {
  if (!plan || !seg) return VA_ERR_NULL;
  PlanLayout L;
  if (!plan_layout(rows, tokens_per_row, &L)) return VA_ERR_SHAPE;
  if (plan_bytes < L.total || ((uintptr_t)plan % kAlign) != 0) return VA_ERR_WORKSPACE;
  char *p = (char *)plan;
  seg->cu_seqlens = (int32_t *)(p + L.cu);
  seg->seg_id = (int32_t *)(p + L.seg_id);
  seg->seg_start = (int32_t *)(p + L.seg_start);
  seg->seg_end = (int32_t *)(p + L.seg_end);
  seg->meta = (int32_t *)(p + L.meta);
  seg->q_tile_order = (int32_t *)(p + L.q_order);
  seg->kv_tile_order = (int32_t *)(p + L.kv_order);
  seg->scratch = (int32_t *)(p + L.scratch);
  return VA_OK;
}

va_status va_pack_to_cu_seqlens(const void *position_ids, va_itype it, int32_t rows,
                                int32_t tokens_per_row, const va_segments *seg, void *stream) {
  if (!position_ids || !seg) return VA_ERR_NULL;
  if (!seg->cu_seqlens || !seg->seg_id || !seg->seg_start || !seg->seg_end || !seg->meta ||
      !seg->q_tile_order || !seg->kv_tile_order || !seg->scratch)
    return VA_ERR_NULL;
  if (rows <= 0 || tokens_per_row <= 0) return VA_ERR_SHAPE;
  if ((long long)rows * tokens_per_row >= (1ll << 31) - 1) return VA_ERR_SHAPE;
  if (it != VA_I32 && it != VA_I64) return VA_ERR_UNSUPPORTED;
  hipError_t e = va::launch_pack(position_ids, it, rows, tokens_per_row, *seg, (hipStream_t)stream);
  return e == hipSuccess ? VA_OK : VA_ERR_HIP;
}

va_status va_collate_padding_free(const void *ids_padded, const void *labels_padded, va_itype it,
                                  const int32_t *lengths, int32_t n_examples, int32_t padded_len,
                                  int32_t n_out, int64_t pad_id, void *input_ids, void *labels,
                                  void *position_ids, int32_t *example_offsets, void *stream) {
  if (n_examples < 0 || padded_len <= 0 || n_out < 0) return VA_ERR_SHAPE;
  if ((long long)n_examples * padded_len >= (1ll << 31) - 1) return VA_ERR_SHAPE;
  if (it != VA_I32 && it != VA_I64) return VA_ERR_UNSUPPORTED;
  if (!example_offsets) return VA_ERR_NULL;
  if (n_examples > 0 && (!ids_padded || !lengths)) return VA_ERR_NULL;
  if (n_out > 0 && (!input_ids || !labels || !position_ids)) return VA_ERR_NULL;
  hipError_t e = va::launch_collate(ids_padded, labels_padded, it, lengths, n_examples, padded_len, n_out,
                                    (long long)pad_id, input_ids, labels, position_ids, example_offsets,
                                    (hipStream_t)stream);
  return e == hipSuccess ? VA_OK : VA_ERR_HIP;
}

va_status va_rope_apply(const void *x, void *y, va_dtype dt, const void *position_ids, va_itype it,
                        int32_t n_tokens, int32_t heads, int32_t d, float theta_base, int inverse,
                        void *stream) {
  if (n_tokens < 0 || heads <= 0 || d <= 0 || (d & 1)) return VA_ERR_SHAPE;
  if (dt != VA_F32 && dt != VA_BF16 && dt != VA_F16) return VA_ERR_UNSUPPORTED;
  if (it != VA_I32 && it != VA_I64) return VA_ERR_UNSUPPORTED;
  if (d > 256) return VA_ERR_UNSUPPORTED;
  if (n_tokens > 0 && (!x || !y || !position_ids)) return VA_ERR_NULL;
  const double base = theta_base > 0.f ? (double)theta_base : 10000.0;
  hipError_t e = va::launch_rope(x, y, dt, position_ids, it, n_tokens, heads, d, base, inverse != 0,
                                 (hipStream_t)stream);
  return e == hipSuccess ? VA_OK : VA_ERR_HIP;
}

size_t va_attn_workspace_bytes(int32_t n_tokens, int32_t hq, int32_t hkv, int32_t d, int is_bwd) {
  if (n_tokens <= 0 || hq <= 0 || hkv <= 0 || d <= 0) return 0;
  if (!is_bwd) return 0;
  return align_up((size_t)n_tokens * (size_t)hq * sizeof(float));  // D = rowsum(dO * O), [Hq, N]
}

va_status va_varlen_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                             const va_segments *seg, int32_t rows, int32_t tokens_per_row,
                             int32_t hq, int32_t hkv, int32_t d, va_dtype dt, float softmax_scale,
                             void *workspace, size_t workspace_bytes, void *stream) {
  (void)workspace;
  (void)workspace_bytes;
  if (!Q || !K || !V || !O || !LSE) return VA_ERR_NULL;
  va_status s = check_common(seg, rows, tokens_per_row, hq, hkv, d, dt);
  if (s != VA_OK) return s;
  const int N = rows * tokens_per_row;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
  hipError_t e;
  if (use_mfma(dt, d, kMfmaFwdMaxD))
    e = va::launch_mfma_fwd(Q, K, V, O, LSE, *seg, rows, tokens_per_row, hq, hkv, d, dt, scale, (hipStream_t)stream);
  else
    e = va::launch_generic_fwd(Q, K, V, O, LSE, *seg, N, hq, hkv, d, dt, scale, (hipStream_t)stream);
  return e == hipSuccess ? VA_OK : VA_ERR_HIP;
}

namespace {
// Host-side validation of a backward call: everything except the workspace.
va_status check_bwd(const void *dO, const void *Q, const void *K, const void *V, const void *O, const float *LSE,
                    void *dQ, void *dK, void *dV, va_dtype grad_dt, const va_segments *seg, int32_t rows,
                    int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d, va_dtype dt, uint32_t stages) {
  if (!dO || !Q || !K || !V || !O || !LSE || !dQ || !dK || !dV) return VA_ERR_NULL;
  va_status s = check_common(seg, rows, tokens_per_row, hq, hkv, d, dt);
  if (s != VA_OK) return s;
  // gradients come out in fp32 or in the inputs' own 16-bit type (fp32 inputs: fp32 or bf16)
  if (grad_dt != VA_F32 && !(grad_dt == VA_BF16 && dt != VA_F16) && !(grad_dt == VA_F16 && dt == VA_F16))
    return VA_ERR_UNSUPPORTED;
  constexpr uint32_t kStages = VA_STAGE_D | VA_STAGE_DKDV | VA_STAGE_DQ;
  constexpr uint32_t kHints = VA_HINT_LONG_EXAMPLES | VA_HINT_SHORT_EXAMPLES;
  if ((stages & kStages) == 0 || (stages & ~(kStages | kHints)) || (stages & kHints) == kHints) return VA_ERR_UNSUPPORTED;
  return VA_OK;
}
}  // namespace

va_status va_varlen_attn_bwd_stages(const void *dO, const void *Q, const void *K, const void *V,
                                    const void *O, const float *LSE, void *dQ, void *dK, void *dV,
                                    va_dtype grad_dt, const va_segments *seg, int32_t rows,
                                    int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d,
                                    va_dtype dt, float softmax_scale, void *workspace,
                                    size_t workspace_bytes, void *stream, uint32_t stages) {
  va_status s = check_bwd(dO, Q, K, V, O, LSE, dQ, dK, dV, grad_dt, seg, rows, tokens_per_row, hq, hkv, d, dt, stages);
  if (s != VA_OK) return s;
  const int N = rows * tokens_per_row;
  const size_t need = va_attn_workspace_bytes(N, hq, hkv, d, 1);
  if (!workspace) return VA_ERR_NULL;
  if (workspace_bytes < need) return VA_ERR_WORKSPACE;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
  float *delta = (float *)workspace;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipSuccess;
  const unsigned hints = stages & (VA_HINT_LONG_EXAMPLES | VA_HINT_SHORT_EXAMPLES);
  const unsigned mfma_stages = ((use_mfma(dt, d, kMfmaDqMaxD) ? VA_STAGE_DQ : 0u) |
                                (use_mfma(dt, d, kMfmaDkdvMaxD) ? VA_STAGE_DKDV : 0u)) & stages;
  const unsigned plain_stages = stages & (VA_STAGE_DKDV | VA_STAGE_DQ) & ~mfma_stages;
  // the MFMA dQ kernel forms D itself (and stores it for the dK/dV kernel, which it precedes)
  if ((stages & VA_STAGE_D) && !(mfma_stages & VA_STAGE_DQ)) e = va::launch_delta(dO, O, delta, N, hq, d, dt, st);
  if (e != hipSuccess) return VA_ERR_HIP;
  if (mfma_stages)
    e = va::launch_mfma_bwd(dO, Q, K, V, O, LSE, delta, dQ, dK, dV, grad_dt, *seg, rows, tokens_per_row, hq, hkv,
                            d, dt, scale, st, mfma_stages | hints);
  if (e != hipSuccess) return VA_ERR_HIP;
  if (plain_stages)
    e = va::launch_generic_bwd(dO, Q, K, V, LSE, delta, dQ, dK, dV, grad_dt, *seg, N, hq, hkv, d, dt, scale, st,
                               plain_stages);
  return e == hipSuccess ? VA_OK : VA_ERR_HIP;
}

va_status va_varlen_attn_bwd(const void *dO, const void *Q, const void *K, const void *V,
                             const void *O, const float *LSE, void *dQ, void *dK, void *dV,
                             va_dtype grad_dt, const va_segments *seg, int32_t rows,
                             int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d,
                             va_dtype dt, float softmax_scale, void *workspace,
                             size_t workspace_bytes, void *stream) {
  return va_varlen_attn_bwd_stages(dO, Q, K, V, O, LSE, dQ, dK, dV, grad_dt, seg, rows, tokens_per_row, hq,
                                   hkv, d, dt, softmax_scale, workspace, workspace_bytes, stream,
                                   VA_STAGE_D | VA_STAGE_DKDV | VA_STAGE_DQ);
}

// ---- the backward for callers that cannot allocate ------------------------------------------
// Its workspace (D = rowsum(dO * O), [Hq, N] float) is this file-scope device array instead of a
// caller's buffer.  Every GPU holds its own copy at its own address: the address is looked up once
// per device (hipGetSymbolAddress with that device current) and only that pointer is ever handed to
// a kernel - the array's name is a host-side stand-in, not a device address.
static __device__ __align__(256) unsigned char scratch[VA_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // per device: address of `scratch` there, once looked up

// Address of this device's copy of `scratch` (nullptr on error).
void *scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

va_status va_varlen_attn_bwd_noalloc(const void *dO, const void *Q, const void *K, const void *V,
                                     const void *O, const float *LSE, void *dQ, void *dK, void *dV,
                                     va_dtype grad_dt, const va_segments *seg, int32_t rows,
                                     int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d,
                                     va_dtype dt, float softmax_scale, void *stream) {
  const va_status s = check_bwd(dO, Q, K, V, O, LSE, dQ, dK, dV, grad_dt, seg, rows, tokens_per_row, hq, hkv, d, dt,
                                 VA_STAGE_D | VA_STAGE_DKDV | VA_STAGE_DQ);
  if (s != VA_OK) return s;  // before anything touches the GPU
  const size_t need = va_attn_workspace_bytes(rows * tokens_per_row, hq, hkv, d, 1);
  if (need == 0 || need > (size_t)VA_NOALLOC_SCRATCH_BYTES) return VA_ERR_WORKSPACE;  // beyond the static array
  void *ws = scratch_on_current_device();
  if (!ws) return VA_ERR_HIP;
  // every byte of D that the dK/dV kernel reads is written by the dQ (or D) kernel of the same call,
  // so nothing of the previous call's contents has to be cleared
  return va_varlen_attn_bwd(dO, Q, K, V, O, LSE, dQ, dK, dV, grad_dt, seg, rows, tokens_per_row, hq, hkv, d, dt,
                            softmax_scale, ws, (size_t)VA_NOALLOC_SCRATCH_BYTES, stream);
}

const char *va_status_string(va_status s) {
  switch (s) {
    case VA_OK: return "ok";
    case VA_ERR_NULL: return "null pointer";
    case VA_ERR_SHAPE: return "bad shape";
    case VA_ERR_UNSUPPORTED: return "unsupported dtype or head_dim";
    case VA_ERR_WORKSPACE: return "plan buffer or workspace too small or misaligned";
    case VA_ERR_HIP: return "HIP launch error";
  }
  return "unknown status";
}

const char *va_version(void) { return "varlen_attn 0.1 (gfx950)"; }


}  // extern "C"
