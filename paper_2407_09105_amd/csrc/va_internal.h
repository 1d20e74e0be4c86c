// Internal declarations shared by the HIP sources of the library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "varlen_attn.h"

namespace va {

constexpr int kTile = VA_TILE;       // tokens per schedule tile
constexpr int kScanChunk = 2048;     // tokens per workgroup in the boundary scan
constexpr int kScanThreads = 256;

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// va_scan.hip
hipError_t launch_pack(const void *pos, va_itype it, int rows, int T, const va_segments &seg,
                       hipStream_t stream);

// va_collate.hip
hipError_t launch_collate(const void *ids, const void *labels_in, va_itype it, const int32_t *lengths,
                          int n, int Lp, int n_out, long long pad_id, void *input_ids, void *labels,
                          void *position_ids, int32_t *offsets, hipStream_t stream);

// va_rope.hip
hipError_t launch_rope(const void *x, void *y, va_dtype dt, const void *pos, va_itype it, long long N,
                       int H, int d, double base, int inverse, hipStream_t stream);

// va_generic.hip : plain fp32-arithmetic kernels, any head_dim <= 256
hipError_t launch_generic_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                              const va_segments &seg, int N, int hq, int hkv, int d, va_dtype dt,
                              float scale, hipStream_t stream);
hipError_t launch_delta(const void *dO, const void *O, float *delta, int N, int hq, int d,
                        va_dtype dt, hipStream_t stream);
hipError_t launch_generic_bwd(const void *dO, const void *Q, const void *K, const void *V,
                              const float *LSE, const float *delta, void *dQ, void *dK, void *dV,
                              va_dtype grad_dt, const va_segments &seg, int N, int hq, int hkv,
                              int d, va_dtype dt, float scale, hipStream_t stream, unsigned stages);

// va_fwd_mfma.hip / va_bwd_mfma.hip : bf16 / fp16, head_dim a multiple of 8 up to 256
hipError_t launch_mfma_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                           const va_segments &seg, int rows, int T, int hq, int hkv, int d, va_dtype dt,
                           float scale, hipStream_t stream);
hipError_t launch_mfma_bwd(const void *dO, const void *Q, const void *K, const void *V, const void *O,
                           const float *LSE, float *delta, void *dQ, void *dK, void *dV,
                           va_dtype grad_dt, const va_segments &seg, int rows, int T, int hq,
                           int hkv, int d, va_dtype dt, float scale, hipStream_t stream, unsigned stages);

}  // namespace va
