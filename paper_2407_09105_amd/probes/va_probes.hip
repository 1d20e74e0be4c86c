// Measurement aids of the benchmark (libva_probes.so; no part of the attention library): what the
// matrix pipe of this GPU sustains alone and in the company it keeps in the attention kernels.
// First kernel: a loop of nothing but v_mfma_f32_32x32x16_bf16 on every SIMD of the chip.  Timed by
// the caller, it gives the matrix throughput this GPU actually sustains, to put next to the
// published peak that the roofline fractions are quoted against.
#include <hip/hip_runtime.h>

#include "va_probes.h"
#include "../csrc/va_mfma_common.h"

namespace va {
namespace {

constexpr int kProbeWgs = 256 * 8;  // 256 compute units, 2 waves per SIMD
constexpr int kMfmaPerIter = 16;

__global__ void __launch_bounds__(256)
mfma_probe_kernel(float *__restrict__ sink, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((threadIdx.x + e) & 7); b[e] = (__bf16)(float)(e & 3); }
  f32x16 c[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[n][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kMfmaPerIter / 4; ++u)
#pragma unroll
      for (int n = 0; n < 4; ++n) c[n] = mfma32(a, b, c[n]);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c[n][v];
  if (s == 12345.678f) sink[threadIdx.x & 63] = s;  // keeps the loop alive; practically never taken
}

// The same matrix instructions with the company they keep in the attention kernels: operands with
// realistic bit patterns (the caller's 64 KB of 16-bit values, staged in LDS), kLds fragment reads
// (1 KB each, the kernels' swizzled row pattern) and kValu groups of {fma, exp2, max, add} per 16
// matrix instructions, all independent of each other so that nothing but issue slots, LDS bandwidth
// and the power limit holds the matrix pipe back.  It bounds what a kernel with that instruction
// mix can reach on this GPU.  Lane 0 of workgroup 0 leaves the shader-clock and wall-clock (100 MHz)
// ticks the loop took in clocks[0..1].
template <int kLds, int kValu>
__global__ void __launch_bounds__(256)
mix_probe_kernel(const uint32_t *__restrict__ operands, float *__restrict__ sink,
                 unsigned long long *__restrict__ clocks, int iters) {
  __shared__ __attribute__((aligned(16))) uint32_t lds[16384];  // 64 KB
  for (int i = threadIdx.x; i < 16384; i += 256) lds[i] = operands[i];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const uint32_t lane_off = swz_row_lane_off(lane);
  bf16x8 a[8], b[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    a[k] = as_x8<Bf16>(*(const u32x4 *)((const char *)lds + ((lane_off ^ (uint32_t)(k << 5)) + 8192u)));
    b[k] = as_x8<Bf16>(*(const u32x4 *)((const char *)lds + ((lane_off ^ (uint32_t)(k << 5)) + 16384u)));
  }
  f32x16 c[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[n][v] = 0.f;
  float x[16], mx = 0.f, sm = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = 0.01f * (float)(lane + e);
  const unsigned long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    const uint32_t blk = (uint32_t)(it & 3) * 8192u;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const uint32_t off = (lane_off ^ (uint32_t)(k << 5)) + blk + (uint32_t)u * 32768u;
        if (kLds == 16 || (kLds == 8 && (k & 1) == 0)) a[k] = as_x8<Bf16>(*(const u32x4 *)((const char *)lds + off));
        c[k & 3] = mfma32(kLds == 8 ? a[k & ~1] : a[k], b[k], c[k & 3]);
      }
    }
#pragma unroll
    for (int e = 0; e < kValu; ++e) {
      float &r = x[e & 15];
      const float p = __builtin_amdgcn_exp2f(fmaf(r, -0.5f, 0.25f));
      mx = fmaxf(mx, p);
      sm += p;
      r = p;
    }
  }
  const unsigned long long t1 = clock64(), w1 = wall_clock64();
  float s = mx + sm;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c[n][v];
#pragma unroll
  for (int e = 0; e < 16; ++e) s += x[e];
  if (s == 12345.678f) sink[threadIdx.x & 63] = s;  // keeps the loop alive; practically never taken
  if (clocks && threadIdx.x == 0 && blockIdx.x == 0) { clocks[0] = t1 - t0; clocks[1] = w1 - w0; }
}

}  // namespace

static hipError_t launch_mix_probe(const void *operands, int lds_reads, int valu_groups, float *sink,
                                   unsigned long long *clocks, int iters, double *flops, hipStream_t stream) {
  const uint32_t *op = (const uint32_t *)operands;
#define VA_MIX(L, V) mix_probe_kernel<L, V><<<kProbeWgs, 256, 0, stream>>>(op, sink, clocks, iters)
  if (lds_reads == 0 && valu_groups == 0) VA_MIX(0, 0);
  else if (lds_reads == 16 && valu_groups == 0) VA_MIX(16, 0);
  else if (lds_reads == 8 && valu_groups == 0) VA_MIX(8, 0);
  else if (lds_reads == 16 && valu_groups == 24) VA_MIX(16, 24);
  else if (lds_reads == 16 && valu_groups == 12) VA_MIX(16, 12);
  else if (lds_reads == 8 && valu_groups == 16) VA_MIX(8, 16);
  else return hipErrorInvalidValue;
#undef VA_MIX
  if (flops) *flops = (double)kProbeWgs * 4.0 * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
  return hipGetLastError();
}

static hipError_t launch_mfma_probe(float *sink, int iters, double *flops, hipStream_t stream) {
  mfma_probe_kernel<<<kProbeWgs, 256, 0, stream>>>(sink, iters);
  if (flops) *flops = (double)kProbeWgs * 4.0 * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
  return hipGetLastError();
}

}  // namespace va

extern "C" {

int vap_probe_mfma(float *sink, int32_t iters, double *flops, void *stream) {
  if (!sink) return VAP_ERR_NULL;
  if (iters <= 0 || iters > (1 << 24)) return VAP_ERR_ARG;
  return va::launch_mfma_probe(sink, iters, flops, (hipStream_t)stream) == hipSuccess ? VAP_OK : VAP_ERR_HIP;
}

int vap_probe_mix(const void *operands, int32_t lds_reads, int32_t valu_groups, float *sink, uint64_t *clocks,
                  int32_t iters, double *flops, void *stream) {
  if (!operands || !sink) return VAP_ERR_NULL;
  if (iters <= 0 || iters > (1 << 24)) return VAP_ERR_ARG;
  const bool known = (valu_groups == 0 && (lds_reads == 0 || lds_reads == 8 || lds_reads == 16)) ||
                     (lds_reads == 16 && (valu_groups == 24 || valu_groups == 12)) ||
                     (lds_reads == 8 && valu_groups == 16);
  if (!known) return VAP_ERR_UNSUPPORTED;
  return va::launch_mix_probe(operands, lds_reads, valu_groups, sink, (unsigned long long *)clocks, iters, flops,
                              (hipStream_t)stream) == hipSuccess ? VAP_OK : VAP_ERR_HIP;
}

}  // extern "C"
