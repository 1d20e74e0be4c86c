// Measurement aid: a loop of nothing but v_mfma_f32_32x32x16_bf16 on every SIMD of the chip.
// Timed by the caller, it gives the matrix throughput this GPU actually sustains, to put next to
// the published peak that the roofline fractions are quoted against.
#include "va_internal.h"
#include "va_mfma_common.h"

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

}  // namespace

hipError_t launch_mfma_probe(float *sink, int iters, double *flops, hipStream_t stream) {
  mfma_probe_kernel<<<kProbeWgs, 256, 0, stream>>>(sink, iters);
  if (flops) *flops = (double)kProbeWgs * 4.0 * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
  return hipGetLastError();
}

}  // namespace va
