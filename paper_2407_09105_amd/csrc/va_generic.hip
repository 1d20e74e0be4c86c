// Plain fp32-arithmetic kernels: any element type (fp32 / bf16 / fp16), any head_dim <= 256.
//
// They serve the fp32 path (where bf16 matrix cores cannot give the required accuracy) and
// head dims the MFMA kernels are not instantiated for.  One 64-lane wave per output row; the
// lanes split the head dimension; the mask is "seg_start[i] <= j <= i" (forward, dQ) or
// "j <= i < seg_end[j]" (dK/dV) -- Table 1's correct cross-attention for contiguous examples.
#include "va_internal.h"
#include "va_mfma_common.h"

namespace va {
namespace {

constexpr int kMaxPerLane = 4;  // head_dim <= 64 * 4

__device__ __forceinline__ float ld(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld(const uint16_t *p, size_t i) {
  return __uint_as_float(((uint32_t)p[i]) << 16);
}
__device__ __forceinline__ void st(float *p, size_t i, float x) { p[i] = x; }
__device__ __forceinline__ void st(uint16_t *p, size_t i, float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) { p[i] = (uint16_t)((u >> 16) | 0x40); return; }  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
  p[i] = (uint16_t)(u >> 16);
}

__device__ __forceinline__ float ld(const _Float16 *p, size_t i) { return (float)p[i]; }
__device__ __forceinline__ void st(_Float16 *p, size_t i, float x) { p[i] = (_Float16)x; }

__device__ __forceinline__ float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// One wave per (token i, head h).  grid.x = ceil(N * hq / waves_per_block).
template <typename T>
__global__ void __launch_bounds__(256)
generic_fwd_kernel(const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
                   T *__restrict__ O, float *__restrict__ LSE, const int32_t *__restrict__ seg_start,
                   int N, int hq, int hkv, int d, float scale) {
  const int lane = threadIdx.x & 63;
  const long long unit = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (unit >= (long long)N * hq) return;
  const int i = (int)(unit / hq), h = (int)(unit % hq), g = h / (hq / hkv);
  const int a = seg_start[i];
  float q[kMaxPerLane], o[kMaxPerLane];
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    const int c = lane + 64 * e;
    q[e] = c < d ? ld(Q, ((size_t)i * hq + h) * d + c) : 0.f;
    o[e] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  for (int j = a; j <= i; ++j) {
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
      const int c = lane + 64 * e;
      if (c < d) part += q[e] * ld(K, ((size_t)j * hkv + g) * d + c);
    }
    const float s = wave_sum(part) * scale;
    const float mn = fmaxf(m, s);
    const float alpha = __expf(m - mn), p = __expf(s - mn);
    l = l * alpha + p;
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
      const int c = lane + 64 * e;
      if (c < d) o[e] = o[e] * alpha + p * ld(V, ((size_t)j * hkv + g) * d + c);
    }
    m = mn;
  }
  const float inv = 1.f / l;
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    const int c = lane + 64 * e;
    if (c < d) st(O, ((size_t)i * hq + h) * d + c, o[e] * inv);
  }
  if (lane == 0) LSE[(size_t)h * N + i] = m + __logf(l);
}

// delta[h, i] = sum_c dO[i,h,c] * O[i,h,c]; one wave per (i, h)
template <typename T>
__global__ void __launch_bounds__(256)
delta_kernel(const T *__restrict__ dO, const T *__restrict__ O, float *__restrict__ delta, int N,
             int hq, int d) {
  const int lane = threadIdx.x & 63;
  const long long unit = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (unit >= (long long)N * hq) return;
  const int i = (int)(unit / hq), h = (int)(unit % hq);
  float part = 0.f;
  for (int c = lane; c < d; c += 64) {
    const size_t x = ((size_t)i * hq + h) * d + c;
    part += ld(dO, x) * ld(O, x);
  }
  part = wave_sum(part);
  if (lane == 0) delta[(size_t)h * N + i] = part;
}

// D for the 16-bit types with head_dim a multiple of 8 up to 128: 16 lanes per (token, head) row,
// 16 B of dO and of O per lane; a block handles 64 consecutive tokens of one head, so the [Hq, N]
// result is written 64 B at a time.
template <class E>
__global__ void __launch_bounds__(256)
delta_16bit_kernel(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ O,
                   float *__restrict__ delta, int N, int hq, int d) {
  const int h = blockIdx.y, c = threadIdx.x & 15, ti = threadIdx.x >> 4;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = blockIdx.x * 64 + it * 16 + ti;
    float part = 0.f;
    if (i < N && c * 8 < d) {
      const size_t x = ((size_t)i * hq + h) * d + c * 8;
      const typename E::x8 a = as_x8<E>(*(const u32x4 *)(dO + x)), b = as_x8<E>(*(const u32x4 *)(O + x));
#pragma unroll
      for (int e = 0; e < 8; ++e) part += (float)a[e] * (float)b[e];
    }
    for (int o = 8; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
    if (c == 0 && i < N) delta[(size_t)h * N + i] = part;
  }
}

// dQ: one wave per (i, h)
template <typename T, typename TG>
__global__ void __launch_bounds__(256)
generic_dq_kernel(const T *__restrict__ dO, const T *__restrict__ Q, const T *__restrict__ K,
                  const T *__restrict__ V, const float *__restrict__ LSE,
                  const float *__restrict__ delta, TG *__restrict__ dQ,
                  const int32_t *__restrict__ seg_start, int N, int hq, int hkv, int d, float scale) {
  const int lane = threadIdx.x & 63;
  const long long unit = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (unit >= (long long)N * hq) return;
  const int i = (int)(unit / hq), h = (int)(unit % hq), g = h / (hq / hkv);
  const int a = seg_start[i];
  float q[kMaxPerLane], go[kMaxPerLane], acc[kMaxPerLane];
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    const int c = lane + 64 * e;
    const size_t x = ((size_t)i * hq + h) * d + c;
    q[e] = c < d ? ld(Q, x) : 0.f;
    go[e] = c < d ? ld(dO, x) : 0.f;
    acc[e] = 0.f;
  }
  const float lse = LSE[(size_t)h * N + i], dl = delta[(size_t)h * N + i];
  for (int j = a; j <= i; ++j) {
    float ps = 0.f, pd = 0.f;
    float kk[kMaxPerLane];
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
      const int c = lane + 64 * e;
      const size_t x = ((size_t)j * hkv + g) * d + c;
      kk[e] = c < d ? ld(K, x) : 0.f;
      ps += q[e] * kk[e];
      pd += c < d ? go[e] * ld(V, x) : 0.f;
    }
    const float p = __expf(wave_sum(ps) * scale - lse);
    const float ds = p * (wave_sum(pd) - dl);
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) acc[e] += ds * kk[e];
  }
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    const int c = lane + 64 * e;
    if (c < d) st(dQ, ((size_t)i * hq + h) * d + c, acc[e] * scale);
  }
}

// dK, dV: one wave per (j, g); sums over the group's query heads and the later rows of the example
template <typename T, typename TG>
__global__ void __launch_bounds__(256)
generic_dkv_kernel(const T *__restrict__ dO, const T *__restrict__ Q, const T *__restrict__ K,
                   const T *__restrict__ V, const float *__restrict__ LSE,
                   const float *__restrict__ delta, TG *__restrict__ dK, TG *__restrict__ dV,
                   const int32_t *__restrict__ seg_end, int N, int hq, int hkv, int d, float scale) {
  const int lane = threadIdx.x & 63;
  const long long unit = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (unit >= (long long)N * hkv) return;
  const int j = (int)(unit / hkv), g = (int)(unit % hkv), G = hq / hkv;
  const int b = seg_end[j];
  float kk[kMaxPerLane], vv[kMaxPerLane], ak[kMaxPerLane], av[kMaxPerLane];
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    const int c = lane + 64 * e;
    const size_t x = ((size_t)j * hkv + g) * d + c;
    kk[e] = c < d ? ld(K, x) : 0.f;
    vv[e] = c < d ? ld(V, x) : 0.f;
    ak[e] = 0.f;
    av[e] = 0.f;
  }
  for (int h = g * G; h < (g + 1) * G; ++h) {
    for (int i = j; i < b; ++i) {
      float ps = 0.f, pd = 0.f, qq[kMaxPerLane], gg[kMaxPerLane];
#pragma unroll
      for (int e = 0; e < kMaxPerLane; ++e) {
        const int c = lane + 64 * e;
        const size_t x = ((size_t)i * hq + h) * d + c;
        qq[e] = c < d ? ld(Q, x) : 0.f;
        gg[e] = c < d ? ld(dO, x) : 0.f;
        ps += qq[e] * kk[e];
        pd += gg[e] * vv[e];
      }
      const float p = __expf(wave_sum(ps) * scale - LSE[(size_t)h * N + i]);
      const float ds = p * (wave_sum(pd) - delta[(size_t)h * N + i]);
#pragma unroll
      for (int e = 0; e < kMaxPerLane; ++e) {
        ak[e] += ds * qq[e];
        av[e] += p * gg[e];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    const int c = lane + 64 * e;
    if (c < d) {
      st(dK, ((size_t)j * hkv + g) * d + c, ak[e] * scale);
      st(dV, ((size_t)j * hkv + g) * d + c, av[e]);
    }
  }
}

inline unsigned blocks_for(long long units) { return (unsigned)((units + 3) / 4); }

}  // namespace

hipError_t launch_generic_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                              const va_segments &seg, int N, int hq, int hkv, int d, va_dtype dt,
                              float scale, hipStream_t stream) {
  const unsigned nb = blocks_for((long long)N * hq);
  if (dt == VA_F32)
    generic_fwd_kernel<float><<<nb, 256, 0, stream>>>((const float *)Q, (const float *)K, (const float *)V,
                                                      (float *)O, LSE, seg.seg_start, N, hq, hkv, d, scale);
  else if (dt == VA_F16)
    generic_fwd_kernel<_Float16><<<nb, 256, 0, stream>>>((const _Float16 *)Q, (const _Float16 *)K,
                                                         (const _Float16 *)V, (_Float16 *)O, LSE,
                                                         seg.seg_start, N, hq, hkv, d, scale);
  else
    generic_fwd_kernel<uint16_t><<<nb, 256, 0, stream>>>((const uint16_t *)Q, (const uint16_t *)K,
                                                         (const uint16_t *)V, (uint16_t *)O, LSE,
                                                         seg.seg_start, N, hq, hkv, d, scale);
  return hipGetLastError();
}

hipError_t launch_delta(const void *dO, const void *O, float *delta, int N, int hq, int d,
                        va_dtype dt, hipStream_t stream) {
  if (dt != VA_F32 && d <= 128 && d % 8 == 0) {
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)hq);
    if (dt == VA_F16)
      delta_16bit_kernel<F16><<<grid, 256, 0, stream>>>((const uint16_t *)dO, (const uint16_t *)O, delta, N, hq, d);
    else
      delta_16bit_kernel<Bf16><<<grid, 256, 0, stream>>>((const uint16_t *)dO, (const uint16_t *)O, delta, N, hq, d);
    return hipGetLastError();
  }
  const unsigned nb = blocks_for((long long)N * hq);
  if (dt == VA_F16)
    delta_kernel<_Float16><<<nb, 256, 0, stream>>>((const _Float16 *)dO, (const _Float16 *)O, delta, N, hq, d);
  else if (dt == VA_F32)
    delta_kernel<float><<<nb, 256, 0, stream>>>((const float *)dO, (const float *)O, delta, N, hq, d);
  else
    delta_kernel<uint16_t><<<nb, 256, 0, stream>>>((const uint16_t *)dO, (const uint16_t *)O, delta, N, hq, d);
  return hipGetLastError();
}

template <typename T, typename TG>
static void launch_bwd_t(const void *dO, const void *Q, const void *K, const void *V, const float *LSE,
                         const float *delta, void *dQ, void *dK, void *dV, const va_segments &seg,
                         int N, int hq, int hkv, int d, float scale, hipStream_t stream, unsigned stages) {
  if (stages & VA_STAGE_DQ)
  generic_dq_kernel<T, TG><<<blocks_for((long long)N * hq), 256, 0, stream>>>(
      (const T *)dO, (const T *)Q, (const T *)K, (const T *)V, LSE, delta, (TG *)dQ, seg.seg_start, N, hq,
      hkv, d, scale);
  if (stages & VA_STAGE_DKDV)
  generic_dkv_kernel<T, TG><<<blocks_for((long long)N * hkv), 256, 0, stream>>>(
      (const T *)dO, (const T *)Q, (const T *)K, (const T *)V, LSE, delta, (TG *)dK, (TG *)dV, seg.seg_end,
      N, hq, hkv, d, scale);
}

hipError_t launch_generic_bwd(const void *dO, const void *Q, const void *K, const void *V,
                              const float *LSE, const float *delta, void *dQ, void *dK, void *dV,
                              va_dtype grad_dt, const va_segments &seg, int N, int hq, int hkv,
                              int d, va_dtype dt, float scale, hipStream_t stream, unsigned stages) {
  if (dt == VA_F16 && grad_dt == VA_F32)
    launch_bwd_t<_Float16, float>(dO, Q, K, V, LSE, delta, dQ, dK, dV, seg, N, hq, hkv, d, scale, stream, stages);
  else if (dt == VA_F16)
    launch_bwd_t<_Float16, _Float16>(dO, Q, K, V, LSE, delta, dQ, dK, dV, seg, N, hq, hkv, d, scale, stream, stages);
  else if (dt == VA_F32 && grad_dt == VA_F32)
    launch_bwd_t<float, float>(dO, Q, K, V, LSE, delta, dQ, dK, dV, seg, N, hq, hkv, d, scale, stream, stages);
  else if (dt == VA_F32)
    launch_bwd_t<float, uint16_t>(dO, Q, K, V, LSE, delta, dQ, dK, dV, seg, N, hq, hkv, d, scale, stream, stages);
  else if (grad_dt == VA_F32)
    launch_bwd_t<uint16_t, float>(dO, Q, K, V, LSE, delta, dQ, dK, dV, seg, N, hq, hkv, d, scale, stream, stages);
  else
    launch_bwd_t<uint16_t, uint16_t>(dO, Q, K, V, LSE, delta, dQ, dK, dV, seg, N, hq, hkv, d, scale, stream, stages);
  return hipGetLastError();
}

}  // namespace va
