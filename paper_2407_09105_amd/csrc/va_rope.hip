// Rotary position embedding driven by the packed stream's position ids (paper, Section 3: a
// model that takes position ids encodes a packed example exactly as if it were alone, because
// the ids restart at 0).  "Rotate-half" pairing: pair c = (x[c], x[c + d/2]) of a head vector
// turns by the angle pos * base^(-2c/d); `inverse` turns by the negative angle (the transpose,
// used for gradients).  HBM-bound: every element is read and written once; the sines and
// cosines of a (token, pair) are computed once and shared by all heads.
#include "va_internal.h"
#include "va_mfma_common.h"

namespace va {
namespace {

template <typename T, int kVec> struct Chunk;
template <> struct Chunk<float, 4> { typedef f32x4 type; };
template <> struct Chunk<float, 1> { typedef float type; };
template <> struct Chunk<uint16_t, 8> { typedef u32x4 type; };
template <> struct Chunk<uint16_t, 1> { typedef uint16_t type; };

__device__ __forceinline__ float elem(const f32x4 &v, int e) { return v[e]; }
__device__ __forceinline__ float elem(const float &v, int) { return v; }
__device__ __forceinline__ float elem(const uint16_t &v, int) { return bf16_to_f32(v); }
__device__ __forceinline__ float elem(const u32x4 &v, int e) {
  const uint32_t w = v[e >> 1];
  return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
}
__device__ __forceinline__ void put(f32x4 &v, int e, float lo, float) { v[e] = lo; }
__device__ __forceinline__ void put(float &v, int, float lo, float) { v = lo; }
__device__ __forceinline__ void put(uint16_t &v, int, float lo, float) { v = (uint16_t)(pack2_bf16(lo, 0.f) & 0xffffu); }
__device__ __forceinline__ void put(u32x4 &v, int e, float lo, float hi) { v[e >> 1] = pack2_bf16(lo, hi); }

// One thread per (token, chunk of kVec pairs); it loops over the heads blockIdx.y, blockIdx.y +
// gridDim.y, ... (the heads are split over gridDim.y when the token count alone cannot fill the chip).
template <typename T, int kVec, typename IdT>
__global__ void __launch_bounds__(256)
rope_kernel(const T *__restrict__ x, T *__restrict__ y, const IdT *__restrict__ pos, long long n_work,
            int chunks_per_token, int H, int d, double neg2_log2base_over_d, int inverse) {
  typedef typename Chunk<T, kVec>::type chunk_t;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n_work) return;
  const long long t = idx / chunks_per_token;
  const int ch = (int)(idx % chunks_per_token);
  const double p = (double)pos[t];
  float cs[kVec], sn[kVec];
#pragma unroll
  for (int e = 0; e < kVec; ++e) {
    const int c = ch * kVec + e;
    // angle in fp64, reduced to [-pi, pi] before the fp32 sine / cosine: exact to ~1e-7 at any position
    double a = p * exp2((double)c * neg2_log2base_over_d);
    a -= 6.283185307179586476925 * rint(a * 0.15915494309189533577);
    sincosf((float)a, &sn[e], &cs[e]);
    if (inverse) sn[e] = -sn[e];
  }
  const int hd = d / 2;
  const int hstep = gridDim.y;
  const T *xp = x + ((size_t)t * H + blockIdx.y) * d + ch * kVec;
  T *yp = y + ((size_t)t * H + blockIdx.y) * d + ch * kVec;
  for (int h = blockIdx.y; h < H; h += hstep, xp += (size_t)hstep * d, yp += (size_t)hstep * d) {
    const chunk_t a = *(const chunk_t *)xp, b = *(const chunk_t *)(xp + hd);
    chunk_t ra, rb;
    constexpr int kStep = (sizeof(T) == 2 && kVec > 1) ? 2 : 1;  // bf16 chunks are written as pairs
#pragma unroll
    for (int e = 0; e < kVec; e += kStep) {
      float o1[2], o2[2];
#pragma unroll
      for (int u = 0; u < kStep; ++u) {
        const float x1 = elem(a, e + u), x2 = elem(b, e + u);
        o1[u] = x1 * cs[e + u] - x2 * sn[e + u];
        o2[u] = x2 * cs[e + u] + x1 * sn[e + u];
      }
      put(ra, e, o1[0], o1[kStep - 1]);
      put(rb, e, o2[0], o2[kStep - 1]);
    }
    *(chunk_t *)yp = ra;
    *(chunk_t *)(yp + hd) = rb;
  }
}

template <typename T, int kVec, typename IdT>
hipError_t launch(const void *x, void *y, const void *pos, long long N, int H, int d, double base,
                  int inverse, hipStream_t stream) {
  const int cpt = d / 2 / kVec;
  const long long n_work = N * cpt;
  const long long grid = (n_work + 255) / 256;
  if (grid > 0x7fffffffll) return hipErrorInvalidValue;
  if (grid == 0) return hipSuccess;
  int hsplit = 1;  // aim at >= 4096 workgroups
  while (hsplit < H && grid * hsplit < 4096 && hsplit < 16) hsplit *= 2;
  if (hsplit > H) hsplit = H;
  rope_kernel<T, kVec, IdT><<<dim3((unsigned)grid, (unsigned)hsplit), 256, 0, stream>>>(
      (const T *)x, (T *)y, (const IdT *)pos, n_work, cpt, H, d, -2.0 * log2(base) / (double)d, inverse);
  return hipGetLastError();
}

template <typename T, int kWide>
hipError_t pick(const void *x, void *y, const void *pos, va_itype it, long long N, int H, int d,
                double base, int inverse, hipStream_t stream) {
  // 16-byte chunks need both halves of every head vector 16-byte aligned
  const bool wide = (d / 2) % kWide == 0 && (((uintptr_t)x | (uintptr_t)y) & 15) == 0;
  if (it == VA_I64)
    return wide ? launch<T, kWide, int64_t>(x, y, pos, N, H, d, base, inverse, stream)
                : launch<T, 1, int64_t>(x, y, pos, N, H, d, base, inverse, stream);
  return wide ? launch<T, kWide, int32_t>(x, y, pos, N, H, d, base, inverse, stream)
              : launch<T, 1, int32_t>(x, y, pos, N, H, d, base, inverse, stream);
}

}  // namespace

hipError_t launch_rope(const void *x, void *y, va_dtype dt, const void *pos, va_itype it, long long N,
                       int H, int d, double base, int inverse, hipStream_t stream) {
  if (dt == VA_BF16) return pick<uint16_t, 8>(x, y, pos, it, N, H, d, base, inverse, stream);
  return pick<float, 4>(x, y, pos, it, N, H, d, base, inverse, stream);
}

}  // namespace va
