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

// A chunk of kVec consecutive elements of type T (float, __bf16 or _Float16), 16 bytes when wide.
template <typename T, int kVec> struct Chunk {
  typedef T type __attribute__((ext_vector_type(kVec)));
  static __device__ __forceinline__ float get(const type &v, int e) { return (float)v[e]; }
  static __device__ __forceinline__ void set(type &v, int e, float x) { v[e] = (T)x; }  // round to nearest even
};
template <typename T> struct Chunk<T, 1> {
  typedef T type;
  static __device__ __forceinline__ float get(const type &v, int) { return (float)v; }
  static __device__ __forceinline__ void set(type &v, int, float x) { v = (T)x; }
};

// One thread per (token, chunk of kVec pairs); it loops over the heads blockIdx.y, blockIdx.y +
// gridDim.y, ... (the heads are split over gridDim.y when the token count alone cannot fill the chip).
template <typename T, int kVec, typename IdT>
__global__ void __launch_bounds__(256)
rope_kernel(const T *x, T *y, const IdT *__restrict__ pos, long long n_work,  // y may be x (in place)
            int chunks_per_token, int H, int d, double neg2_log2base_over_d, int inverse) {
  typedef Chunk<T, kVec> C;
  typedef typename C::type chunk_t;
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
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
      const float x1 = C::get(a, e), x2 = C::get(b, e);
      C::set(ra, e, x1 * cs[e] - x2 * sn[e]);
      C::set(rb, e, x2 * cs[e] + x1 * sn[e]);
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
  if (dt == VA_BF16) return pick<__bf16, 8>(x, y, pos, it, N, H, d, base, inverse, stream);
  if (dt == VA_F16) return pick<_Float16, 8>(x, y, pos, it, N, H, d, base, inverse, stream);
  return pick<float, 4>(x, y, pos, it, N, H, d, base, inverse, stream);
}

}  // namespace va
