// Shared device helpers of the MFMA kernels (bf16 / fp16, head_dim <= 256, gfx950).
//
// Matrix-core tile used throughout: v_mfma_f32_32x32x16_{bf16,f16}, D[32x32] += A[32x16] * B[16x32].
// Register layout per 64-lane wave (lane l, half = l / 32):
//   A : lane holds row  l % 32, k = 8 * half .. 8 * half + 7   (8 bf16, contiguous in k)
//   B : lane holds col  l % 32, k = 8 * half .. 8 * half + 7
//   D : lane holds col  l % 32, 16 floats v = 0..15 at row 8 * (v / 4) + 4 * half + v % 4
// All kernels keep the workgroup-resident index (query row in the forward and dQ kernels,
// key row in the dK/dV kernel) on the lane/column axis, so that per-row softmax statistics
// are per-lane scalars and the streamed index sits on the register axis, where it can feed
// the next contraction as a B operand without leaving registers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace va {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// LDS rows of a streamed block always hold 128 elements (256 B); a kernel instantiated for a
// padded head_dim kDh (64, 96 or 128) uses the first kDh of them, and a tensor whose head_dim d is
// smaller than kDh contributes zeros for the columns d..kDh-1 (they add nothing to any product).
constexpr int kD = 128;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// The two 16-bit element types: 8-element operand vector, conversions (round to nearest even).
struct Bf16 {
  typedef bf16x8 x8;
  typedef __bf16 elem;
};
struct F16 {
  typedef f16x8 x8;
  typedef _Float16 elem;
};
template <class E> __device__ __forceinline__ typename E::x8 as_x8(u32x4 x) {
  return __builtin_bit_cast(typename E::x8, x);
}

// Row (register axis) index of accumulator element v for a lane of the given half.
__device__ __forceinline__ int acc_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// Eight consecutive accumulator floats v0..v0+7 -> one B operand (8 bf16).  With the layout
// above these are rows {8a + 4 half + b : a in {2s2, 2s2+1}, b in 0..3} of a 16-row k-step.
template <class E> __device__ __forceinline__ typename E::x8 pack_x8(const f32x16 &x, int v0) {
  typename E::x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (typename E::elem)x[v0 + e];
  return r;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

template <class E> __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  typedef typename E::elem x2 __attribute__((ext_vector_type(2)));
  x2 r;
  r.x = (typename E::elem)lo;
  r.y = (typename E::elem)hi;
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) { return pack2<Bf16>(lo, hi); }

// Transposing LDS read (ds_read_b64_tr_b16).  Within each block of 16 lanes, lane 4r + q supplies
// the address of 4 consecutive bf16 M[r][4q..4q+3] of a 4 x 16 matrix; lane i of the block receives
// the column M[0..3][i].  With a row-major [rows][cols] LDS block this hands lane (c = lane % 32,
// half = lane / 32) the elements X[j0 + 4 half + 0..3][c0 + c] -- four consecutive rows of one
// column -- which is exactly what an A operand "rows = columns of X, k = rows of X" needs.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// s_waitcnt vmcnt(0), visible to the compiler's wait-count bookkeeping (expcnt and lgkmcnt fields
// left at their maxima: 7 << 4, 15 << 8).
__device__ __forceinline__ void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by workgroup id.  With
// grouped-query attention the G query heads of one KV head stream the same K/V blocks; this maps
// workgroup id -> logical index so that G consecutive logical indices (the heads of one group, which
// are adjacent in the logical order) land on one XCD in consecutive slots, while the logical
// (longest-first) order is otherwise preserved at a granularity of 8 G workgroups.
__device__ __forceinline__ int xcd_group_remap(int wg, int G, int n_wg) {
  if (G == 1 || n_wg % (8 * G) != 0) return wg;
  const int xcd = wg & 7, slot = wg >> 3;
  return ((slot / G) * 8 + xcd) * G + slot % G;
}

// A tile-order entry of the pack: tile index in bits 0..23, head rotation of the tile above.
// Workgroup w runs on XCD w % 8, and the workgroups of one schedule tile are numbered head by head;
// the heads (KV-head groups) of the tile are rotated by this amount, which is the same for all tiles of
// one long example (each head's K/V or Q/dO stream then stays in one XCD's L2) and advances with the
// launch order among tiles of short examples (every XCD meets every head and with it every memory
// channel): the boundary scan decides, see order_entry there.
__device__ __forceinline__ int order_tile(int entry) { return entry & 0xffffff; }
__device__ __forceinline__ int head_rotation(int entry) { return (entry >> 24) & 127; }

// Wave-uniform value -> scalar register, so that conditions on it compile to scalar branches.
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// max / sum of a lane's value with that of lane ^ 32 (the lane holding the other keys of the
// same row): v_permlane32_swap hands every lane both halves.
__device__ __forceinline__ float pair_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float pair_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);
}

// Untyped buffer descriptor over `bytes` bytes at `base`: loads through it take a 32-bit byte
// offset and return zero beyond the end, so block loads need no per-lane bounds branches.  The
// whole offset goes into the per-lane (vector) operand: only that operand is range-checked, a
// scalar offset is added after the check and can reach past the end of the tensor.
typedef __amdgpu_buffer_rsrc_t buffer_t;
constexpr uint32_t kPastEnd = 0xfffffff0u;  // an offset no buffer made by make_buffer contains
__device__ __forceinline__ buffer_t make_buffer(const void *base, size_t bytes) {
  const uint32_t n = bytes > 0xffffff00ull ? 0xffffff00u : (uint32_t)bytes;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)n, 0x00020000);
}
__device__ __forceinline__ u32x4 buffer_load16(buffer_t b, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(b, (int)byte_off, 0, 0);
}

// ---- swizzled LDS blocks --------------------------------------------------------------------
// A [rows][128] bf16 block stored without padding (256 B per row, 16 chunks of 16 B); chunk ch of
// row j sits at chunk position ch ^ swz(j).  With swz(j) = ((j & 3) << 2) | ((j >> 2) & 3) both
// access patterns the backward needs are free of bank conflicts on the same copy of the data:
//   - row reads (A operand "rows = block rows"): 16 consecutive rows, one chunk each, land on 16
//     different chunk positions;
//   - transposing reads (A operand "rows = block columns"): 4 consecutive rows x 4 chunks land on
//     4 different groups of 4 chunk positions.
__device__ __forceinline__ int swz(int j) { return ((j & 3) << 2) | ((j >> 2) & 3); }

// Byte offset inside a swizzled block of this lane's row-read fragment for k-step 0 of the 32-row
// group starting at row 0: row = lane % 32, chunk = half.  For k-step ks XOR the result with
// (2 * ks) << 4; for the next 32-row group add 32 * 256.
__device__ __forceinline__ uint32_t swz_row_lane_off(int lane) {
  const int l32 = lane & 31, half = lane >> 5;
  return (uint32_t)(l32 * 256 + ((half ^ swz(l32)) << 4));
}
template <class E>
__device__ __forceinline__ typename E::x8 swz_read_row(const uint16_t *blk, uint32_t lane_off, int ks, int row0) {
  const uint32_t off = (lane_off ^ (uint32_t)(ks << 5)) + (uint32_t)row0 * 256u;
  return as_x8<E>(*(const u32x4 *)((const char *)blk + off));
}

// Transposing reads from a swizzled block: byte offsets of this lane's two 8-byte reads (rows
// 4 half + r and 8 + 4 half + r of a 16-row k-step, column block 0).  For column block cb XOR with
// cb << 6; for k-step base row j0 (a multiple of 16) add j0 * 256.
__device__ __forceinline__ void swz_tr_lane_off(int lane, uint32_t (&off)[2]) {
  const int b = lane >> 4, r = (lane & 15) >> 2, q = lane & 3;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j16 = 8 * t + 4 * (b >> 1) + r;
    const int ch = 2 * (b & 1) + (q >> 1);
    off[t] = (uint32_t)(j16 * 256 + ((ch ^ swz(j16)) << 4) + (q & 1) * 8);
  }
}
template <class E>
__device__ __forceinline__ typename E::x8 swz_read_tr(const uint16_t *blk, const uint32_t (&lane_off)[2], int cb, int j0) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const char *base = (const char *)blk + (uint32_t)j0 * 256u;
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(base + (lane_off[0] ^ (uint32_t)(cb << 6))));
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(base + (lane_off[1] ^ (uint32_t)(cb << 6))));
  const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(typename E::x8, r);
}

// 16-byte global load with a validity guard (zero when !ok)
__device__ __forceinline__ u32x4 ldg16(const uint16_t *p, bool ok) {
  u32x4 z = {0u, 0u, 0u, 0u};
  return ok ? *(const u32x4 *)p : z;
}
// Cache-policy operand of a block copy whose rows no other workgroup reads again (a dQ workgroup's
// own Q, dO and O rows, a dK/dV workgroup's own K and V rows): non-temporal, so that they do not
// displace the streamed blocks that neighbouring workgroups share through L2.  The result stores of
// store_transposed_tile carry the same hint.  Measured: backward 1-4 % faster on every workload.  Not
// for loads that fetch a cache line piecewise (the forward's per-lane Q fragments: 8 % slower).
constexpr int kOnce = 2;

// This lane's row of a [N, H, d] tensor as kKs operand fragments: fragment ks holds columns
// 16 ks + 8 half .. + 7; columns at or beyond d read as zeros.
template <class E, int kKs>
__device__ __forceinline__ void load_row_fragments(const uint16_t *row, int d, int half, typename E::x8 (&f)[kKs]) {
#pragma unroll
  for (int ks = 0; ks < kKs; ++ks) {
    const int c = ks * 16 + half * 8;
    f[ks] = as_x8<E>(ldg16(row + c, c < d));
  }
}

// Per-lane part of the HBM -> LDS copy of swizzled blocks (see the forward kernel): the lane that
// lands at chunk position lane % 16 of LDS row `row` fetches global chunk (lane % 16) ^ swz(row) of
// that row and head.  A chunk at or beyond the head_dim must bring zeros: dma_lane_ok is false for
// it and the copy then uses the offset kPastEnd (beyond every buffer) instead.
__device__ __forceinline__ uint32_t dma_lane_offset(int lane, int row, size_t row_bytes, int head, int d) {
  const int gc = (lane & 15) ^ swz(row);
  return (uint32_t)(row * row_bytes + (size_t)head * d * 2 + gc * 16);
}
__device__ __forceinline__ bool dma_lane_ok(int lane, int row, int d) { return (((lane & 15) ^ swz(row)) * 8) < d; }

// Epilogue shared by all three kernels: a wave holds a transposed result tile
//   acc[cb][v] = R[row = lane % 32][col = 32 cb + acc_row(v, half)],   32 rows x 32 kCb cols,
// multiplies row `lane % 32` by `mul`, and writes columns < d of rows 0..nrows-1 to
// out[(row0 + row) * H + head] (a [N, H, d] tensor) with coalesced stores.  The tile is staged
// through LDS in halves of 64 columns; `stage` is this wave's private [32][kStageStride] float
// buffer, so only wave-level ordering is needed here (LDS operations of one wave execute in
// order).  The caller must have passed a workgroup barrier after the last use of the memory `stage`
// overlays.  EOut = float stores fp32, otherwise the 16-bit element type of EOut.
constexpr int kStageStride = 64 + 4;
constexpr int kStageFloatsPerWave = 32 * kStageStride;

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <class EOut> struct is_f32_out { static constexpr bool value = false; };
template <> struct is_f32_out<float> { static constexpr bool value = true; };
template <class EOut, bool kF32 = is_f32_out<EOut>::value> struct OutPack {
  static __device__ __forceinline__ uint32_t two(float lo, float hi) { return pack2<EOut>(lo, hi); }
};
template <class EOut> struct OutPack<EOut, true> {
  static __device__ __forceinline__ uint32_t two(float, float) { return 0u; }
};

template <class EOut, int kCb>
__device__ __forceinline__ void store_transposed_tile(const f32x16 (&acc)[kCb], float mul, float *stage,
                                                      void *out, long long row0, int nrows, int H,
                                                      int head, int d) {
  const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
#pragma unroll
  for (int p = 0; p < (kCb + 1) / 2; ++p) {
    wave_lds_fence();  // the reads of the previous half (or tile) are done before it is overwritten
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      if (2 * p + cc >= kCb) continue;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 w;
#pragma unroll
        for (int b = 0; b < 4; ++b) w[b] = acc[2 * p + cc][4 * q4 + b] * mul;
        *(f32x4 *)(stage + l32 * kStageStride + cc * 32 + q4 * 8 + half * 4) = w;
      }
    }
    wave_lds_fence();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int rr = it * 4 + (lane >> 4), c4 = lane & 15;
      const int col = p * 64 + c4 * 4;
      if (rr < nrows && col < d && col < kCb * 32) {
        const f32x4 x = *(const f32x4 *)(stage + rr * kStageStride + c4 * 4);
        const size_t off = ((size_t)(row0 + rr) * H + head) * d + col;
        if (is_f32_out<EOut>::value) {
          __builtin_nontemporal_store(x, (f32x4 *)((float *)out + off));
        } else {
          u32x2 w;
          w.x = OutPack<EOut>::two(x[0], x[1]);
          w.y = OutPack<EOut>::two(x[2], x[3]);
          __builtin_nontemporal_store(w, (u32x2 *)((uint16_t *)out + off));
        }
      }
    }
  }
}


}  // namespace va
