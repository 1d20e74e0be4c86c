// Backward kernels: dQ (query-major) and dK/dV (key-major), bf16, head_dim 128.
//
// What they compute (see include/varlen_attn.h), from the saved LSE and D = rowsum(dO * O):
//   P_ij = exp(scale q_i.k_j - LSE_i),  dP_ij = dO_i.v_j,  dS_ij = P_ij (dP_ij - D_i)
//   dQ_i = scale sum_j dS_ij k_j;   dK_j = scale sum_i dS_ij q_i;   dV_j = sum_i P_ij dO_i
// over the pairs a <= j <= i of one example (Table 1's mask; bounds from the position-id scan,
// paper Section 3), dK/dV also summed over the query heads that share the KV head.
//
// Two kernels, no atomics, bitwise reproducible:
//   dq_mfma_kernel   : workgroup = (128-query tile, query head); streams K/V blocks of 64 rows.
//                      Lane owns a query row: S^T = K Q^T, dP^T = V dO^T, dQ^T += K^T dS^T.
//   dkdv_mfma_kernel : workgroup = (128-key tile, KV head); streams Q/dO blocks of 64 rows of every
//                      query head of the group.  Lane owns a key row: S = Q K^T, dP = dO V^T,
//                      dV^T += dO^T P, dK^T += Q^T dS.
// In both, the streamed index lies on the accumulator's register axis and feeds the last
// contraction as a B operand straight from registers (see va_mfma_common.h).
#include "va_internal.h"
#include "va_mfma_common.h"

namespace va {
namespace {

constexpr int kBT = 128;        // resident rows per workgroup (queries for dQ, keys for dK/dV)
constexpr int kSub = VA_TILE / kBT;  // workgroup tiles per schedule tile
constexpr int kBS = 64;         // streamed rows per LDS block
constexpr int kRS = kD + 8;     // LDS stride of a row-major [64][128] block (elements)
constexpr int kTS = kBS + 8;    // LDS stride of a transposed [128][64] block
constexpr int kRowBlk = kBS * kRS;
constexpr int kTrBlk = kD * kTS;
constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------------
template <bool kF32Out>
__global__ void __launch_bounds__(256, 2)
dq_mfma_kernel(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ Q,
               const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
               const float *__restrict__ LSE, const float *__restrict__ delta, void *__restrict__ dQ,
               const int32_t *__restrict__ seg_start, const int32_t *__restrict__ q_tile_order, int N,
               int T, int tiles_per_row, int hq, int hkv, float scale_log2, float scale) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[2 * kRowBlk + kTrBlk];
  static_assert((2 * kRowBlk + kTrBlk) * 2 >= 4 * kStageFloatsPerWave * 4, "staging must fit");
  uint16_t *Ks = lds, *Vs = lds + kRowBlk, *Kt = lds + 2 * kRowBlk;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // schedule tiles hold kSub workgroup tiles; workgroups of one schedule tile are adjacent
  const int tile = q_tile_order[blockIdx.x / (hq * kSub)];
  const int sub = (blockIdx.x / hq) % kSub;
  const int h = blockIdx.x % hq;
  const int g = h / (hq / hkv);
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;
  const int t0 = r * T + m * VA_TILE + sub * kBT;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kBT, row_end) - 1;

  const int i_abs = t0 + wave * 32 + l32;
  const bool row_ok = i_abs <= t_last;
  const int ss_i = row_ok ? seg_start[i_abs] : 0x7fffffff;
  const int iw0 = t0 + wave * 32;
  const int iw1 = min(iw0 + 31, t_last);
  const bool wave_ok = iw0 <= t_last;
  const int ss_min = wave_ok ? seg_start[iw0] : 0;
  const int ss_max = wave_ok ? seg_start[iw1] : 0;

  bf16x8 qf[8], gf[8];  // Q and dO rows of this lane: B operands
  {
    const size_t off = ((size_t)(row_ok ? i_abs : t0) * hq + h) * kD + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qf[ks] = as_bf16x8(ldg16(Q + off + ks * 16, row_ok));
      gf[ks] = as_bf16x8(ldg16(dO + off + ks * 16, row_ok));
    }
  }
  const float lse2 = row_ok ? LSE[(size_t)h * N + i_abs] * kLog2e : 0.f;
  const float dl = row_ok ? delta[(size_t)h * N + i_abs] : 0.f;

  f32x16 acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;

  const int jb_lo = seg_start[t0] / kBS, jb_hi = t_last / kBS;
  for (int jb = jb_lo; jb <= jb_hi; ++jb) {
    const int j0 = jb * kBS;
    __syncthreads();
    load_rows_to_lds(K, j0, N, hkv, g, Ks, kRS);
    load_rows_to_lds(V, j0, N, hkv, g, Vs, kRS);
    load_rows_to_lds_transposed(K, j0, N, hkv, g, Kt, kTS);
    __syncthreads();
    if (!wave_ok || j0 > iw1 || j0 + kBS - 1 < ss_min) continue;

#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      const int jl = j0 + sb * 32;
      if (jl > iw1 || jl + 31 < ss_min) continue;  // wave-uniform
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int o = (sb * 32 + l32) * kRS + ks * 16 + half * 8;
        s = mfma32(as_bf16x8(*(const u32x4 *)(Ks + o)), qf[ks], s);
        dp = mfma32(as_bf16x8(*(const u32x4 *)(Vs + o)), gf[ks], dp);
      }
      const bool need_mask = !(jl >= ss_max && jl + 31 <= iw0);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float p = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, -lse2));
        if (need_mask) {
          const int j = jl + acc_row(v, half);
          if (j < ss_i || j > i_abs) p = 0.f;
        }
        s[v] = p * (dp[v] - dl);  // dS^T
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 df = pack_bf16x8(s, 8 * s2);
        const int kstep = sb * 2 + s2;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
          bf16x8 kf = as_bf16x8(*(const u32x4 *)(Kt + (cb * 32 + l32) * kTS + kstep * 16 + half * 8));
          acc[cb] = mfma32(kf, df, acc[cb]);
        }
      }
    }
  }

  float *stage = (float *)lds + wave * kStageFloatsPerWave;
  store_transposed_tile<kF32Out>(acc, scale, stage, dQ, iw0, wave_ok ? iw1 - iw0 + 1 : 0, hq, h);
}

// ---------------------------------------------------------------------------------------------
template <bool kF32Out>
__global__ void __launch_bounds__(256, 1)
dkdv_mfma_kernel(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ Q,
                 const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
                 const float *__restrict__ LSE, const float *__restrict__ delta, void *__restrict__ dK,
                 void *__restrict__ dV, const int32_t *__restrict__ seg_end,
                 const int32_t *__restrict__ kv_tile_order, int N, int T, int tiles_per_row, int hq,
                 int hkv, float scale_log2, float scale) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[2 * kRowBlk + 2 * kTrBlk + 4 * kBS];
  static_assert((2 * kRowBlk + 2 * kTrBlk) * 2 >= 4 * kStageFloatsPerWave * 4, "staging must fit");
  uint16_t *Qs = lds, *Gs = lds + kRowBlk, *Qt = lds + 2 * kRowBlk, *Gt = Qt + kTrBlk;
  float *lse_s = (float *)(Gt + kTrBlk);  // [64] LSE * log2(e)
  float *dl_s = lse_s + kBS;              // [64] D

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int tile = kv_tile_order[blockIdx.x / (hkv * kSub)];
  const int sub = (blockIdx.x / hkv) % kSub;
  const int g = blockIdx.x % hkv;
  const int G = hq / hkv;
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;
  const int t0 = r * T + m * VA_TILE + sub * kBT;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kBT, row_end) - 1;

  const int j_abs = t0 + wave * 32 + l32;
  const bool row_ok = j_abs <= t_last;
  const int se_j = row_ok ? seg_end[j_abs] : 0;  // queries j_abs <= i < se_j see key j_abs
  const int jw0 = t0 + wave * 32;
  const int jw1 = min(jw0 + 31, t_last);
  const bool wave_ok = jw0 <= t_last;
  const int se_min = wave_ok ? seg_end[jw0] : 0;
  const int se_max = wave_ok ? seg_end[jw1] : 0;

  bf16x8 kf[8], vf[8];  // K and V rows of this lane: B operands
  {
    const size_t off = ((size_t)(row_ok ? j_abs : t0) * hkv + g) * kD + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kf[ks] = as_bf16x8(ldg16(K + off + ks * 16, row_ok));
      vf[ks] = as_bf16x8(ldg16(V + off + ks * 16, row_ok));
    }
  }

  f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk_acc[cb][v] = 0.f; dv_acc[cb][v] = 0.f; }

  const int ib_lo = t0 / kBS, ib_hi = (seg_end[t_last] - 1) / kBS;
  for (int hh = 0; hh < G; ++hh) {
    const int h = g * G + hh;
    for (int ib = ib_lo; ib <= ib_hi; ++ib) {
      const int i0 = ib * kBS;
      __syncthreads();
      load_rows_to_lds(Q, i0, N, hq, h, Qs, kRS);
      load_rows_to_lds(dO, i0, N, hq, h, Gs, kRS);
      load_rows_to_lds_transposed(Q, i0, N, hq, h, Qt, kTS);
      load_rows_to_lds_transposed(dO, i0, N, hq, h, Gt, kTS);
      if (threadIdx.x < kBS) {
        const int i = i0 + threadIdx.x;
        lse_s[threadIdx.x] = i < N ? LSE[(size_t)h * N + i] * kLog2e : 0.f;
        dl_s[threadIdx.x] = i < N ? delta[(size_t)h * N + i] : 0.f;
      }
      __syncthreads();
      if (!wave_ok || i0 + kBS - 1 < jw0 || i0 >= se_max) continue;

#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const int il = i0 + sb * 32;
        if (il + 31 < jw0 || il >= se_max) continue;  // wave-uniform
        f32x16 s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const int o = (sb * 32 + l32) * kRS + ks * 16 + half * 8;
          s = mfma32(as_bf16x8(*(const u32x4 *)(Qs + o)), kf[ks], s);
          dp = mfma32(as_bf16x8(*(const u32x4 *)(Gs + o)), vf[ks], dp);
        }
        const bool need_mask = !(il >= jw1 && il + 31 < se_min);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 l4 = *(const f32x4 *)(lse_s + sb * 32 + q4 * 8 + half * 4);
          const f32x4 d4 = *(const f32x4 *)(dl_s + sb * 32 + q4 * 8 + half * 4);
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const int v = q4 * 4 + b;
            float p = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, -l4[b]));
            if (need_mask) {
              const int i = il + acc_row(v, half);
              if (i < j_abs || i >= se_j) p = 0.f;
            }
            s[v] = p;                     // P
            dp[v] = p * (dp[v] - d4[b]);  // dS
          }
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 pf = pack_bf16x8(s, 8 * s2);
          const bf16x8 df = pack_bf16x8(dp, 8 * s2);
          const int kstep = sb * 2 + s2;
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) {
            const int o = (cb * 32 + l32) * kTS + kstep * 16 + half * 8;
            dv_acc[cb] = mfma32(as_bf16x8(*(const u32x4 *)(Gt + o)), pf, dv_acc[cb]);
            dk_acc[cb] = mfma32(as_bf16x8(*(const u32x4 *)(Qt + o)), df, dk_acc[cb]);
          }
        }
      }
    }
  }

  float *stage = (float *)lds + wave * kStageFloatsPerWave;
  const int nrows = wave_ok ? jw1 - jw0 + 1 : 0;
  store_transposed_tile<kF32Out>(dk_acc, scale, stage, dK, jw0, nrows, hkv, g);
  store_transposed_tile<kF32Out>(dv_acc, 1.f, stage, dV, jw0, nrows, hkv, g);
}

}  // namespace

hipError_t launch_mfma_bwd(const void *dO, const void *Q, const void *K, const void *V,
                           const float *LSE, const float *delta, void *dQ, void *dK, void *dV,
                           va_dtype grad_dt, const va_segments &seg, int rows, int T, int hq,
                           int hkv, float scale, hipStream_t stream, unsigned stages) {
  const int tiles_per_row = ceil_div(T, VA_TILE);
  const long long ntiles = (long long)rows * tiles_per_row * kSub;
  if (ntiles * hq > 0x7fffffffll) return hipErrorInvalidValue;
  const int N = rows * T;
  const float scale_log2 = scale * kLog2e;
  const uint16_t *q = (const uint16_t *)Q, *k = (const uint16_t *)K, *v = (const uint16_t *)V,
                 *g = (const uint16_t *)dO;
  const unsigned gq = (unsigned)(ntiles * hq), gkv = (unsigned)(ntiles * hkv);
  const bool do_kv = stages & VA_STAGE_DKDV, do_q = stages & VA_STAGE_DQ;
  if (grad_dt == VA_F32) {
    if (do_kv) dkdv_mfma_kernel<true><<<gkv, 256, 0, stream>>>(g, q, k, v, LSE, delta, dK, dV, seg.seg_end,
                                                    seg.kv_tile_order, N, T, tiles_per_row, hq, hkv,
                                                    scale_log2, scale);
    if (do_q) dq_mfma_kernel<true><<<gq, 256, 0, stream>>>(g, q, k, v, LSE, delta, dQ, seg.seg_start,
                                                 seg.q_tile_order, N, T, tiles_per_row, hq, hkv,
                                                 scale_log2, scale);
  } else {
    if (do_kv) dkdv_mfma_kernel<false><<<gkv, 256, 0, stream>>>(g, q, k, v, LSE, delta, dK, dV, seg.seg_end,
                                                     seg.kv_tile_order, N, T, tiles_per_row, hq, hkv,
                                                     scale_log2, scale);
    if (do_q) dq_mfma_kernel<false><<<gq, 256, 0, stream>>>(g, q, k, v, LSE, delta, dQ, seg.seg_start,
                                                  seg.q_tile_order, N, T, tiles_per_row, hq, hkv,
                                                  scale_log2, scale);
  }
  return hipGetLastError();
}

}  // namespace va
