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

constexpr int kBT = 128;             // resident rows per workgroup (queries for dQ, keys for dK/dV)
constexpr int kSub = VA_TILE / kBT;  // workgroup tiles per schedule tile
constexpr int kBS = 64;              // streamed rows per LDS block
constexpr int kBlk = kBS * kD;       // elements of one swizzled [64][128] LDS block (16 KB)
constexpr float kLog2e = 1.4426950408889634f;

typedef BlockCopy<kBS, 256> Copy;  // 4 x 16 B per thread and block

// ---------------------------------------------------------------------------------------------
template <bool kF32Out>
__global__ void __launch_bounds__(256, 2)
dq_mfma_kernel(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ Q,
               const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
               const float *__restrict__ LSE, const float *__restrict__ delta, void *__restrict__ dQ,
               const int32_t *__restrict__ seg_start, const int32_t *__restrict__ q_tile_order, int N,
               int T, int tiles_per_row, int hq, int hkv, float scale_log2, float scale) {
  // two stages of {K block, V block}, swizzled
  __shared__ __attribute__((aligned(16))) uint16_t lds[4 * kBlk];
  static_assert(4 * kBlk * 2 >= 4 * kStageFloatsPerWave * 4, "staging must fit");

  const int lane = threadIdx.x & 63, wave = uniform(threadIdx.x >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  // schedule tiles hold kSub workgroup tiles; workgroups of one schedule tile are adjacent
  const int wg = xcd_group_remap(blockIdx.x, hq / hkv, gridDim.x);
  const int tile = uniform(q_tile_order[wg / (hq * kSub)]);
  const int sub = (wg / hq) % kSub;
  const int h = wg % hq;
  const int g = h / (hq / hkv);
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;
  const int t0 = r * T + m * VA_TILE + sub * kBT;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kBT, row_end) - 1;
  const int jb_lo = uniform(seg_start[t0]) / kBS, jb_hi = t_last / kBS;

  const int iw0 = t0 + wave * 32;
  const int iw1 = min(iw0 + 31, t_last);
  const bool wave_ok = iw0 <= t_last;
  const bool wave_full = iw0 + 31 <= t_last;
  const int ss_min = uniform(seg_start[min(iw0, t_last)]);
  const int ss_max = uniform(seg_start[iw1 < iw0 ? t_last : iw1]);
  const int i_abs = iw0 + l32;
  const bool row_ok = i_abs <= t_last;
  const int i_ld = min(i_abs, t_last);  // clamped: loads stay in bounds, results of dead rows are dropped
  const int ss_i = row_ok ? seg_start[i_ld] : 0x7fffffff;

  bf16x8 qf[8], gf[8];  // Q and dO rows of this lane: B operands
  {
    const size_t off = ((size_t)i_ld * hq + h) * kD + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qf[ks] = as_bf16x8(*(const u32x4 *)(Q + off + ks * 16));
      gf[ks] = as_bf16x8(*(const u32x4 *)(dO + off + ks * 16));
    }
  }
  const float lse2 = LSE[(size_t)h * N + i_ld] * kLog2e;
  const float dl = delta[(size_t)h * N + i_ld];

  f32x16 acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;

  const uint32_t row_lane = swz_row_lane_off(lane);
  uint32_t tr_lane[2];
  swz_tr_lane_off(lane, tr_lane);

  const size_t row_bytes = (size_t)hkv * kD * 2;
  const size_t base_off = (size_t)jb_lo * kBS * row_bytes;
  const size_t total = (size_t)N * row_bytes;
  const buffer_t kbuf = make_buffer((const char *)K + base_off, total - base_off);
  const buffer_t vbuf = make_buffer((const char *)V + base_off, total - base_off);
  // HBM -> LDS copy of a 64-row block by the load unit (see the forward kernel): 4 loads per wave and
  // tensor, each 1 KB = 4 rows at LDS address (4 p + wave) KB; lane L lands at row 16 p + 4 wave + L / 16,
  // chunk position L % 16, and fetches global chunk (L % 16) ^ swz(row).
  const int dma_row = wave * 4 + (lane >> 4);
  const uint32_t dma_off = (uint32_t)(dma_row * row_bytes + g * kD * 2 + (((lane & 15) ^ swz(dma_row)) << 4));
  const uint32_t blk_bytes = (uint32_t)(kBS * row_bytes);
  const uint32_t p_bytes = (uint32_t)(16 * row_bytes);
  typedef __attribute__((address_space(3))) void *lds_void;
  auto copy_block = [&](uint16_t *Kd, uint16_t *Vd, int jb) {  // rows past the tensor arrive as zeros
    const uint32_t off = dma_off + (uint32_t)(jb - jb_lo) * blk_bytes;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kbuf, (lds_void)(Kd + (4 * p + wave) * 512), 16, off + p * p_bytes, 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vbuf, (lds_void)(Vd + (4 * p + wave) * 512), 16, off + p * p_bytes, 0, 0, 0);
    }
  };

  // One iteration: start the copy of block jb+1 into the other stage (last read before the previous
  // barrier), consume block jb from (Kb, Vb); the barrier at the end publishes the copied block.
  auto iteration = [&](int jb, const uint16_t *__restrict__ Kb, const uint16_t *__restrict__ Vb,
                       uint16_t *__restrict__ Kn, uint16_t *__restrict__ Vn) {
    if (jb < jb_hi) copy_block(Kn, Vn, jb + 1);  // workgroup-uniform
    const int j0 = jb * kBS;
    if (wave_ok && j0 <= iw1 && j0 + kBS - 1 >= ss_min) {  // wave-uniform
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const int jl = j0 + sb * 32;
        if (jl > iw1 || jl + 31 < ss_min) continue;  // wave-uniform
        f32x16 s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          s = mfma32(swz_read_row(Kb, row_lane, ks, sb * 32), qf[ks], s);     // S^T  = K Q^T
          dp = mfma32(swz_read_row(Vb, row_lane, ks, sb * 32), gf[ks], dp);   // dP^T = V dO^T
        }
        const bool interior = wave_full && jl >= ss_max && jl + 31 <= iw0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float p = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, -lse2));
          if (!interior) {
            const int j = jl + acc_row(v, half);
            if (j < ss_i || j > i_abs) p = 0.f;
          }
          s[v] = p * (dp[v] - dl);  // dS^T
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 df = pack_bf16x8(s, 8 * s2);
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)  // dQ^T += K^T dS^T
            acc[cb] = mfma32(swz_read_tr(Kb, tr_lane, cb, sb * 32 + s2 * 16), df, acc[cb]);
        }
      }
    }
    __syncthreads();
  };

  uint16_t *K0 = lds, *V0 = lds + kBlk, *K1 = lds + 2 * kBlk, *V1 = lds + 3 * kBlk;
  copy_block(K0, V0, jb_lo);
  wait_all_loads();  // Q / dO fragments too: inside the loop only block copies are in flight
  __syncthreads();
  for (int jb = jb_lo; jb <= jb_hi; jb += 2) {  // bounds are workgroup-uniform: barriers stay aligned
    iteration(jb, K0, V0, K1, V1);
    if (jb + 1 <= jb_hi) iteration(jb + 1, K1, V1, K0, V0);
  }

  float *stage = (float *)lds + wave * kStageFloatsPerWave;
  store_transposed_tile<kF32Out>(acc, scale, stage, dQ, iw0, wave_ok ? iw1 - iw0 + 1 : 0, hq, h);
}

// One 32-query sub-block of the dK/dV kernel for this wave's 32 keys.  All LDS fragments of a phase
// are requested before the MFMAs that consume them, and the transposed fragments of the second
// phase are requested before the exp / dS arithmetic, so LDS latency overlaps matrix and vector work.
__device__ __forceinline__ void dkdv_subblock(bool need_mask, f32x16 (&dk_acc)[4], f32x16 (&dv_acc)[4], const bf16x8 (&kf)[8],
                                              const bf16x8 (&vf)[8], const uint16_t *Qs, const uint16_t *Gs,
                                              const float *lse_s, const float *dl_s, int row0, uint32_t row_lane,
                                              const uint32_t (&tr_lane)[2], int half, int il, int j_abs, int se_j,
                                              float scale_log2) {
  // the accumulators start from the per-query constants: S from -LSE / scale, dP from -D
  f32x16 s, dp;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const f32x4 l = *(const f32x4 *)(lse_s + row0 + q4 * 8 + half * 4);
    const f32x4 d = *(const f32x4 *)(dl_s + row0 + q4 * 8 + half * 4);
#pragma unroll
    for (int b = 0; b < 4; ++b) { s[q4 * 4 + b] = l[b]; dp[q4 * 4 + b] = d[b]; }
  }
  bf16x8 aq[8], ag[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    aq[ks] = swz_read_row(Qs, row_lane, ks, row0);
    ag[ks] = swz_read_row(Gs, row_lane, ks, row0);
  }
  __builtin_amdgcn_sched_barrier(0);  // keep every read above in flight before the first MFMA
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    s = mfma32(aq[ks], kf[ks], s);     // S - LSE / scale  = Q K^T - LSE / scale
    dp = mfma32(ag[ks], vf[ks], dp);   // dP - D           = dO V^T - D
  }
  bf16x8 tq[2][4], tg[2][4];
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      tg[s2][cb] = swz_read_tr(Gs, tr_lane, cb, row0 + s2 * 16);
      tq[s2][cb] = swz_read_tr(Qs, tr_lane, cb, row0 + s2 * 16);
    }
  __builtin_amdgcn_sched_barrier(0);  // transposed fragments land while the arithmetic below runs
#pragma unroll
  for (int v = 0; v < 16; ++v) s[v] = __builtin_amdgcn_exp2f(s[v] * scale_log2);  // P
  if (need_mask) {  // wave-uniform; touches only the probabilities
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = il + acc_row(v, half);
      if (i < j_abs || i >= se_j) s[v] = 0.f;
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) dp[v] *= s[v];  // dS
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2) {
    const bf16x8 pf = pack_bf16x8(s, 8 * s2);
    const bf16x8 df = pack_bf16x8(dp, 8 * s2);
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      dv_acc[cb] = mfma32(tg[s2][cb], pf, dv_acc[cb]);  // dV^T += dO^T P
      dk_acc[cb] = mfma32(tq[s2][cb], df, dk_acc[cb]);  // dK^T += Q^T dS
    }
  }
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
  // two stages of {Q block, dO block (swizzled), -LSE / scale [64], -D [64]}
  constexpr int kStage = 2 * kBlk + 4 * kBS;  // elements (floats take two)
  __shared__ __attribute__((aligned(16))) uint16_t lds[2 * kStage];
  static_assert(2 * kStage * 2 >= 4 * kStageFloatsPerWave * 4, "staging must fit");

  const int lane = threadIdx.x & 63, wave = uniform(threadIdx.x >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int tile = uniform(kv_tile_order[blockIdx.x / (hkv * kSub)]);
  const int sub = (blockIdx.x / hkv) % kSub;
  const int g = blockIdx.x % hkv;
  const int G = hq / hkv;
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;
  const int t0 = r * T + m * VA_TILE + sub * kBT;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kBT, row_end) - 1;
  const int ib_lo = t0 / kBS;  // first query block that can see a key of this tile

  const size_t row_bytes = (size_t)hq * kD * 2;
  const size_t base_off = (size_t)ib_lo * kBS * row_bytes;
  const size_t total = (size_t)N * row_bytes;
  const buffer_t qbuf = make_buffer((const char *)Q + base_off, total - base_off);
  const buffer_t gbuf = make_buffer((const char *)dO + base_off, total - base_off);
  // HBM -> LDS copy of a 64-row Q / dO block by the load unit (see the forward kernel)
  const int dma_row = wave * 4 + (lane >> 4);
  const uint32_t dma_off = (uint32_t)(dma_row * row_bytes + (((lane & 15) ^ swz(dma_row)) << 4));
  const uint32_t blk_bytes = (uint32_t)(kBS * row_bytes);
  const uint32_t p_bytes = (uint32_t)(16 * row_bytes);
  typedef __attribute__((address_space(3))) void *lds_void;
  const int stat_row = threadIdx.x & (kBS - 1);
  const bool stat_is_lse = (threadIdx.x & kBS) == 0;  // threads 0..63 (and 128..191): LSE; others: D
  const float *stat_src = stat_is_lse ? LSE : delta;
  const float stat_mul = stat_is_lse ? -1.f / scale : -1.f;
  float rstat;
  // Q, dO blocks (query head g * G + hh, block ib) -> stage at dst; LSE / D value -> rstat
  auto copy_block = [&](uint16_t *dst, int hh, int ib) {
    const int i = min(ib * kBS + stat_row, N - 1);
    rstat = stat_src[(size_t)(g * G + hh) * N + i];
    const uint32_t off = dma_off + (uint32_t)(ib - ib_lo) * blk_bytes + (uint32_t)((g * G + hh) * kD * 2);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(qbuf, (lds_void)(dst + (4 * p + wave) * 512), 16, off + p * p_bytes, 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(gbuf, (lds_void)(dst + kBlk + (4 * p + wave) * 512), 16,
                                               off + p * p_bytes, 0, 0, 0);
    }
  };
  // the first block needs nothing but the tile: its copy starts before the example bounds arrive
  uint16_t *S0 = lds, *S1 = lds + kStage;
  copy_block(S0, 0, ib_lo);

  // query blocks end with the example holding the tile's last key
  const int ib_hi = (uniform(seg_end[t_last]) - 1) / kBS;
  const int nb = ib_hi - ib_lo + 1;

  const int jw0 = t0 + wave * 32;
  const int jw1 = min(jw0 + 31, t_last);
  const bool wave_ok = jw0 <= t_last;
  const bool wave_full = jw0 + 31 <= t_last;
  const int se_min = uniform(seg_end[min(jw0, t_last)]);
  const int se_max = uniform(seg_end[jw1 < jw0 ? t_last : jw1]);
  const int j_abs = jw0 + l32;
  const bool row_ok = j_abs <= t_last;
  const int j_ld = min(j_abs, t_last);
  const int se_j = row_ok ? seg_end[j_ld] : 0;  // queries j_abs <= i < se_j see key j_abs

  bf16x8 kf[8], vf[8];  // K and V rows of this lane: B operands
  {
    const size_t off = ((size_t)j_ld * hkv + g) * kD + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kf[ks] = as_bf16x8(*(const u32x4 *)(K + off + ks * 16));
      vf[ks] = as_bf16x8(*(const u32x4 *)(V + off + ks * 16));
    }
  }

  f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk_acc[cb][v] = 0.f; dv_acc[cb][v] = 0.f; }

  const uint32_t row_lane = swz_row_lane_off(lane);
  uint32_t tr_lane[2];
  swz_tr_lane_off(lane, tr_lane);

  // iteration `it` streams query block ib_lo + it % nb of query head g * G + it / nb
  const int n_it = nb * G;
  auto put_stats = [&](uint16_t *dst) {  // [64] -LSE / scale, [64] -D behind the two blocks
    if (threadIdx.x < 2 * kBS) ((float *)(dst + 2 * kBlk))[threadIdx.x] = rstat * stat_mul;
  };

  // One iteration: start the copy of the next block into the other stage (last read before the
  // previous barrier), consume the current one, publish the next with the barrier at the end.
  int ib_cur = ib_lo, ib_nxt = ib_lo, hh_nxt = 0;  // block being consumed; block / head being copied
  auto iteration = [&](int it, const uint16_t *__restrict__ cur, uint16_t *__restrict__ nxt) {
    const bool more = it + 1 < n_it;  // workgroup-uniform
    if (++ib_nxt > ib_hi) { ib_nxt = ib_lo; ++hh_nxt; }
    if (more) copy_block(nxt, hh_nxt, ib_nxt);
    const uint16_t *Qs = cur, *Gs = cur + kBlk;
    const float *lse_s = (const float *)(cur + 2 * kBlk), *dl_s = lse_s + kBS;
    const int i0 = ib_cur * kBS;
    ib_cur = ib_nxt;
    if (wave_ok && i0 + kBS - 1 >= jw0 && i0 < se_max) {  // wave-uniform
#pragma unroll 1  // one code instance per stage: the accumulators keep their registers
      for (int sb = 0; sb < 2; ++sb) {
        const int il = i0 + sb * 32;
        if (il + 31 < jw0 || il >= se_max) continue;  // wave-uniform
        const bool interior = wave_full && il >= jw1 && il + 31 < se_min;
        dkdv_subblock(!interior, dk_acc, dv_acc, kf, vf, Qs, Gs, lse_s, dl_s, sb * 32, row_lane, tr_lane, half, il,
                      j_abs, se_j, scale_log2);
      }
    }
    if (more) put_stats(nxt);
    __syncthreads();
  };

  put_stats(S0);
  // every load issued so far (K/V fragments included) lands here: inside the loop only the block
  // copies are in flight, and nothing but the barrier waits for them
  wait_all_loads();
  __syncthreads();
  for (int it = 0; it < n_it; it += 2) {  // bounds are workgroup-uniform: barriers stay aligned
    iteration(it, S0, S1);
    if (it + 1 < n_it) iteration(it + 1, S1, S0);
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
