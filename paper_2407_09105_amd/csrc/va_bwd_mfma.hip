// Backward kernels: dQ (query-major) and dK/dV (key-major), bf16 / fp16, head_dim <= 256.
//
// What they compute (see include/varlen_attn.h), from the saved LSE and D = rowsum(dO * O):
//   P_ij = exp(scale q_i.k_j - LSE_i),  dP_ij = dO_i.v_j,  dS_ij = P_ij (dP_ij - D_i)
//   dQ_i = scale sum_j dS_ij k_j;   dK_j = scale sum_i dS_ij q_i;   dV_j = sum_i P_ij dO_i
// over the pairs a <= j <= i of one example (Table 1's mask; bounds from the position-id scan,
// paper Section 3), dK/dV also summed over the query heads that share the KV head.
//
// Two kernels, no atomics, bitwise reproducible:
//   dq_mfma_kernel   : workgroup = (128-query tile, query head); streams K/V blocks of 64 rows.
//                      Lane owns a query row: S^T = K Q^T, dP^T = V dO^T, dQ^T += K^T dS^T.  It also
//                      forms D for its rows (dO . O, then made exact by the row sums of dS) and stores
//                      it for the other kernel, so it runs first.
//   dkdv_mfma_kernel : workgroup = (128- or 64-key tile, KV head); streams Q/dO blocks of 64 rows of
//                      every query head of the group.  Lane owns a key row: S = Q K^T, dP = dO V^T,
//                      dV^T += dO^T P, dK^T += Q^T dS; the dV and the dK halves run on different waves.
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

// ---- where bf16 operands of the second contraction are carried in two parts ----------------------
// P and dS enter the matrix instructions as 16-bit values.  With bf16 (8 significant bits) the
// rounding of the few large entries - rows with a short context, or a peaked softmax - dominates the
// error of dV, dK and dQ (they are sums over many queries and, with grouped heads, over several
// heads).  A 32x32 sub-block that holds a probability above kSplitP (a score gradient above kSplitS
// in magnitude) therefore adds a second pass with the rounding residuals x - bf16(x); elsewhere the
// residuals are below 2^-9 of those thresholds and are dropped.  fp16 operands (11 bits) need none.
constexpr float kSplitP = 0.125f;
constexpr float kSplitS = 1.0f;
// Waves holding queries with fewer keys than this correct their dQ for the rounding of O in
// D = dO . O (see dq_mfma_kernel).
constexpr int kNearCtx = 64;
// k-steps by which the LDS fragment reads of S and dP run ahead of the matrix instructions that use
// them: in the dQ kernel (two products interleaved) and in the dK/dV kernel (one product per wave).
// Depths 2 to 4 measure the same; the rings occupy registers that the next phase's fragments reuse.
constexpr int kAhead = 2;
constexpr int kAheadKv = 3;

template <class E> struct needs_split { static constexpr bool value = false; };
template <> struct needs_split<Bf16> { static constexpr bool value = true; };

// max |x[v]| over a lane's 16 accumulator values.  x must come from vector arithmetic (not straight from
// a matrix instruction: the compiler does not see a hazard through the asm).  Written as three-operand
// maxima with magnitude modifiers, 8 instructions; from fmaxf(fabsf()) the compiler makes 27.
__device__ __forceinline__ float abs_max16(const f32x16 &x) {
  float m = 0.f;
#pragma unroll
  for (int v = 0; v < 16; v += 2) asm("v_max3_f32 %0, |%1|, |%2|, %3" : "=v"(m) : "v"(x[v]), "v"(x[v + 1]), "v"(m));
  return m;
}
// Rounding residuals x[v0..v0+7] - float(hi[0..7]) as a second operand.
template <class E> __device__ __forceinline__ typename E::x8 pack_residual_x8(const f32x16 &x, int v0, typename E::x8 hi) {
  typename E::x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (typename E::elem)(x[v0 + e] - (float)hi[e]);
  return r;
}


// ---------------------------------------------------------------------------------------------
// Template parameters of both kernels: E element type of the inputs (Bf16 / F16); EOut the
// gradients' type (float, or E); kDh head_dim rounded up to 64, 96, 128 or 256 (the unrolling); the
// argument d is the tensors' head_dim (a multiple of 8, <= kDh).  With kDh = 256 a block is two
// 128-column halves and the dQ kernel runs one workgroup per CU (accumulators in AGPRs).
template <class E, class EOut, int kDh>
__global__ void __launch_bounds__(256, kDh > 128 ? 1 : 2)
dq_mfma_kernel(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ Q,
               const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
               const uint16_t *__restrict__ O, const float *__restrict__ LSE,
               float *__restrict__ delta, void *__restrict__ dQ,
               const int32_t *__restrict__ seg_start, const int32_t *__restrict__ q_tile_order, int N,
               int T, int tiles_per_row, int hq, int hkv, int d, float scale_log2, float scale) {
  constexpr int kKs = kDh / 16, kCb = kDh / 32;
  constexpr int kHf = kDh > 128 ? 2 : 1;   // 128-column sub-blocks per block (head_dim above 128: two)
  constexpr int kBlkT = kBlk * kHf;        // elements of one tensor's streamed block
  constexpr int kTileSub = kBT * kD;       // elements of one sub-block of the tile's own rows
  typedef typename E::x8 x8;
  // two stages of {K block, V block}, swizzled
  __shared__ __attribute__((aligned(16))) uint16_t lds[4 * kBlkT];
  static_assert(4 * kBlk * 2 >= 4 * kStageFloatsPerWave * 4, "staging must fit");

  const int lane = threadIdx.x & 63, wave = uniform(threadIdx.x >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  // schedule tiles hold kSub workgroup tiles; workgroups of one schedule tile are adjacent
  const int wg = xcd_group_remap(blockIdx.x, hq / hkv, gridDim.x);
  const int entry = uniform(q_tile_order[wg / (hq * kSub)]);
  const int tile = order_tile(entry);
  const int sub = (wg / hq) % kSub;
  const int h = (wg % hq + head_rotation(entry) * (hq / hkv)) % hq;
  const int g = h / (hq / hkv);
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;
  const int t0 = r * T + m * VA_TILE + sub * kBT;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kBT, row_end) - 1;
  // Prologue.  The tile's own Q, dO and O rows come in through LDS as whole-row block copies, into
  // the memory of the K/V stages, which is idle until the loop starts (loading the per-lane
  // fragments straight from HBM -- 32 rows x 32 B per instruction -- took 8 us per workgroup):
  //   batch 1: Q -> first half of the stage memory, dO -> second half; scalars (example bounds, LSE)
  //   batch 2: O -> second half, first K/V block -> first half (= stage 0 of the loop)
  // All loads of a batch are requested before any is consumed.
  const int iw0 = t0 + wave * 32;
  const int iw1 = min(iw0 + 31, t_last);
  const bool wave_ok = iw0 <= t_last;
  const bool wave_full = iw0 + 31 <= t_last;
  const int i_abs = iw0 + l32;
  const bool row_ok = i_abs <= t_last;
  const int i_ld = min(i_abs, t_last);  // clamped: loads stay in bounds, results of dead rows are dropped
  const uint32_t row_lane = swz_row_lane_off(lane);
  uint32_t tr_lane[2];
  swz_tr_lane_off(lane, tr_lane);
  typedef __attribute__((address_space(3))) void *lds_void;
  uint16_t *K0 = lds, *V0 = lds + kBlkT, *K1 = lds + 2 * kBlkT, *V1 = lds + 3 * kBlkT;
  const int dma_row = wave * 4 + (lane >> 4);
  bool dma_ok[kHf];  // the same for every transfer of this lane into a sub-block (rows 16 apart)
#pragma unroll
  for (int hf = 0; hf < kHf; ++hf) dma_ok[hf] = dma_lane_ok(lane, dma_row, d - 128 * hf);

  const size_t q_row_bytes = (size_t)hq * d * 2;
  const size_t q_off = (size_t)t0 * q_row_bytes, q_total = (size_t)N * q_row_bytes;
  const uint32_t tile_off = dma_lane_offset(lane, dma_row, q_row_bytes, h, d);
  // 128 rows of one tensor (head h) -> 32 KB per sub-block at dst: 8 transfers of 4 rows per wave
  auto copy_tile = [&](const uint16_t *X, uint16_t *dst) {
    const buffer_t xb = make_buffer((const char *)X + q_off, q_total - q_off);
#pragma unroll
    for (int hf = 0; hf < kHf; ++hf)
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const uint32_t o = dma_ok[hf] ? tile_off + p * (uint32_t)(16 * q_row_bytes) + hf * 256 : kPastEnd;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (lds_void)(dst + hf * kTileSub + (4 * p + wave) * 512), 16, o, 0, 0, kOnce);
      }
  };
  copy_tile(Q, K0);
  copy_tile(dO, K1);
  const int ss_t0_v = seg_start[t0];
  const int ss_min_v = seg_start[min(iw0, t_last)];
  const int ss_max_v = seg_start[iw1 < iw0 ? t_last : iw1];
  const int ss_i_v = seg_start[i_ld];
  const float lse_v = LSE[(size_t)h * N + i_ld];

  // Key blocks are counted from the packed row's first token (block jb = tokens jbase + 64 jb ...):
  // a tile's own rows are then exactly its last two blocks whatever T, which the short-context
  // correction after the loop relies on (with blocks counted from token 0 a tile of a row that does
  // not start on a multiple of 64 straddles three).
  const int jbase = (r * T) % kBS;
  const int jb_lo = (uniform(ss_t0_v) - jbase) / kBS, jb_hi = (t_last - jbase) / kBS;  // jb_hi - 1, jb_hi: the tile's own rows
  const int ss_min = uniform(ss_min_v), ss_max = uniform(ss_max_v);
  const int ss_i = row_ok ? ss_i_v : 0x7fffffff;
  f32x16 acc[kCb];
#pragma unroll
  for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;

  const size_t row_bytes = (size_t)hkv * d * 2;
  const size_t base_off = ((size_t)jb_lo * kBS + jbase) * row_bytes;
  const size_t total = (size_t)N * row_bytes;
  const buffer_t kbuf = make_buffer((const char *)K + base_off, total - base_off);
  const buffer_t vbuf = make_buffer((const char *)V + base_off, total - base_off);
  // HBM -> LDS copy of a 64-row block by the load unit (see the forward kernel): 4 loads per wave and
  // tensor, each 1 KB = 4 rows at LDS address (4 p + wave) KB; lane L lands at row 16 p + 4 wave + L / 16,
  // chunk position L % 16, and fetches global chunk (L % 16) ^ swz(row).
  const uint32_t dma_off = dma_lane_offset(lane, dma_row, row_bytes, g, d);
  const uint32_t blk_bytes = (uint32_t)(kBS * row_bytes);
  const uint32_t p_bytes = (uint32_t)(16 * row_bytes);
  auto copy_block = [&](uint16_t *Kd, uint16_t *Vd, int jb) {  // rows past the tensor arrive as zeros
    const uint32_t off = dma_off + (uint32_t)(jb - jb_lo) * blk_bytes;
#pragma unroll
    for (int hf = 0; hf < kHf; ++hf)
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const uint32_t o = dma_ok[hf] ? off + p * p_bytes + hf * 256 : kPastEnd;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(kbuf, (lds_void)(Kd + hf * kBlk + (4 * p + wave) * 512), 16, o, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(vbuf, (lds_void)(Vd + hf * kBlk + (4 * p + wave) * 512), 16, o, 0, 0, 0);
      }
  };

  // The example of the tile's first row began fewer than kNearCtx tokens before the tile (workgroup-
  // uniform): the short-context correction of the first waves then needs the kNearCtx K rows before the
  // tile, the end of block jb_prev = jb_hi - 2, which has left the stages by the end of the loop.  They
  // are copied once more during the last iteration, into the V half of the other stage (dead by then).
  // (A tile of at most 64 rows has jb_prev = jb_hi - 1, still in its stage: nothing to copy.)
  static_assert(kNearCtx == 32 || kNearCtx == 64, "the rows kept for the correction are part of one 64-row block");
  // head_dim <= 32 (the smallest instantiation only): the whole correction -c_i sum_j P_ij k_j is kept, in a
  // second accumulator fed by the K^T fragments the dQ product reads anyway.  The softmax scale 1 / sqrt(d)
  // is large there, the same error in D weighs 2..4 times more in dQ than at head_dim 128, and the
  // instantiation has the registers; larger head dims take the correction on the nearest keys only (below).
  constexpr bool kHasPk = kDh == 64;
  const bool pk_on = kHasPk && d <= 32;  // workgroup-uniform
  f32x16 pk[kHasPk ? kCb : 1];
  if constexpr (kHasPk) {
#pragma unroll
    for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
      for (int v = 0; v < 16; ++v) pk[cb][v] = 0.f;
  }
  const int ss_t0 = uniform(ss_t0_v);
  const int jb_prev = (t0 - jbase) / kBS - 1;
  const bool need_prev = !pk_on && ss_t0 < t0 && t0 - ss_t0 < kNearCtx && jb_prev == jb_hi - 2 && jb_prev >= jb_lo;
  auto copy_prev_rows = [&](uint16_t *dst) {
    const uint32_t off = dma_off + (uint32_t)(jb_prev - jb_lo) * blk_bytes;
#pragma unroll
    for (int hf = 0; hf < kHf; ++hf)
#pragma unroll
      for (int p = (kBS - kNearCtx) / 16; p < 4; ++p) {
        const uint32_t o = dma_ok[hf] ? off + p * p_bytes + hf * 256 : kPastEnd;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(kbuf, (lds_void)(dst + hf * kBlk + (4 * p + wave) * 512), 16, o, 0, 0, 0);
      }
  };

  x8 qf[kKs], gf[kKs];  // Q and dO rows of this lane: B operands
  wait_all_loads();
  __syncthreads();  // batch 1 has landed
#pragma unroll
  for (int ks = 0; ks < kKs; ++ks) {
    qf[ks] = swz_read_row<E>(K0 + (ks >> 3) * kTileSub, row_lane, ks & 7, wave * 32);
    gf[ks] = swz_read_row<E>(K1 + (ks >> 3) * kTileSub, row_lane, ks & 7, wave * 32);
  }
  __syncthreads();  // every wave has its Q and dO fragments: the memory is free again
  copy_tile(O, K1);
  copy_block(K0, V0, jb_lo);
  const float lse2 = lse_v * kLog2e;
  wait_all_loads();
  __syncthreads();  // batch 2 has landed
  // D = dO . O of this lane's query row, computed here (each lane of a pair holds half of the row)
  // and left in `delta` for the dK/dV kernel, which runs after this one
  float dl = 0.f;
#pragma unroll
  for (int ks = 0; ks < kKs; ++ks) {
    const x8 of = swz_read_row<E>(K1 + (ks >> 3) * kTileSub, row_lane, ks & 7, wave * 32);
#pragma unroll
    for (int e = 0; e < 8; ++e) dl = fmaf((float)gf[ks][e], (float)of[e], dl);
  }
  dl = pair_sum(dl);  // D~: exact up to the rounding of the stored O; refined below
  float csum = 0.f;   // this lane's share of sum_j dS~_ij
  __syncthreads();  // O has been read: stage 1 may receive the second K/V block

  // One iteration: start the copy of block jb+1 into the other stage (last read before the previous
  // barrier), consume block jb from (Kb, Vb); the barrier at the end publishes the copied block.
  auto iteration = [&](int jb, const uint16_t *__restrict__ Kb, const uint16_t *__restrict__ Vb,
                       uint16_t *__restrict__ Kn, uint16_t *__restrict__ Vn) {
    if (jb < jb_hi) copy_block(Kn, Vn, jb + 1);  // workgroup-uniform
    else if (need_prev) copy_prev_rows(Vn);
    const int j0 = jbase + jb * kBS;
    if (wave_ok && j0 <= iw1 && j0 + kBS - 1 >= ss_min) {  // wave-uniform
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const int jl = j0 + sb * 32;
        if (jl > iw1 || jl + 31 < ss_min) continue;  // wave-uniform
        f32x16 s, dp;  // dP accumulates onto -D of this lane's query row
#pragma unroll
        for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = -dl; }
        // Fragment reads run kAhead k-steps ahead of the matrix instructions that use them, in this order
        // (the scheduling barriers keep it): left alone the compiler requests each pair of fragments right
        // before the pair of matrix instructions that uses it, and the wave waits out the LDS latency 8 times.
        x8 kf[kAhead], vf[kAhead];
#pragma unroll
        for (int ks = 0; ks < kAhead; ++ks) {
          kf[ks] = swz_read_row<E>(Kb + (ks >> 3) * kBlk, row_lane, ks & 7, sb * 32);
          vf[ks] = swz_read_row<E>(Vb + (ks >> 3) * kBlk, row_lane, ks & 7, sb * 32);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < kKs; ++ks) {
          s = mfma32(kf[ks % kAhead], qf[ks], s);     // S^T  = K Q^T
          dp = mfma32(vf[ks % kAhead], gf[ks], dp);   // dP^T - D = V dO^T - D
          if (ks + kAhead < kKs) {
            const int kn = ks + kAhead;
            kf[ks % kAhead] = swz_read_row<E>(Kb + (kn >> 3) * kBlk, row_lane, kn & 7, sb * 32);
            vf[ks % kAhead] = swz_read_row<E>(Vb + (kn >> 3) * kBlk, row_lane, kn & 7, sb * 32);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // K^T fragments of the sub-block's first 16 keys: requested here, in the registers the row
        // fragments have just left, so that they arrive during the vector work below
        x8 kt0[kCb], kt1[kCb];
#pragma unroll
        for (int cb = 0; cb < kCb; ++cb) kt0[cb] = swz_read_tr<E>(Kb + (cb >> 2) * kBlk, tr_lane, cb & 3, sb * 32);
        __builtin_amdgcn_sched_barrier(0);
        const bool interior = wave_full && jl >= ss_max && jl + 31 <= iw0;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, -lse2));  // P^T
        if (!interior) {  // one wave-uniform branch around all 16 tests (inside the loop above it stays 16 branches)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int j = jl + acc_row(v, half);
            if (j < ss_i || j > i_abs) s[v] = 0.f;
          }
        }
        x8 pf0, pf1;  // P^T as an operand, where the whole correction is kept
        if constexpr (kHasPk) {
          if (pk_on) { pf0 = pack_x8<E>(s, 0); pf1 = pack_x8<E>(s, 8); }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s[v] *= dp[v];  // dS~^T = P (dP - D~)
          csum += s[v];
        }
        // large score gradients are carried in two bf16 parts: a second pass with the residuals
        // (wave-uniform choice; rare on long examples)
        const bool split = needs_split<E>::value && __any(abs_max16(s) > kSplitS);
        const x8 df0 = pack_x8<E>(s, 0), df1 = pack_x8<E>(s, 8);
#pragma unroll
        for (int cb = 0; cb < kCb; ++cb) kt1[cb] = swz_read_tr<E>(Kb + (cb >> 2) * kBlk, tr_lane, cb & 3, sb * 32 + 16);
#pragma unroll
        for (int cb = 0; cb < kCb; ++cb) acc[cb] = mfma32(kt0[cb], df0, acc[cb]);  // dQ^T += K^T dS^T
#pragma unroll
        for (int cb = 0; cb < kCb; ++cb) acc[cb] = mfma32(kt1[cb], df1, acc[cb]);
        if constexpr (kHasPk) {
          if (pk_on) {
#pragma unroll
            for (int cb = 0; cb < kCb; ++cb) pk[cb] = mfma32(kt1[cb], pf1, mfma32(kt0[cb], pf0, pk[cb]));  // sum_j k_j P_ij
          }
        }
        if (split) {  // the K^T fragments are simply read again
          const x8 dr0 = pack_residual_x8<E>(s, 0, df0), dr1 = pack_residual_x8<E>(s, 8, df1);
#pragma unroll
          for (int cb = 0; cb < kCb; ++cb)
            acc[cb] = mfma32(swz_read_tr<E>(Kb + (cb >> 2) * kBlk, tr_lane, cb & 3, sb * 32), dr0, acc[cb]);
#pragma unroll
          for (int cb = 0; cb < kCb; ++cb)
            acc[cb] = mfma32(swz_read_tr<E>(Kb + (cb >> 2) * kBlk, tr_lane, cb & 3, sb * 32 + 16), dr1, acc[cb]);
        }
      }
    }
    if (jb < jb_hi) __syncthreads();  // workgroup-uniform; the last block's barrier follows the correction pass below
  };

  for (int jb = jb_lo; jb <= jb_hi; jb += 2) {  // bounds are workgroup-uniform: barriers stay aligned
    iteration(jb, K0, V0, K1, V1);
    if (jb + 1 <= jb_hi) iteration(jb + 1, K1, V1, K0, V0);
  }

  // Softmax rows sum to one, so sum_j P_ij (dP_ij - D_i) = 0 for the exact D_i = sum_j P_ij dP_ij.  The
  // row sum of dS~ is therefore D_i - D~_i, the error that the rounding of the stored O left in
  // D~ = dO . O: the dK/dV kernel gets D_i itself.
  const float c_row = pair_sum(csum);
  if (row_ok && half == 0) delta[(size_t)h * N + i_abs] = dl + c_row;
  // dQ was accumulated with D~: what is missing is -c_i sum_j P_ij k_j.  It matters where the
  // probabilities are large, i.e. for queries with a short context (it falls off as 1 / context^2).
  // Waves that hold queries with fewer than kNearCtx keys recompute P on the key sub-blocks from
  // kNearCtx before their first row on and add K^T (-c P)^T - on the last two key blocks only, which
  // are still in the stage memory (nothing was copied after them): no copy, no extra barrier - and,
  // where the example of the tile's first row began shortly before the tile, on the kNearCtx keys before
  // the tile (copy_prev_rows above: one copy under the last iteration and one barrier).  With 64 instead of
  // 32 the rows whose softmax peaks a few dozen keys back are covered too (dQ of a batch of 8..128-token
  // examples: 1.1e-2 -> 3.7e-3 max-abs) for 7 % of this kernel's time on such a batch, under 2 % elsewhere.
  if constexpr (kHasPk) {
    if (pk_on) {
#pragma unroll
      for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[cb][v] = fmaf(-c_row, pk[cb][v], acc[cb][v]);
    }
  }
  if (need_prev) {  // workgroup-uniform: the extra rows were requested an iteration ago
    wait_all_loads();
    __syncthreads();
  }
  if (!pk_on && wave_ok && ss_max > iw0 - kNearCtx) {  // wave-uniform
    const int j_first = max(ss_min, iw0 - kNearCtx);
    auto near_sub = [&](const uint16_t *Kb, int row0, int jl) {  // keys jl .. jl + 31 = rows row0 .. of the block at Kb
      f32x16 sc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < kKs; ++ks)
        sc = mfma32(swz_read_row<E>(Kb + (ks >> 3) * kBlk, row_lane, ks & 7, row0), qf[ks], sc);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int j = jl + acc_row(v, half);
        const float p = __builtin_amdgcn_exp2f(fmaf(sc[v], scale_log2, -lse2));
        sc[v] = (j < ss_i || j > i_abs) ? 0.f : -c_row * p;
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const x8 cf = pack_x8<E>(sc, 8 * s2);
#pragma unroll
        for (int cb = 0; cb < kCb; ++cb)
          acc[cb] = mfma32(swz_read_tr<E>(Kb + (cb >> 2) * kBlk, tr_lane, cb & 3, row0 + s2 * 16), cf, acc[cb]);
      }
    };
    if (need_prev && iw0 - kNearCtx < t0) {  // wave-uniform: this wave's keys begin before the tile
      const uint16_t *Kp = ((jb_hi - jb_lo) & 1) ? V0 : V1;
#pragma unroll 1
      for (int sb = (kBS - kNearCtx) / 32; sb < 2; ++sb) {
        const int jl = t0 - kBS + sb * 32;
        if (jl + 31 >= j_first) near_sub(Kp, sb * 32, jl);
      }
    }
#pragma unroll 1
    for (int jb = max(jb_lo, jb_hi - 1); jb <= jb_hi; ++jb) {
      const uint16_t *Kb = ((jb - jb_lo) & 1) ? K1 : K0;
#pragma unroll 1
      for (int sb = 0; sb < 2; ++sb) {
        const int jl = jbase + jb * kBS + sb * 32;
        if (jl > iw1 || jl + 31 < j_first) continue;  // wave-uniform
        near_sub(Kb, sb * 32, jl);
      }
    }
  }
  __syncthreads();  // every wave is done with the stages: the result staging below overlays them
  float *stage = (float *)lds + wave * kStageFloatsPerWave;
  store_transposed_tile<EOut, kCb>(acc, scale, stage, dQ, iw0, wave_ok ? iw1 - iw0 + 1 : 0, hq, h, d);
}

// ---------------------------------------------------------------------------------------------
// dK/dV with the two gradients on different waves.  Workgroup = 8 waves = (128-key tile, KV head);
// waves 0..3 ("V side") and 4..7 ("K side") each own 32 keys, wave w and w + 4 the same ones, and
// share a SIMD.  Per 32-query sub-block:
//   V side: S = Q K^T (on -LSE / scale), P = exp2, mask; leaves P (fp16) in LDS for its partner;
//           dV^T += dO^T P.
//   K side: dP = dO V^T (on -D); one sub-block later, with that P: dS = P * dP; dK^T += Q^T dS.
// Each wave holds one accumulator tile and one operand tile (about 200 registers), so two waves fit
// per SIMD and one wave's exp / convert / LDS work overlaps the other's matrix instructions.
// head_dim above 128 (kDh = 256): operand and accumulator tiles are twice as large, so a workgroup is
// 4 waves = (64-key tile, KV head), one wave per SIMD with 512 registers each; blocks are two
// 128-column halves, and the tile's own K and V rows pass through the memory of the second stage.
// Two shapes for head_dim <= 128, chosen on the device from the mean example length of the packed
// batch (both are launched; the workgroups of the one that does not apply leave at once):
//   large: 8 waves on a 128-key tile, one workgroup per CU: each streamed Q/dO block serves 128 keys
//          (examples of thousands of tokens: 6 % faster than the small shape);
//   small: 4 waves on a 64-key tile, two workgroups per CU that hide each other's prologue, epilogue
//          and barriers (examples of 8..128 tokens: 14 % faster), at twice the block copies per
//          matrix instruction.
constexpr int kDkdvSmallBelow = 1024;  // mean example length (tokens) below which the small shape runs
template <int kDh, bool kSmall> struct DkdvShape {
  static_assert(!(kSmall && kDh > 128), "head_dim above 128 has one shape");
  static constexpr int kKg = (kDh > 128 || kSmall) ? 2 : 4;  // key groups (of 32 keys) per workgroup
  static constexpr int kWgPerCu = kSmall ? 2 : 1;
  static constexpr int kWaves = 2 * kKg;                // V side + K side
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kKeys = 32 * kKg;                // keys per workgroup
  static constexpr int kSubTiles = VA_TILE / kKeys;     // workgroup tiles per schedule tile
};

__device__ __forceinline__ void lds_barrier() {  // LDS traffic of this wave done, then workgroup barrier
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// select: 0 = run; 1 = run only if the examples have kDkdvSmallBelow tokens or more on average; 2 =
// only if they have fewer (meta[0] is the number of examples, left there by the boundary scan).
template <class E, class EOut, int kDh, bool kSmall>
__global__ void __launch_bounds__((DkdvShape<kDh, kSmall>::kThreads), (DkdvShape<kDh, kSmall>::kWgPerCu))
dkdv_mfma_kernel(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ Q,
                  const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
                  const float *__restrict__ LSE, const float *__restrict__ delta, void *__restrict__ dK,
                  void *__restrict__ dV, const int32_t *__restrict__ seg_end,
                  const int32_t *__restrict__ kv_tile_order, const int32_t *__restrict__ meta, int select,
                  int N, int T, int tiles_per_row, int hq, int hkv, int d, float scale_log2, float scale) {
  if (select != 0 && (((long long)N < (long long)kDkdvSmallBelow * meta[0]) != (select == 2))) return;  // workgroup-uniform
  constexpr int kKs = kDh / 16, kCb = kDh / 32;
  constexpr int kHf = kDh > 128 ? 2 : 1;  // 128-column sub-blocks per block
  constexpr int kBlkT = kBlk * kHf;       // elements of one tensor's streamed block
  typedef DkdvShape<kDh, kSmall> Shape;
  constexpr int kKg = Shape::kKg, kWaves = Shape::kWaves, kKeys = Shape::kKeys, kSubTiles = Shape::kSubTiles;
  constexpr int kKvSub = kKeys * kD;      // elements of one sub-block of the tile's own K (or V) rows
  constexpr bool kKvInStage = kHf > 1 || kSmall;  // no room for a kv_tile of its own: the rows pass through stage 1
  typedef typename E::x8 x8;
  // two stages of {Q block, dO block (swizzled), -LSE / scale [64], -D [64]}; reused as the staging
  // area of the result stores
  constexpr int kStage = 2 * kBlkT + 4 * kBS;
  constexpr int kStagingElems = kWaves * kStageFloatsPerWave * 2;
  constexpr int kStagesElems = kStagingElems > 2 * kStage ? kStagingElems : 2 * kStage;
  static_assert(!kKvInStage || 2 * kHf * kKvSub <= kStage, "the tile's K and V rows must fit in one stage");
  // One LDS object for everything (with several, the compiler makes every LDS read after a block copy
  // wait until the copy has landed: it can tell copy destinations from read addresses by offset inside
  // one object only):
  //   stages: as above
  //   exch:   P hand-over, [key group][parity 2][part 2][lane 64] x 16 B
  //   kv_own: the tile's own K rows and V rows (swizzled like the streamed blocks), only used in the
  //           prologue: each wave takes its 32-row operand from here.  Going through LDS lets the rows
  //           arrive as whole 1 KB transfers; loading the per-lane fragments straight from HBM (32 rows x
  //           32 B per instruction) took 3 us per workgroup.
  constexpr int kExchElems = kKg * 2 * 2 * 64 * 8;
  constexpr int kKvOwnElems = kKvInStage ? 0 : 2 * kKvSub;
  __shared__ __attribute__((aligned(16))) uint16_t lds_all[kStagesElems + kExchElems + kKvOwnElems];
  uint16_t *const stages = lds_all;
  u32x4 *const exch = (u32x4 *)(lds_all + kStagesElems);
  uint16_t *const kv_own = lds_all + kStagesElems + kExchElems;

  const int lane = threadIdx.x & 63, wave = uniform(threadIdx.x >> 6);
  const int kg = wave % kKg;
  const bool k_side = wave >= kKg;
  const int l32 = lane & 31, half = lane >> 5;
  const int entry = uniform(kv_tile_order[blockIdx.x / (hkv * kSubTiles)]);
  const int tile = order_tile(entry);
  const int sub = (blockIdx.x / hkv) % kSubTiles;
  const int g = (blockIdx.x % hkv + head_rotation(entry)) % hkv;
  const int G = hq / hkv;
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;
  const int t0 = r * T + m * VA_TILE + sub * kKeys;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kKeys, row_end) - 1;
  const int ib_lo = t0 / kBS;

  const size_t row_bytes = (size_t)hq * d * 2;
  const size_t base_off = (size_t)ib_lo * kBS * row_bytes;
  const size_t total = (size_t)N * row_bytes;
  const buffer_t qbuf = make_buffer((const char *)Q + base_off, total - base_off);
  const buffer_t gbuf = make_buffer((const char *)dO + base_off, total - base_off);
  // HBM -> LDS copy of a 64-row block: 16 transfers of 1 KB (4 rows) per tensor and sub-block, shared
  // out over the waves (transfers of one wave are 4 kWaves rows apart: the same swizzle)
  const int dma_row = wave * 4 + (lane >> 4);
  const uint32_t dma_off = dma_lane_offset(lane, dma_row, row_bytes, 0, d);
  bool dma_ok[kHf];
#pragma unroll
  for (int hf = 0; hf < kHf; ++hf) dma_ok[hf] = dma_lane_ok(lane, dma_row, d - 128 * hf);
  const uint32_t blk_bytes = (uint32_t)(kBS * row_bytes);
  const uint32_t p_bytes = (uint32_t)(4 * kWaves * row_bytes);
  typedef __attribute__((address_space(3))) void *lds_void;
  const int stat_row = threadIdx.x & (kBS - 1);
  const bool stat_is_lse = (threadIdx.x & kBS) == 0;
  const float *stat_src = stat_is_lse ? LSE : delta;
  const float stat_mul = stat_is_lse ? -1.f / scale : -1.f;
  float rstat = 0.f;
  uint16_t *const S0 = stages, *const S1 = stages + kStage;
  auto copy_block = [&](uint16_t *dst, int hh, int ib) {
    {  // every thread loads (a load under a condition would be waited for at the end of the branch)
      const int i = min(ib * kBS + stat_row, N - 1);
      rstat = stat_src[(size_t)(g * G + hh) * N + i];
    }
    const uint32_t off = dma_off + (uint32_t)(ib - ib_lo) * blk_bytes + (uint32_t)((g * G + hh) * d * 2);
#pragma unroll
    for (int hf = 0; hf < kHf; ++hf)
#pragma unroll
      for (int p = 0; p < 16 / kWaves; ++p) {
        const uint32_t o = dma_ok[hf] ? off + p * p_bytes + hf * 256 : kPastEnd;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(qbuf, (lds_void)(dst + hf * kBlk + (kWaves * p + wave) * 512), 16, o, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(gbuf, (lds_void)(dst + kBlkT + hf * kBlk + (kWaves * p + wave) * 512), 16, o, 0, 0, 0);
      }
  };
  auto put_stats = [&](uint16_t *dst) {
    if (threadIdx.x < 2 * kBS) ((float *)(dst + 2 * kBlkT))[threadIdx.x] = rstat * stat_mul;
  };
  copy_block(S0, 0, ib_lo);  // needs nothing but the tile: in flight while the bounds arrive

  // Everything else the prologue needs depends on the tile only: all of it is requested before any
  // of it is looked at (a value made wave-uniform right after its load would hold the next load
  // back by a full memory round trip, four times in a row).
  uint16_t *const kv_tile = kKvInStage ? S1 : kv_own;  // K sub-blocks, then V sub-blocks
  const int jw0 = t0 + kg * 32;
  const int jw1 = min(jw0 + 31, t_last);
  const bool wave_ok = jw0 <= t_last;
  const bool wave_full = jw0 + 31 <= t_last;
  const int j_abs = jw0 + l32;
  const bool row_ok = j_abs <= t_last;
  const int j_ld = min(j_abs, t_last);
  const int se_last_v = seg_end[t_last];
  const int se_min_v = seg_end[min(jw0, t_last)];
  const int se_max_v = seg_end[jw1 < jw0 ? t_last : jw1];
  const int se_j_v = seg_end[j_ld];
  {  // K and V rows t0 .. t0 + kKeys - 1 of head g -> kv_tile: 4 transfers of 4 rows per wave, tensor and sub-block
    const size_t kv_row_bytes = (size_t)hkv * d * 2;
    const size_t kv_off = (size_t)t0 * kv_row_bytes, kv_total = (size_t)N * kv_row_bytes;
    const buffer_t kb = make_buffer((const char *)K + kv_off, kv_total - kv_off);
    const buffer_t vb = make_buffer((const char *)V + kv_off, kv_total - kv_off);
    const uint32_t o0 = dma_lane_offset(lane, dma_row, kv_row_bytes, g, d);
    const uint32_t step = (uint32_t)(4 * kWaves * kv_row_bytes);
#pragma unroll
    for (int hf = 0; hf < kHf; ++hf)
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const uint32_t o = dma_ok[hf] ? o0 + p * step + hf * 256 : kPastEnd;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(kb, (lds_void)(kv_tile + hf * kKvSub + (kWaves * p + wave) * 512), 16, o, 0, 0, kOnce);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(vb, (lds_void)(kv_tile + (kHf + hf) * kKvSub + (kWaves * p + wave) * 512), 16, o, 0, 0, kOnce);
      }
  }

  const int ib_hi = (uniform(se_last_v) - 1) / kBS;  // query blocks end with the example of the tile's last key
  const int nb = ib_hi - ib_lo + 1;
  const int n_it = nb * G;
  const int se_min = uniform(se_min_v), se_max = uniform(se_max_v);
  const int se_j = row_ok ? se_j_v : 0;  // queries j_abs <= i < se_j see key j_abs

  f32x16 acc[kCb];
#pragma unroll
  for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;

  const uint32_t row_lane = swz_row_lane_off(lane);
  uint32_t tr_lane[2];
  swz_tr_lane_off(lane, tr_lane);
  u32x4 *const ex = exch + kg * 256 + lane;  // + parity * 128 + part * 64

  x8 rf[kKs];  // this lane's key row: K (the V side computes S) or V (the K side computes dP); set below
  // Order of the streamed blocks.  One query head per KV head: ib_lo, ib_lo + 1, ... ib_hi; neighbouring
  // key tiles of an example, which run next to each other on one XCD, then follow each other two steps
  // apart and find the blocks in L2.  Grouped heads: block ib_lo (the tile's own first rows; needs no
  // bounds, so its copy is in flight while they arrive) for every head of the group, then blocks ib_hi,
  // ib_hi - 1, ... ib_lo + 1, each for every head: the key tiles of one example share ib_hi, so they
  // stream the same block at about the same time, whereas ascending they would run 2 G steps apart per
  // tile and the blocks would have left the L2 (measured traffic of the kernel with 5 query heads per KV
  // head and examples of thousands of tokens: 3.8 GB ascending, 2.9 GB this way; the same run time).
  int ib_cur = ib_lo, ib_nxt = ib_lo, hh_nxt = 0;
  // The K side runs one sub-block behind the V side: in step k the V side computes S(k), P(k) (left in
  // LDS) and dV(k), the K side computes dP(k) and, with the P(k-1) published by the previous barrier,
  // dS(k-1) and dK(k-1).  No wave waits for another inside a step; one barrier ends each step.  The
  // two sides run separate loops (same barriers, same block copies) so that each keeps only its own
  // values in registers.
  auto read_ty = [&](x8 (&ty)[2][kCb], const uint16_t *__restrict__ Ys, int row0) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int cb = 0; cb < kCb; ++cb) ty[s2][cb] = swz_read_tr<E>(Ys + (cb >> 2) * kBlk, tr_lane, cb & 3, row0 + s2 * 16);
  };
  auto first_product = [&](f32x16 &x, const uint16_t *__restrict__ Xs, const float *__restrict__ st, int row0) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 c = *(const f32x4 *)(st + row0 + q4 * 8 + half * 4);
#pragma unroll
      for (int b = 0; b < 4; ++b) x[q4 * 4 + b] = c[b];
    }
    // fragment reads run kAheadKv k-steps ahead of their matrix instructions (see kAhead)
    x8 ax[kAheadKv];
#pragma unroll
    for (int ks = 0; ks < kAheadKv; ++ks) ax[ks] = swz_read_row<E>(Xs + (ks >> 3) * kBlk, row_lane, ks & 7, row0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < kKs; ++ks) {
      x = mfma32(ax[ks % kAheadKv], rf[ks], x);  // S - LSE / scale, or dP - D
      if (ks + kAheadKv < kKs) {
        const int kn = ks + kAheadKv;
        ax[ks % kAheadKv] = swz_read_row<E>(Xs + (kn >> 3) * kBlk, row_lane, kn & 7, row0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // `split` (wave-uniform): x holds entries large enough for their bf16 rounding to matter; their
  // residuals go through the matrix pipe as a second operand (see kSplitP / kSplitS)
  auto second_product = [&](const f32x16 &x, const x8 (&ty)[2][kCb], bool split) {
    const x8 f0 = pack_x8<E>(x, 0), f1 = pack_x8<E>(x, 8);
#pragma unroll
    for (int cb = 0; cb < kCb; ++cb) acc[cb] = mfma32(ty[0][cb], f0, acc[cb]);  // dV^T += dO^T P, dK^T += Q^T dS
#pragma unroll
    for (int cb = 0; cb < kCb; ++cb) acc[cb] = mfma32(ty[1][cb], f1, acc[cb]);
    if (split) {
      const x8 r0 = pack_residual_x8<E>(x, 0, f0), r1 = pack_residual_x8<E>(x, 8, f1);
#pragma unroll
      for (int cb = 0; cb < kCb; ++cb) acc[cb] = mfma32(ty[0][cb], r0, acc[cb]);
#pragma unroll
      for (int cb = 0; cb < kCb; ++cb) acc[cb] = mfma32(ty[1][cb], r1, acc[cb]);
    }
  };
  auto v_step = [&](const uint16_t *__restrict__ cur, int il, int row0, int pw) {
    f32x16 x;
    x8 ty[2][kCb];
    first_product(x, cur, (const float *)(cur + 2 * kBlkT), row0);
    read_ty(ty, cur + kBlkT, row0);
#pragma unroll
    for (int v = 0; v < 16; ++v) x[v] = __builtin_amdgcn_exp2f(x[v] * scale_log2);  // P
    const bool interior = wave_full && il >= jw1 && il + 31 < se_min;
    if (!interior) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = il + acc_row(v, half);
        if (i < j_abs || i >= se_j) x[v] = 0.f;
      }
    }
    // P goes to the K side as fp16 whatever the inputs' type: probabilities lie in [0, 1], where fp16
    // keeps 11 significant bits (bf16: 8) down to 6e-5 and absolute 2^-25 below
    ex[pw * 128] = __builtin_bit_cast(u32x4, pack_x8<F16>(x, 0));
    ex[pw * 128 + 64] = __builtin_bit_cast(u32x4, pack_x8<F16>(x, 8));
    second_product(x, ty, needs_split<E>::value && __any(abs_max16(x) > kSplitP));
  };
  auto k_finish = [&](f32x16 &x, const x8 (&ty)[2][kCb], int pr) {  // dS = P (dP - D); dK
    const f16x8 p0 = as_x8<F16>(ex[pr * 128]), p1 = as_x8<F16>(ex[pr * 128 + 64]);
#pragma unroll
    for (int e = 0; e < 8; ++e) {  // written as fma(p, x, +0): one mixed-precision instruction instead of convert + multiply
      x[e] = __builtin_fmaf((float)p0[e], x[e], 0.f);
      x[8 + e] = __builtin_fmaf((float)p1[e], x[8 + e], 0.f);
    }
    second_product(x, ty, needs_split<E>::value && __any(abs_max16(x) > kSplitS));
  };
  bool more = false;
  auto begin_block = [&](int it, uint16_t *__restrict__ nxt) {  // returns the block's first query
    more = it + 1 < n_it;  // workgroup-uniform
    if (++hh_nxt == G) {  // all heads of the group have had this block
      hh_nxt = 0;
      ib_nxt = G == 1 ? ib_nxt + 1 : ib_nxt == ib_lo ? ib_hi : ib_nxt - 1;
    }
    if (more) copy_block(nxt, hh_nxt, ib_nxt);
    const int i0 = ib_cur * kBS;
    ib_cur = ib_nxt;
    return i0;
  };
  auto end_block = [&](uint16_t *__restrict__ nxt) {
    if (more) put_stats(nxt);
    wait_all_loads();
    lds_barrier();  // P published; next block published; every read of this stage is done
  };
  // wave-uniform and the same on both sides: does sub-block [il, il + 32) hold a pair of this wave?
  auto is_active = [&](int il) { return wave_ok && il + 31 >= jw0 && il < se_max; };
  auto v_iteration = [&](int it, const uint16_t *__restrict__ cur, uint16_t *__restrict__ nxt) {
    const int i0 = begin_block(it, nxt);
    if (is_active(i0)) v_step(cur, i0, 0, 0);
    lds_barrier();
    if (is_active(i0 + 32)) v_step(cur, i0 + 32, 32, 1);
    end_block(nxt);
  };
  f32x16 xa, xb;       // K side: dP - D of the two sub-blocks of a block, each waiting for its P
  x8 tyb[2][kCb];      // K side: Q^T fragments of sub-block b (its stage is overwritten before they are used)
  bool act_b = false;  // K side: sub-block b of the previous block is waiting for its P
  auto k_iteration = [&](int it, const uint16_t *__restrict__ cur, uint16_t *__restrict__ nxt) {
    const int i0 = begin_block(it, nxt);
    const float *st = (const float *)(cur + 2 * kBlkT) + kBS;
    const bool act0 = is_active(i0), act1 = is_active(i0 + 32);
    // step 2 it: dP of sub-block a; dS, dK of the previous block's b (P at parity 1)
    if (act0) first_product(xa, cur + kBlkT, st, 0);
    if (act_b) k_finish(xb, tyb, 1);
    lds_barrier();
    // step 2 it + 1: dP of sub-block b; dS, dK of a (P at parity 0)
    if (act1) {
      first_product(xb, cur + kBlkT, st, 32);
      read_ty(tyb, cur, 32);
    }
    if (act0) {
      x8 tya[2][kCb];
      read_ty(tya, cur, 0);
      k_finish(xa, tya, 0);
    }
    act_b = act1;
    end_block(nxt);
  };
  put_stats(S0);
  wait_all_loads();
  lds_barrier();
#pragma unroll
  for (int ks = 0; ks < kKs; ++ks)
    rf[ks] = swz_read_row<E>(kv_tile + ((k_side ? kHf : 0) + (ks >> 3)) * kKvSub, row_lane, ks & 7, kg * 32);
  if (kKvInStage) lds_barrier();  // every wave has its rows before stage 1 receives its first block
  if (!k_side) {
    for (int it = 0; it < n_it; it += 2) {  // bounds are workgroup-uniform: barriers stay aligned
      v_iteration(it, S0, S1);
      if (it + 1 < n_it) v_iteration(it + 1, S1, S0);
    }
  } else {
    for (int it = 0; it < n_it; it += 2) {
      k_iteration(it, S0, S1);
      if (it + 1 < n_it) k_iteration(it + 1, S1, S0);
    }
    if (act_b) k_finish(xb, tyb, 1);  // the last sub-block's dK
  }
  float *stage = (float *)stages + wave * kStageFloatsPerWave;
  const int nrows = wave_ok ? jw1 - jw0 + 1 : 0;
  if (k_side)
    store_transposed_tile<EOut, kCb>(acc, scale, stage, dK, jw0, nrows, hkv, g, d);
  else
    store_transposed_tile<EOut, kCb>(acc, 1.f, stage, dV, jw0, nrows, hkv, g, d);
}

}  // namespace

template <class E, class EOut, int kDh>
static void launch_bwd_t(const uint16_t *g, const uint16_t *q, const uint16_t *k, const uint16_t *v,
                         const uint16_t *o, const float *LSE, float *delta, void *dQ, void *dK, void *dV,
                         const va_segments &seg, int N, int T, int tiles_per_row, int hq, int hkv, int d,
                         float scale, unsigned gq, unsigned gkv, hipStream_t stream, unsigned stages) {
  const float scale_log2 = scale * kLog2e;
  if (stages & VA_STAGE_DQ)  // first: it also produces D for the dK/dV kernel
    dq_mfma_kernel<E, EOut, kDh><<<gq, 256, 0, stream>>>(g, q, k, v, o, LSE, delta, dQ, seg.seg_start,
                                                         seg.q_tile_order, N, T, tiles_per_row, hq, hkv, d,
                                                         scale_log2, scale);
  if (stages & VA_STAGE_DKDV) {
    typedef DkdvShape<kDh, false> Large;
    const unsigned g_large = gkv * (Large::kSubTiles / kSub);
    if constexpr (kDh <= 128) {
      typedef DkdvShape<kDh, true> Small;
      const unsigned g_small = gkv * (Small::kSubTiles / kSub);
      // nothing about the lengths is known on the host: both are launched and the device picks,
      // unless the caller's hint names the shape (select 0 = run unconditionally)
      const bool only_large = stages & VA_HINT_LONG_EXAMPLES, only_small = stages & VA_HINT_SHORT_EXAMPLES;
      if (!only_small)
        dkdv_mfma_kernel<E, EOut, kDh, false><<<g_large, Large::kThreads, 0, stream>>>(
            g, q, k, v, LSE, delta, dK, dV, seg.seg_end, seg.kv_tile_order, seg.meta, only_large ? 0 : 1, N, T,
            tiles_per_row, hq, hkv, d, scale_log2, scale);
      if (!only_large)
        dkdv_mfma_kernel<E, EOut, kDh, true><<<g_small, Small::kThreads, 0, stream>>>(
            g, q, k, v, LSE, delta, dK, dV, seg.seg_end, seg.kv_tile_order, seg.meta, only_small ? 0 : 2, N, T,
            tiles_per_row, hq, hkv, d, scale_log2, scale);
    } else {
      dkdv_mfma_kernel<E, EOut, kDh, false><<<g_large, Large::kThreads, 0, stream>>>(
          g, q, k, v, LSE, delta, dK, dV, seg.seg_end, seg.kv_tile_order, seg.meta, 0, N, T, tiles_per_row, hq, hkv, d,
          scale_log2, scale);
    }
  }
}

template <class E, class EOut, class... A>
static void launch_bwd_d(int d, A... a) {
  if (d <= 64) launch_bwd_t<E, EOut, 64>(a...);
  else if (d <= 96) launch_bwd_t<E, EOut, 96>(a...);
  else if (d <= 128) launch_bwd_t<E, EOut, 128>(a...);
  else launch_bwd_t<E, EOut, 256>(a...);
}

hipError_t launch_mfma_bwd(const void *dO, const void *Q, const void *K, const void *V, const void *O,
                           const float *LSE, float *delta, void *dQ, void *dK, void *dV,
                           va_dtype grad_dt, const va_segments &seg, int rows, int T, int hq,
                           int hkv, int d, va_dtype dt, float scale, hipStream_t stream, unsigned stages) {
  const int tiles_per_row = ceil_div(T, VA_TILE);
  const long long ntiles = (long long)rows * tiles_per_row * kSub;
  if (ntiles * hq > 0x7fffffffll) return hipErrorInvalidValue;
  const int N = rows * T;
  const uint16_t *q = (const uint16_t *)Q, *k = (const uint16_t *)K, *v = (const uint16_t *)V,
                 *g = (const uint16_t *)dO, *o = (const uint16_t *)O;
  const unsigned gq = (unsigned)(ntiles * hq), gkv = (unsigned)(ntiles * hkv);
  if (dt == VA_F16) {
    if (grad_dt == VA_F32)
      launch_bwd_d<F16, float>(d, g, q, k, v, o, LSE, delta, dQ, dK, dV, seg, N, T, tiles_per_row, hq, hkv, d, scale,
                               gq, gkv, stream, stages);
    else
      launch_bwd_d<F16, F16>(d, g, q, k, v, o, LSE, delta, dQ, dK, dV, seg, N, T, tiles_per_row, hq, hkv, d, scale,
                             gq, gkv, stream, stages);
  } else {
    if (grad_dt == VA_F32)
      launch_bwd_d<Bf16, float>(d, g, q, k, v, o, LSE, delta, dQ, dK, dV, seg, N, T, tiles_per_row, hq, hkv, d, scale,
                                gq, gkv, stream, stages);
    else
      launch_bwd_d<Bf16, Bf16>(d, g, q, k, v, o, LSE, delta, dQ, dK, dV, seg, N, T, tiles_per_row, hq, hkv, d, scale,
                               gq, gkv, stream, stages);
  }
  return hipGetLastError();
}


}  // namespace va
