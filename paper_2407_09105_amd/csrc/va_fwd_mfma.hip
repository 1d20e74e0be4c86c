// Forward kernel: causal attention inside each example of a packed stream, bf16 / fp16, head_dim <= 256.
//
// What it computes (see include/varlen_attn.h): O_i = softmax_j(scale q_i.k_j) v_j over the keys
// a <= j <= i of token i's own example, and LSE_i.  The example bound a = seg_start[i] comes from
// the position-id scan (paper, Section 3); keys of other examples are never attended (Table 1)
// and key blocks that lie wholly outside [seg_start[first row], last row] are never loaded.
//
// Shape of the computation: one workgroup (4 waves) per (128-token query tile, query head), three
// workgroups resident per CU so that one wave's softmax (vector ALU) overlaps another wave's
// MFMAs on the same SIMD.  Wave w owns query rows 32w..32w+31.  Key/value rows stream through
// LDS in blocks of 32, double-buffered (small stages and <= 168 registers keep three workgroups
// resident per CU: short tiles are chains of dependent memory latencies that only other
// workgroups can hide); the next block is copied HBM -> LDS by the load unit itself
// (buffer loads with an LDS destination: no registers, no LDS store instructions) while the
// current one is consumed.  Blocks are stored unpadded in the XOR-swizzled layout of
// va_mfma_common.h; since such a load writes 64 consecutive 16-byte chunks, the swizzle is applied
// on the global side (each lane fetches the chunk that belongs at its LDS position).  Scores are produced transposed, S^T = K Q^T, so a lane owns one query row
// (see va_mfma_common.h): the online-softmax row maximum and sum are per-lane values plus one
// exchange with lane ^ 32, and P^T leaves the accumulator registers directly as the B operand
// of O^T += V^T P^T.  V stays row-major in LDS; its transposed fragments come from the
// transposing LDS read.  The running maximum is only moved (and O rescaled) when a row's
// maximum grows by more than 2^kLazyLog2, which after the first block almost never happens.
#include "va_internal.h"
#include "va_mfma_common.h"

namespace va {
namespace {

constexpr int kBM = 128;          // query rows per workgroup
constexpr int kSub = VA_TILE / kBM;
constexpr int kBN = 32;           // key rows per LDS block
constexpr int kBlk = kBN * kD;    // elements of one swizzled [32][128] LDS block (8 KB)
constexpr int kStagingElems = 4 * kStageFloatsPerWave * 2;  // the result staging of four waves, in 16-bit units
constexpr float kLazyLog2 = 8.f;  // keep a stale row maximum while probabilities stay <= 2^8

// E: element type (Bf16 / F16); kDh: head_dim rounded up to 64, 96, 128 or 256 (k-steps and column
// blocks the kernel is unrolled for); d: the tensors' head_dim (a multiple of 8, <= kDh).  With
// kDh = 256 a block of K or V is two swizzled [32][128] sub-blocks (columns 0..127 and 128..255),
// the stages are twice as large and two workgroups share a CU instead of three.
template <class E, int kDh>
__global__ void __launch_bounds__(256, kDh > 128 ? 2 : 3)
fwd_mfma_kernel(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
                const uint16_t *__restrict__ V, uint16_t *__restrict__ O, float *__restrict__ LSE,
                const int32_t *__restrict__ seg_start, const int32_t *__restrict__ q_tile_order,
                int N, int T, int tiles_per_row, int hq, int hkv, int d, float scale_log2, float scale) {
  constexpr int kKs = kDh / 16, kCb = kDh / 32;
  constexpr int kHf = kDh > 128 ? 2 : 1;  // 128-column sub-blocks per block
  constexpr int kBlkT = kBlk * kHf;       // elements of one tensor's block
  typedef typename E::x8 x8;
  // stage 0 = {K, V} at lds[0 .. 2 kBlkT), stage 1 = {K, V} at lds[2 kBlkT .. 4 kBlkT)
  __shared__ __attribute__((aligned(16))) uint16_t lds[4 * kBlkT > kStagingElems ? 4 * kBlkT : kStagingElems];
  const int lane = threadIdx.x & 63, wave = uniform(threadIdx.x >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const uint32_t row_lane = swz_row_lane_off(lane);
  uint32_t tr_lane[2];
  swz_tr_lane_off(lane, tr_lane);

  // heavy schedule tiles first; the workgroups of one schedule tile (sub-tiles x heads) are adjacent
  const int wg = xcd_group_remap(blockIdx.x, hq / hkv, gridDim.x);
  const int entry = uniform(q_tile_order[wg / (hq * kSub)]);
  const int tile = order_tile(entry);
  const int sub = (wg / hq) % kSub;
  const int h = (wg % hq + head_rotation(entry) * (hq / hkv)) % hq;
  const int g = h / (hq / hkv);
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;  // one past the last token of this packed row
  const int t0 = r * T + m * VA_TILE + sub * kBM;
  if (t0 >= row_end) return;  // workgroup-uniform: the schedule tile is ragged
  const int t_last = min(t0 + kBM, row_end) - 1;
  // Everything the prologue needs depends on the tile only: all of it is requested before any of it
  // is looked at (a value made wave-uniform right after its load would hold the next load back by
  // a full memory round trip, several times in a row).
  const int iw0 = t0 + wave * 32;  // this wave's rows (wave-uniform) and this lane's query row
  const int iw1 = min(iw0 + 31, t_last);
  const bool wave_ok = iw0 <= t_last;
  const bool wave_full = iw0 + 31 <= t_last;
  const int i_abs = iw0 + l32;
  const bool row_ok = i_abs <= t_last;
  const int i_ld = min(i_abs, t_last);  // clamped: loads stay in bounds, results of dead rows are dropped
  const int ss_t0_v = seg_start[t0];
  const int ss_min_v = seg_start[min(iw0, t_last)];
  const int ss_max_v = seg_start[iw1 < iw0 ? t_last : iw1];
  const int ss_i_v = seg_start[i_ld];
  x8 qf[kKs];  // B operands of S^T = K Q^T; k-steps of 16
  load_row_fragments<E, kKs>(Q + ((size_t)i_ld * hq + h) * d, d, half, qf);
  const int jb_lo = uniform(ss_t0_v) / kBN, jb_hi = t_last / kBN;  // key blocks of this tile
  const int ss_min = uniform(ss_min_v), ss_max = uniform(ss_max_v);
  const int ss_i = row_ok ? ss_i_v : 0x7fffffff;

  f32x16 o_acc[kCb];
#pragma unroll
  for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) o_acc[cb][v] = 0.f;
  float m_ref = -INFINITY;  // reference maximum the stored probabilities are relative to (raw scores)
  float l_run = 0.f;        // this lane's share of the running row sum, relative to m_ref
  float m_thr = -INFINITY;  // m_ref + kLazyLog2 / scale_log2: a block maximum above it moves m_ref
  float mneg = 0.f;         // -m_ref * scale_log2; 0 while m_ref = -inf (nothing unmasked yet), so that exp2(-inf - 0) = 0
  const float lazy_raw = kLazyLog2 / scale_log2;

  // K/V block loads: buffer descriptors based at the workgroup's first key row
  const size_t row_bytes = (size_t)hkv * d * 2;
  const size_t base_off = (size_t)jb_lo * kBN * row_bytes;
  const size_t total = (size_t)N * row_bytes;
  const buffer_t kbuf = make_buffer((const char *)K + base_off, total - base_off);
  const buffer_t vbuf = make_buffer((const char *)V + base_off, total - base_off);
  // HBM -> LDS copy of a kBN-row block: kBN / 16 load instructions per wave and tensor, each writing
  // 1 KB (4 rows) at wave-uniform LDS address (4 p + wave) KB; lane L lands at row 16 p + 4 wave + L / 16,
  // chunk position L % 16, and therefore fetches global chunk (L % 16) ^ swz(row) of that row.
  const int dma_row = wave * 4 + (lane >> 4);
  const uint32_t dma_off = dma_lane_offset(lane, dma_row, row_bytes, g, d);
  bool dma_ok[kHf];  // the same for every transfer of this lane into a sub-block (rows 16 apart)
#pragma unroll
  for (int hf = 0; hf < kHf; ++hf) dma_ok[hf] = dma_lane_ok(lane, dma_row, d - 128 * hf);
  const uint32_t blk_bytes = (uint32_t)(kBN * row_bytes);
  const uint32_t p_bytes = (uint32_t)(16 * row_bytes);
  typedef __attribute__((address_space(3))) void *lds_void;
  auto copy_block = [&](uint16_t *Kd, uint16_t *Vd, int jb) {  // rows past the tensor arrive as zeros
    const uint32_t off = dma_off + (uint32_t)(jb - jb_lo) * blk_bytes;
#pragma unroll
    for (int hf = 0; hf < kHf; ++hf)
#pragma unroll
      for (int p = 0; p < kBN / 16; ++p) {
        const uint32_t o = dma_ok[hf] ? off + p * p_bytes + hf * 256 : kPastEnd;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(kbuf, (lds_void)(Kd + hf * kBlk + (4 * p + wave) * 512), 16, o, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(vbuf, (lds_void)(Vd + hf * kBlk + (4 * p + wave) * 512), 16, o, 0, 0, 0);
      }
  };

  // One iteration: start the copy of block jb+1 into the other stage (last read before the previous
  // barrier), consume block jb from (Kb, Vb); the barrier at the end publishes the copied block.
  auto iteration = [&](int jb, const uint16_t *__restrict__ Kb, const uint16_t *__restrict__ Vb,
                       uint16_t *__restrict__ Kn, uint16_t *__restrict__ Vn) {
    if (jb < jb_hi) copy_block(Kn, Vn, jb + 1);  // workgroup-uniform
    const int j0 = jb * kBN;
    if (wave_ok && j0 <= iw1 && j0 + kBN - 1 >= ss_min) {  // wave-uniform
#pragma unroll
      for (int sb = 0; sb < kBN / 32; ++sb) {
        const int jl = j0 + sb * 32;
        if (jl > iw1 || jl + 31 < ss_min) continue;  // wave-uniform: sub-block outside this wave's keys
        // ---- S^T = K Q^T ----
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < kKs; ++ks) s = mfma32(swz_read_row<E>(Kb + (ks >> 3) * kBlk, row_lane, ks & 7, sb * 32), qf[ks], s);
        const bool interior = wave_full && jl >= ss_max && jl + 31 <= iw0;
        if (!interior) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int j = jl + acc_row(v, half);
            if (j < ss_i || j > i_abs) s[v] = -INFINITY;
          }
        }
        // ---- online softmax with a lazily moved reference maximum ----
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int v = 2; v < 16; v += 2) mx = fmaxf(fmaxf(mx, s[v]), s[v + 1]);
        mx = pair_max(mx);
        if (__any(mx > m_thr)) {  // rare after the first block
          const float m_new = fmaxf(m_ref, mx);
          const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((m_ref - m_new) * scale_log2);
          l_run *= alpha;
#pragma unroll
          for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o_acc[cb][v] *= alpha;
          m_ref = m_new;
          m_thr = m_new + lazy_raw;
          mneg = (m_new == -INFINITY) ? 0.f : -m_new * scale_log2;
        }
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, mneg));
          s[v] = p;
          psum += p;
        }
        l_run += psum;
        // ---- O^T += V^T P^T ----
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const x8 pf = pack_x8<E>(s, 8 * s2);
#pragma unroll
          for (int cb = 0; cb < kCb; ++cb)
            o_acc[cb] = mfma32(swz_read_tr<E>(Vb + (cb >> 2) * kBlk, tr_lane, cb & 3, sb * 32 + s2 * 16), pf, o_acc[cb]);
        }
      }
    }
    __syncthreads();
  };

  uint16_t *K0 = lds, *V0 = lds + kBlkT, *K1 = lds + 2 * kBlkT, *V1 = lds + 3 * kBlkT;
  copy_block(K0, V0, jb_lo);
  wait_all_loads();  // Q fragments too: inside the loop only block copies are in flight
  __syncthreads();
  for (int jb = jb_lo; jb <= jb_hi; jb += 2) {  // bounds are workgroup-uniform: barriers stay aligned
    iteration(jb, K0, V0, K1, V1);
    if (jb + 1 <= jb_hi) iteration(jb + 1, K1, V1, K0, V0);
  }

  // ---- epilogue: normalise, stage O through LDS, coalesced stores ----
  const float l_tot = pair_sum(l_run);
  const float inv = row_ok ? 1.f / l_tot : 0.f;
  if (row_ok && half == 0) LSE[(size_t)h * N + i_abs] = m_ref * scale + __logf(l_tot);
  float *stage = (float *)lds + wave * kStageFloatsPerWave;
  store_transposed_tile<E, kCb>(o_acc, inv, stage, O, iw0, wave_ok ? iw1 - iw0 + 1 : 0, hq, h, d);
}

}  // namespace

template <class E>
static void launch_fwd_e(const void *Q, const void *K, const void *V, void *O, float *LSE, const va_segments &seg,
                         int rows, int T, int hq, int hkv, int d, float scale, unsigned nwg, hipStream_t stream) {
  const int tiles_per_row = ceil_div(T, VA_TILE);
  const float scale_log2 = scale * 1.4426950408889634f;
  const uint16_t *q = (const uint16_t *)Q, *k = (const uint16_t *)K, *v = (const uint16_t *)V;
#define VA_LAUNCH_FWD(DH)                                                                             \
  fwd_mfma_kernel<E, DH><<<nwg, 256, 0, stream>>>(q, k, v, (uint16_t *)O, LSE, seg.seg_start,          \
                                                  seg.q_tile_order, rows * T, T, tiles_per_row, hq,   \
                                                  hkv, d, scale_log2, scale)
  if (d <= 64) VA_LAUNCH_FWD(64);
  else if (d <= 96) VA_LAUNCH_FWD(96);
  else if (d <= 128) VA_LAUNCH_FWD(128);
  else VA_LAUNCH_FWD(256);
#undef VA_LAUNCH_FWD
}

hipError_t launch_mfma_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                           const va_segments &seg, int rows, int T, int hq, int hkv, int d, va_dtype dt,
                           float scale, hipStream_t stream) {
  const int tiles_per_row = ceil_div(T, VA_TILE);
  const long long nwg = (long long)rows * tiles_per_row * kSub * hq;
  if (nwg <= 0 || nwg > 0x7fffffffll) return hipErrorInvalidValue;
  if (dt == VA_F16)
    launch_fwd_e<F16>(Q, K, V, O, LSE, seg, rows, T, hq, hkv, d, scale, (unsigned)nwg, stream);
  else
    launch_fwd_e<Bf16>(Q, K, V, O, LSE, seg, rows, T, hq, hkv, d, scale, (unsigned)nwg, stream);
  return hipGetLastError();
}


}  // namespace va
