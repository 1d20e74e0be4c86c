// Forward kernel: causal attention inside each example of a packed stream, bf16, head_dim 128.
//
// What it computes (see include/varlen_attn.h): O_i = softmax_j(scale q_i.k_j) v_j over the keys
// a <= j <= i of token i's own example, and LSE_i.  The example bound a = seg_start[i] comes from
// the position-id scan (paper, Section 3); keys of other examples are never attended (Table 1)
// and key blocks that lie wholly outside [seg_start[first row], last row] are never loaded.
//
// Shape of the computation: one workgroup (4 waves) per (128-token query tile, query head); wave
// w owns query rows 32w..32w+31.  Key/value rows stream through LDS in blocks of 64.  Scores are
// produced transposed, S^T = K Q^T, so a lane owns one query row (see va_mfma_common.h): the
// online-softmax row maximum and sum are per-lane values plus one exchange with lane ^ 32, and
// P^T leaves the accumulator registers directly as the B operand of O^T += V^T P^T.
#include "va_internal.h"
#include "va_mfma_common.h"

namespace va {
namespace {

constexpr int kBM = 128;          // query rows per workgroup
constexpr int kBN = 64;           // key rows per LDS block
constexpr int kKS = kD + 8;       // LDS row stride of the K block (elements): 272 B
constexpr int kVS = kBN + 8;      // LDS row stride of the transposed V block: 144 B
constexpr int kLdsK = kBN * kKS;  // elements
constexpr int kLdsV = kD * kVS;

__global__ void __launch_bounds__(256, 2)
fwd_mfma_kernel(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
                const uint16_t *__restrict__ V, uint16_t *__restrict__ O, float *__restrict__ LSE,
                const int32_t *__restrict__ seg_start, const int32_t *__restrict__ q_tile_order,
                int N, int T, int tiles_per_row, int hq, int hkv, float scale_log2, float scale) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[kLdsK + kLdsV];
  static_assert((kLdsK + kLdsV) * 2 >= 4 * kStageFloatsPerWave * 4, "staging must fit in the K/V buffers");
  uint16_t *Ks = lds, *Vt = lds + kLdsK;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, half = lane >> 5;

  // heavy tiles first; the heads of one tile are adjacent workgroups
  const int tile = q_tile_order[blockIdx.x / hq];
  const int h = blockIdx.x % hq;
  const int g = h / (hq / hkv);
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int row_end = (r + 1) * T;                     // one past the last token of this packed row
  const int t0 = r * T + m * kBM;                      // first token of the tile
  const int t_last = min(t0 + kBM, row_end) - 1;       // last valid token of the tile

  // this lane's query row
  const int i_abs = t0 + wave * 32 + l32;
  const bool row_ok = i_abs <= t_last;
  const int ss_i = row_ok ? seg_start[i_abs] : 0x7fffffff;
  // this wave's row range (wave-uniform)
  const int iw0 = t0 + wave * 32;
  const int iw1 = min(iw0 + 31, t_last);
  const bool wave_ok = iw0 <= t_last;
  const int ss_min = wave_ok ? seg_start[iw0] : 0;
  const int ss_max = wave_ok ? seg_start[iw1] : 0;

  // Q fragment: B operand of S^T = K Q^T; 8 k-steps of 16
  bf16x8 qf[8];
  {
    const uint16_t *qp = Q + ((size_t)(row_ok ? i_abs : t0) * hq + h) * kD + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = as_bf16x8(ldg16(qp + ks * 16, row_ok));
  }

  f32x16 o_acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) o_acc[cb][v] = 0.f;
  float m_run = -INFINITY;  // running row maximum (raw scores)
  float l_run = 0.f;        // this lane's share of the running row sum

  const int jb_lo = seg_start[t0] / kBN, jb_hi = t_last / kBN;
  for (int jb = jb_lo; jb <= jb_hi; ++jb) {
    const int j0 = jb * kBN;
    __syncthreads();  // previous block fully consumed
    load_rows_to_lds(K, j0, N, hkv, g, Ks, kKS);
    load_rows_to_lds_transposed(V, j0, N, hkv, g, Vt, kVS);
    __syncthreads();

    if (!wave_ok || j0 > iw1 || j0 + kBN - 1 < ss_min) continue;  // wave-uniform

    // ---- S^T = K Q^T for the two 32-key sub-blocks ----
    f32x16 s[2];
    bool sub_on[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      const int jl = j0 + sb * 32;
      sub_on[sb] = !(jl > iw1 || jl + 31 < ss_min);
#pragma unroll
      for (int v = 0; v < 16; ++v) s[sb][v] = 0.f;
      if (sub_on[sb]) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          bf16x8 kf = as_bf16x8(*(const u32x4 *)(Ks + (sb * 32 + l32) * kKS + ks * 16 + half * 8));
          s[sb] = mfma32(kf, qf[ks], s[sb]);
        }
        const bool need_mask = !(jl >= ss_max && jl + 31 <= iw0);
        if (need_mask) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int j = jl + acc_row(v, half);
            if (j < ss_i || j > i_abs) s[sb][v] = -INFINITY;
          }
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[sb][v] = -INFINITY;
      }
    }

    // ---- online softmax (lane owns a row; partner lane ^ 32 holds the other keys) ----
    float mx = -INFINITY;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[sb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2);
    const float mneg = -m_use * scale_log2;
    float psum = 0.f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[sb][v], scale_log2, mneg));
        s[sb][v] = p;
        psum += p;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[cb][v] *= alpha;
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      if (!sub_on[sb]) continue;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 pf = pack_bf16x8(s[sb], 8 * s2);
        const int kstep = sb * 2 + s2;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
          bf16x8 vf = as_bf16x8(*(const u32x4 *)(Vt + (cb * 32 + l32) * kVS + kstep * 16 + half * 8));
          o_acc[cb] = mfma32(vf, pf, o_acc[cb]);
        }
      }
    }
  }

  // ---- epilogue: normalise, stage O through LDS, coalesced stores ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = row_ok ? 1.f / l_tot : 0.f;
  if (row_ok && half == 0) LSE[(size_t)h * N + i_abs] = m_run * scale + __logf(l_tot);

  float *stage = (float *)lds + wave * kStageFloatsPerWave;
  store_transposed_tile<false>(o_acc, inv, stage, O, iw0, wave_ok ? iw1 - iw0 + 1 : 0, hq, h);
}

}  // namespace

hipError_t launch_mfma_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                           const va_segments &seg, int rows, int T, int hq, int hkv, float scale,
                           hipStream_t stream) {
  const int tiles_per_row = ceil_div(T, kBM);
  const long long nwg = (long long)rows * tiles_per_row * hq;
  if (nwg <= 0 || nwg > 0x7fffffffll) return hipErrorInvalidValue;
  const float scale_log2 = scale * 1.4426950408889634f;
  fwd_mfma_kernel<<<(unsigned)nwg, 256, 0, stream>>>((const uint16_t *)Q, (const uint16_t *)K,
                                                     (const uint16_t *)V, (uint16_t *)O, LSE,
                                                     seg.seg_start, seg.q_tile_order, rows * T, T,
                                                     tiles_per_row, hq, hkv, scale_log2, scale);
  return hipGetLastError();
}

}  // namespace va
