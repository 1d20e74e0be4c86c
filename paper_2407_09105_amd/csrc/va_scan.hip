// Boundary scan: position_ids -> cu_seqlens, per-token example ids / bounds, tile schedule.
//
// Paper, Section 3: the attention wrapper gets position_ids and derives cu_seq_len from
// them; Section 3.1: ids restart at 0 at each example.  A token starts an example iff it
// is the first of its row or its id is 0.  Integer work only, exact.
//
// Three passes over chunks of kScanChunk tokens (no cross-workgroup waiting):
//   1. per-chunk aggregates: number of starts, last start, first start
//   2. one workgroup scans the aggregates into per-chunk carries
//   3. per-chunk final scan with carries -> seg_id, seg_start, seg_end, cu_seqlens, max_seqlen
// then the tile schedule: a cost per query tile / key tile and a rank sort (heaviest first).
#include "va_internal.h"

namespace va {
namespace {

constexpr int kPerThread = kScanChunk / kScanThreads;  // 8 consecutive tokens per thread

template <typename IdT>
__device__ __forceinline__ bool is_start(const IdT *pos, int t, int T) {
  return (t % T == 0) || (pos[t] == 0);
}

// ---- block-wide scans over kScanThreads values (LDS, Hillis-Steele per wave + wave carries) ----

__device__ __forceinline__ int wave_incl_add(int x) {
  const int lane = threadIdx.x & 63;
  for (int o = 1; o < 64; o <<= 1) {
    int y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  return x;
}
__device__ __forceinline__ int wave_incl_max(int x) {
  const int lane = threadIdx.x & 63;
  for (int o = 1; o < 64; o <<= 1) {
    int y = __shfl_up(x, o, 64);
    if (lane >= o) x = max(x, y);
  }
  return x;
}
// suffix (right-to-left) inclusive min
__device__ __forceinline__ int wave_suffix_min(int x) {
  const int lane = threadIdx.x & 63;
  for (int o = 1; o < 64; o <<= 1) {
    int y = __shfl_down(x, o, 64);
    if (lane + o < 64) x = min(x, y);
  }
  return x;
}

struct ChunkAgg { int count, last, first; };

// pass 1
template <typename IdT>
__global__ void __launch_bounds__(kScanThreads)
scan_aggregate_kernel(const IdT *__restrict__ pos, int N, int T, int32_t *__restrict__ agg) {
  __shared__ int s_cnt[kScanThreads / 64], s_last[kScanThreads / 64], s_first[kScanThreads / 64];
  const int base = blockIdx.x * kScanChunk + threadIdx.x * kPerThread;
  int cnt = 0, last = -1, first = N;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    if (t < N && is_start(pos, t, T)) {
      ++cnt;
      last = t;
      first = min(first, t);
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    cnt += __shfl_xor(cnt, o, 64);
    last = max(last, __shfl_xor(last, o, 64));
    first = min(first, __shfl_xor(first, o, 64));
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_cnt[w] = cnt; s_last[w] = last; s_first[w] = first; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < kScanThreads / 64; ++i) {
      cnt += s_cnt[i]; last = max(last, s_last[i]); first = min(first, s_first[i]);
    }
    agg[3 * blockIdx.x + 0] = cnt;
    agg[3 * blockIdx.x + 1] = last;
    agg[3 * blockIdx.x + 2] = first;
  }
}

// pass 2: carries[3*b] = starts before chunk b, [3*b+1] = last start before it, [3*b+2] = first
// start after it (N if none).  Also meta[0] = n, meta[1] = 0 (max_seqlen accumulator), cu[n] = N.
__global__ void __launch_bounds__(64)
scan_carry_kernel(const int32_t *__restrict__ agg, int nchunks, int N, int32_t *__restrict__ carry,
                  int32_t *__restrict__ meta, int32_t *__restrict__ cu) {
  const int lane = threadIdx.x;
  int run_cnt = 0, run_last = -1;
  for (int b0 = 0; b0 < nchunks; b0 += 64) {
    const int b = b0 + lane;
    int c = 0, l = -1;
    if (b < nchunks) { c = agg[3 * b]; l = agg[3 * b + 1]; }
    const int ic = wave_incl_add(c);
    const int il = wave_incl_max(l);
    int ec = __shfl_up(ic, 1, 64), el = __shfl_up(il, 1, 64);
    if (lane == 0) { ec = 0; el = -1; }
    if (b < nchunks) {
      carry[3 * b] = run_cnt + ec;
      carry[3 * b + 1] = max(run_last, el);
    }
    run_cnt += __shfl(ic, 63, 64);
    run_last = max(run_last, __shfl(il, 63, 64));
  }
  int run_first = N;
  for (int b0 = ((nchunks - 1) / 64) * 64; b0 >= 0; b0 -= 64) {
    const int b = b0 + lane;
    int f = N;
    if (b < nchunks) f = agg[3 * b + 2];
    const int sf = wave_suffix_min(f);
    int ef = __shfl_down(sf, 1, 64);
    if (lane == 63) ef = N;
    if (b < nchunks) carry[3 * b + 2] = min(run_first, ef);
    run_first = min(run_first, __shfl(sf, 0, 64));
  }
  if (lane == 0) {
    meta[0] = run_cnt;
    meta[1] = 0;
    for (int i = 2; i < 8; ++i) meta[i] = 0;
    cu[run_cnt] = N;
  }
}

// pass 3
template <typename IdT>
__global__ void __launch_bounds__(kScanThreads)
scan_finalize_kernel(const IdT *__restrict__ pos, int N, int T, const int32_t *__restrict__ carry,
                     int32_t *__restrict__ cu, int32_t *__restrict__ seg_id,
                     int32_t *__restrict__ seg_start, int32_t *__restrict__ seg_end,
                     int32_t *__restrict__ meta) {
  __shared__ int s_cnt[kScanThreads / 64], s_last[kScanThreads / 64], s_first[kScanThreads / 64];
  const int base = blockIdx.x * kScanChunk + threadIdx.x * kPerThread;
  bool flag[kPerThread];
  int cnt = 0, last = -1, first = N;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    flag[e] = (t < N) && is_start(pos, t, T);
    if (flag[e]) { ++cnt; last = t; first = min(first, t); }
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int icnt = wave_incl_add(cnt), ilast = wave_incl_max(last), sfirst = wave_suffix_min(first);
  if (lane == 63) { s_cnt[w] = icnt; s_last[w] = ilast; }
  if (lane == 0) s_first[w] = sfirst;
  __syncthreads();
  // exclusive values for this thread: wave-exclusive + earlier waves + chunk carry
  int ecnt = __shfl_up(icnt, 1, 64), elast = __shfl_up(ilast, 1, 64), efirst = __shfl_down(sfirst, 1, 64);
  if (lane == 0) { ecnt = 0; elast = -1; }
  if (lane == 63) efirst = N;
  for (int i = 0; i < w; ++i) { ecnt += s_cnt[i]; elast = max(elast, s_last[i]); }
  for (int i = w + 1; i < kScanThreads / 64; ++i) efirst = min(efirst, s_first[i]);
  ecnt += carry[3 * blockIdx.x];
  elast = max(elast, carry[3 * blockIdx.x + 1]);
  efirst = min(efirst, carry[3 * blockIdx.x + 2]);
  // next start strictly after each of this thread's tokens (right to left)
  int nxt[kPerThread];
  int run = efirst;
#pragma unroll
  for (int e = kPerThread - 1; e >= 0; --e) {
    nxt[e] = run;
    if (flag[e]) run = base + e;
  }
  int c = ecnt, l = elast, longest = 0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    if (t >= N) break;
    if (flag[e]) {
      cu[c] = t;
      ++c;
      l = t;
      longest = max(longest, nxt[e] - t);
    }
    seg_id[t] = c - 1;
    seg_start[t] = l;
    seg_end[t] = nxt[e];
  }
  for (int o = 32; o > 0; o >>= 1) longest = max(longest, __shfl_xor(longest, o, 64));
  if (lane == 0 && longest > 0) atomicMax(&meta[1], longest);
}

// ---- tile schedule -------------------------------------------------------------------------
// Query tile m of row r covers tokens [r*T + m*kTile, min(r*T + (m+1)*kTile, (r+1)*T)).
// Its keys run from seg_start[first token] to its last token: cost = number of 64-key blocks.
// Key tile (same token range): its queries run from its first token to seg_end[last token]:
// cost = number of 64-query blocks.  Every tile has cost >= 1 (the diagonal is never masked).
__global__ void __launch_bounds__(256)
tile_cost_kernel(const int32_t *__restrict__ seg_start, const int32_t *__restrict__ seg_end, int T,
                 int tiles_per_row, int ntiles, int32_t *__restrict__ cost_q,
                 int32_t *__restrict__ cost_kv) {
  const int tile = blockIdx.x * blockDim.x + threadIdx.x;
  if (tile >= ntiles) return;
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int t0 = r * T + m * kTile;
  const int t1 = min(t0 + kTile, (r + 1) * T) - 1;  // last token of the tile
  cost_q[tile] = (t1 >> 6) - (seg_start[t0] >> 6) + 1;
  cost_kv[tile] = ((seg_end[t1] - 1) >> 6) - (t0 >> 6) + 1;
}

// order[rank] = tile, rank = number of tiles that are heavier (ties: lower index first)
__global__ void __launch_bounds__(256)
tile_rank_kernel(const int32_t *__restrict__ cost_q, const int32_t *__restrict__ cost_kv, int ntiles,
                 int32_t *__restrict__ order_q, int32_t *__restrict__ order_kv) {
  __shared__ int s_q[256], s_kv[256];
  const int tile = blockIdx.x * blockDim.x + threadIdx.x;
  const int cq = tile < ntiles ? cost_q[tile] : 0, ckv = tile < ntiles ? cost_kv[tile] : 0;
  int rq = 0, rkv = 0;
  for (int b0 = 0; b0 < ntiles; b0 += 256) {
    const int o = b0 + threadIdx.x;
    s_q[threadIdx.x] = o < ntiles ? cost_q[o] : -1;
    s_kv[threadIdx.x] = o < ntiles ? cost_kv[o] : -1;
    __syncthreads();
    const int lim = min(256, ntiles - b0);
    for (int i = 0; i < lim; ++i) {
      const int other = b0 + i;
      rq += (s_q[i] > cq) || (s_q[i] == cq && other < tile);
      rkv += (s_kv[i] > ckv) || (s_kv[i] == ckv && other < tile);
    }
    __syncthreads();
  }
  if (tile < ntiles) { order_q[rq] = tile; order_kv[rkv] = tile; }
}

// ---- one-workgroup path for short streams ------------------------------------------------------
// Everything above in a single launch: 1024 threads scan up to kSmallMax tokens in passes of 8192
// (8 consecutive tokens per thread), then compute tile costs and ranks.  Launch latency, not
// bandwidth, bounds the scan at these sizes.
constexpr int kSmallThreads = 1024;
constexpr int kSmallPass = kSmallThreads * kPerThread;  // 8192 tokens
constexpr int kSmallMaxPasses = 4;
constexpr int kSmallMax = kSmallPass * kSmallMaxPasses;  // 32768 tokens
constexpr int kSmallMaxTiles = kSmallMax / kTile * 8;    // rows may end in ragged tiles

template <typename IdT>
__global__ void __launch_bounds__(kSmallThreads)
pack_small_kernel(const IdT *__restrict__ pos, int N, int T, int tiles_per_row, int ntiles,
                  int32_t *__restrict__ cu, int32_t *__restrict__ seg_id, int32_t *__restrict__ seg_start,
                  int32_t *__restrict__ seg_end, int32_t *__restrict__ meta,
                  int32_t *__restrict__ order_q, int32_t *__restrict__ order_kv) {
  constexpr int kWaves = kSmallThreads / 64;
  __shared__ int s_cnt[kWaves], s_last[kWaves], s_first[kWaves];
  __shared__ int p_cnt[kSmallMaxPasses], p_last[kSmallMaxPasses], p_first[kSmallMaxPasses];
  __shared__ int s_longest[kWaves];
  __shared__ int s_cq[kSmallMaxTiles], s_ckv[kSmallMaxTiles];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int npass = (N + kSmallPass - 1) / kSmallPass;

  // pass aggregates
  for (int ps = 0; ps < npass; ++ps) {
    const int base = ps * kSmallPass + threadIdx.x * kPerThread;
    int cnt = 0, last = -1, first = N;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      const int t = base + e;
      if (t < N && is_start(pos, t, T)) { ++cnt; last = t; first = min(first, t); }
    }
    for (int o = 32; o > 0; o >>= 1) {
      cnt += __shfl_xor(cnt, o, 64);
      last = max(last, __shfl_xor(last, o, 64));
      first = min(first, __shfl_xor(first, o, 64));
    }
    if (lane == 0) { s_cnt[w] = cnt; s_last[w] = last; s_first[w] = first; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int i = 1; i < kWaves; ++i) { cnt += s_cnt[i]; last = max(last, s_last[i]); first = min(first, s_first[i]); }
      p_cnt[ps] = cnt; p_last[ps] = last; p_first[ps] = first;
    }
    __syncthreads();
  }

  // final scan per pass with carries from the other passes
  int longest = 0;
  for (int ps = 0; ps < npass; ++ps) {
    int c_cnt = 0, c_last = -1, c_first = N;
    for (int i = 0; i < ps; ++i) { c_cnt += p_cnt[i]; c_last = max(c_last, p_last[i]); }
    for (int i = npass - 1; i > ps; --i) c_first = min(c_first, p_first[i]);
    const int base = ps * kSmallPass + threadIdx.x * kPerThread;
    bool flag[kPerThread];
    int cnt = 0, last = -1, first = N;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      const int t = base + e;
      flag[e] = (t < N) && is_start(pos, t, T);
      if (flag[e]) { ++cnt; last = t; first = min(first, t); }
    }
    const int icnt = wave_incl_add(cnt), ilast = wave_incl_max(last), sfirst = wave_suffix_min(first);
    __syncthreads();  // previous pass finished with the wave arrays
    if (lane == 63) { s_cnt[w] = icnt; s_last[w] = ilast; }
    if (lane == 0) s_first[w] = sfirst;
    __syncthreads();
    int ecnt = __shfl_up(icnt, 1, 64), elast = __shfl_up(ilast, 1, 64), efirst = __shfl_down(sfirst, 1, 64);
    if (lane == 0) { ecnt = 0; elast = -1; }
    if (lane == 63) efirst = N;
    for (int i = 0; i < w; ++i) { ecnt += s_cnt[i]; elast = max(elast, s_last[i]); }
    for (int i = w + 1; i < kWaves; ++i) efirst = min(efirst, s_first[i]);
    ecnt += c_cnt;
    elast = max(elast, c_last);
    efirst = min(efirst, c_first);
    int nxt[kPerThread];
    int run = efirst;
#pragma unroll
    for (int e = kPerThread - 1; e >= 0; --e) {
      nxt[e] = run;
      if (flag[e]) run = base + e;
    }
    int c = ecnt, l = elast;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      const int t = base + e;
      if (t >= N) break;
      if (flag[e]) { cu[c] = t; ++c; l = t; longest = max(longest, nxt[e] - t); }
      seg_id[t] = c - 1;
      seg_start[t] = l;
      seg_end[t] = nxt[e];
    }
  }
  for (int o = 32; o > 0; o >>= 1) longest = max(longest, __shfl_xor(longest, o, 64));
  if (lane == 0) s_longest[w] = longest;
  __syncthreads();  // also orders this workgroup's seg_start / seg_end stores before the loads below
  if (threadIdx.x == 0) {
    int n = 0;
    for (int i = 0; i < npass; ++i) n += p_cnt[i];
    for (int i = 1; i < kWaves; ++i) longest = max(longest, s_longest[i]);
    meta[0] = n;
    meta[1] = longest;
    for (int i = 2; i < 8; ++i) meta[i] = 0;
    cu[n] = N;
  }

  // tile costs and ranks (see tile_cost_kernel / tile_rank_kernel)
  for (int tile = threadIdx.x; tile < ntiles; tile += kSmallThreads) {
    const int r = tile / tiles_per_row, m = tile % tiles_per_row;
    const int t0 = r * T + m * kTile;
    const int t1 = min(t0 + kTile, (r + 1) * T) - 1;
    s_cq[tile] = (t1 >> 6) - (seg_start[t0] >> 6) + 1;
    s_ckv[tile] = ((seg_end[t1] - 1) >> 6) - (t0 >> 6) + 1;
  }
  __syncthreads();
  for (int tile = threadIdx.x; tile < ntiles; tile += kSmallThreads) {
    const int cq = s_cq[tile], ckv = s_ckv[tile];
    int rq = 0, rkv = 0;
    for (int o = 0; o < ntiles; ++o) {
      rq += (s_cq[o] > cq) || (s_cq[o] == cq && o < tile);
      rkv += (s_ckv[o] > ckv) || (s_ckv[o] == ckv && o < tile);
    }
    order_q[rq] = tile;
    order_kv[rkv] = tile;
  }
}

}  // namespace

hipError_t launch_pack(const void *pos, va_itype it, int rows, int T, const va_segments &seg,
                       hipStream_t stream) {
  const int N = rows * T;
  const int nchunks = ceil_div(N, kScanChunk);
  const int tiles_per_row = ceil_div(T, kTile), ntiles = rows * tiles_per_row;
  if (N <= kSmallMax && ntiles <= kSmallMaxTiles) {
    if (it == VA_I64)
      pack_small_kernel<int64_t><<<1, kSmallThreads, 0, stream>>>(
          (const int64_t *)pos, N, T, tiles_per_row, ntiles, seg.cu_seqlens, seg.seg_id, seg.seg_start,
          seg.seg_end, seg.meta, seg.q_tile_order, seg.kv_tile_order);
    else
      pack_small_kernel<int32_t><<<1, kSmallThreads, 0, stream>>>(
          (const int32_t *)pos, N, T, tiles_per_row, ntiles, seg.cu_seqlens, seg.seg_id, seg.seg_start,
          seg.seg_end, seg.meta, seg.q_tile_order, seg.kv_tile_order);
    return hipGetLastError();
  }
  int32_t *agg = seg.scratch;                  // [3 * nchunks]
  int32_t *carry = seg.scratch + 3 * nchunks;  // [3 * nchunks]
  int32_t *cost_q = carry + 3 * nchunks;       // [ntiles]
  int32_t *cost_kv = cost_q + ntiles;          // [ntiles]
  if (it == VA_I64)
    scan_aggregate_kernel<int64_t><<<nchunks, kScanThreads, 0, stream>>>((const int64_t *)pos, N, T, agg);
  else
    scan_aggregate_kernel<int32_t><<<nchunks, kScanThreads, 0, stream>>>((const int32_t *)pos, N, T, agg);
  scan_carry_kernel<<<1, 64, 0, stream>>>(agg, nchunks, N, carry, seg.meta, seg.cu_seqlens);
  if (it == VA_I64)
    scan_finalize_kernel<int64_t><<<nchunks, kScanThreads, 0, stream>>>(
        (const int64_t *)pos, N, T, carry, seg.cu_seqlens, seg.seg_id, seg.seg_start, seg.seg_end, seg.meta);
  else
    scan_finalize_kernel<int32_t><<<nchunks, kScanThreads, 0, stream>>>(
        (const int32_t *)pos, N, T, carry, seg.cu_seqlens, seg.seg_id, seg.seg_start, seg.seg_end, seg.meta);
  const int tb = ceil_div(ntiles, 256);
  tile_cost_kernel<<<tb, 256, 0, stream>>>(seg.seg_start, seg.seg_end, T, tiles_per_row, ntiles, cost_q, cost_kv);
  tile_rank_kernel<<<tb, 256, 0, stream>>>(cost_q, cost_kv, ntiles, seg.q_tile_order, seg.kv_tile_order);
  return hipGetLastError();
}

}  // namespace va
