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

// Start flags of the kPerThread consecutive tokens from `base`.  The ids are loaded
// unconditionally (index clamped into the stream) before any of them is looked at: loads under a
// condition would be issued one at a time, each waiting for the one before.
template <typename IdT>
__device__ __forceinline__ void start_flags(const IdT *pos, int base, int N, int T, bool (&flag)[kPerThread]) {
  IdT id[kPerThread];
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) id[e] = pos[min(base + e, N - 1)];
  int r = base % T;  // position inside the packed row, advanced without further divisions
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    flag[e] = base + e < N && (id[e] == 0 || r == 0);
    if (++r == T) r = 0;
  }
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
  bool flag[kPerThread];
  start_flags(pos, base, N, T, flag);
  int cnt = 0, last = -1, first = N;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    if (flag[e]) {
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
  start_flags(pos, base, N, T, flag);
  int cnt = 0, last = -1, first = N;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
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
//
// Order: tiles are sorted by a key (longest governing example first, then that example's start,
// then cost, heaviest first; ties by tile index).  The governing example is the one that fixes the
// streamed range: the example of the first token for a query tile, of the last token for a key
// tile.  Tiles of one long example thus run next to each other -- they stream the same K/V (or
// Q/dO) blocks at about the same time and share them in L2 -- and long work still starts first.
// Examples of at most one schedule tile all rank alike, so their tiles keep the order of the stream:
// a tile whose first example began in the previous tile reads that tile's last K/V rows again (a key
// tile the next tile's first Q/dO rows), and finds them in L2 only if the neighbour ran just before
// it on the same XCD.  With examples of 8..128 tokens that saves 9 % of the step.
constexpr int kShortExample = VA_TILE;
__device__ __forceinline__ unsigned long long tile_key(int len, int start, int cost) {
  return ((unsigned long long)(len <= kShortExample ? 0 : min(len, (1 << 20) - 1)) << 43) |
         ((unsigned long long)(0x7fffffff - start) << 12) | (unsigned long long)min(cost, 4095);
}
// An order entry carries, above the tile index (bits 0..23), the head rotation of its tile (bits
// 24..30; see head_rotation in va_mfma_common.h).  Tiles of an example longer than a schedule tile
// all get one rotation, derived from the example's first token: workgroup w runs on XCD w % 8 and the
// rotation decides which head lands on which XCD, so the tiles of one example - which stream the same
// K/V (or Q/dO) rows - keep each head on one XCD and fetch its rows into one L2 only, while different
// examples start from different rotations.  Tiles of short examples take their rank / 8: over a
// launch every XCD then meets every head (with a fixed assignment every XCD would always read the
// same 256-byte columns of the token rows, i.e. a fixed subset of the memory channels; measured on
// examples of 8..128 tokens, where the kernels are bound by HBM: two XCDs ran 20 % slower than the
// rest), while neighbours in launch order still mostly share an XCD.
__device__ __forceinline__ int32_t order_entry(int tile, unsigned long long key, int rank) {
  const unsigned len_class = (unsigned)(key >> 43);
  const unsigned start = 0x7fffffffu - (unsigned)((key >> 12) & 0x7fffffffu);
  const unsigned rot = len_class ? (start / kTile) * 5u + (start >> 13) : (unsigned)rank >> 3;
  return (int32_t)((unsigned)tile | ((rot & 127u) << 24));
}

__global__ void __launch_bounds__(256)
tile_cost_kernel(const int32_t *__restrict__ seg_start, const int32_t *__restrict__ seg_end, int T,
                 int tiles_per_row, int ntiles, unsigned long long *__restrict__ key_q,
                 unsigned long long *__restrict__ key_kv) {
  const int tile = blockIdx.x * blockDim.x + threadIdx.x;
  if (tile >= ntiles) return;
  const int r = tile / tiles_per_row, m = tile % tiles_per_row;
  const int t0 = r * T + m * kTile;
  const int t1 = min(t0 + kTile, (r + 1) * T) - 1;  // last token of the tile
  key_q[tile] = tile_key(seg_end[t0] - seg_start[t0], seg_start[t0], (t1 >> 6) - (seg_start[t0] >> 6) + 1);
  key_kv[tile] = tile_key(seg_end[t1] - seg_start[t1], seg_start[t1], ((seg_end[t1] - 1) >> 6) - (t0 >> 6) + 1);
}

// order[rank] = tile, rank = number of tiles with a larger key (ties: lower index first)
__global__ void __launch_bounds__(256)
tile_rank_kernel(const unsigned long long *__restrict__ cost_q, const unsigned long long *__restrict__ cost_kv,
                 int ntiles, int32_t *__restrict__ order_q, int32_t *__restrict__ order_kv) {
  __shared__ unsigned long long s_q[256], s_kv[256];
  const int tile = blockIdx.x * blockDim.x + threadIdx.x;
  const unsigned long long cq = tile < ntiles ? cost_q[tile] : 0, ckv = tile < ntiles ? cost_kv[tile] : 0;
  int rq = 0, rkv = 0;
  for (int b0 = 0; b0 < ntiles; b0 += 256) {
    const int o = b0 + threadIdx.x;
    s_q[threadIdx.x] = o < ntiles ? cost_q[o] : 0;
    s_kv[threadIdx.x] = o < ntiles ? cost_kv[o] : 0;
    __syncthreads();
    const int lim = min(256, ntiles - b0);
    for (int i = 0; i < lim; ++i) {
      const int other = b0 + i;
      rq += (s_q[i] > cq) || (s_q[i] == cq && other < tile);
      rkv += (s_kv[i] > ckv) || (s_kv[i] == ckv && other < tile);
    }
    __syncthreads();
  }
  if (tile < ntiles) { order_q[rq] = order_entry(tile, cq, rq); order_kv[rkv] = order_entry(tile, ckv, rkv); }
}

// ---- two-launch path for streams of up to kOnePassMaxChunks chunks --------------------------------
// Launch 1: every chunk's workgroup derives its own carries by reading the ids of all other chunks
// (count and last start before it, first start after it) -- redundant reads that stay in L2, in
// exchange for no inter-workgroup dependency and no separate carry kernel.  Launch 2: sort keys of
// all tiles into LDS, ranks of this workgroup's tiles, and max_seqlen from the per-chunk maxima.
constexpr int kOnePassMaxChunks = 4;  // 8192 tokens: beyond that the redundant reads cost more than two launches
constexpr int kFusedMaxTiles = 2048;

template <typename IdT>
__global__ void __launch_bounds__(kScanThreads)
scan_onepass_kernel(const IdT *__restrict__ pos, int N, int T, int32_t *__restrict__ cu,
                    int32_t *__restrict__ seg_id, int32_t *__restrict__ seg_start,
                    int32_t *__restrict__ seg_end, int32_t *__restrict__ meta,
                    int32_t *__restrict__ chunk_longest) {
  __shared__ int s_cnt[kScanThreads / 64], s_last[kScanThreads / 64], s_first[kScanThreads / 64];
  __shared__ int c_cnt, c_last, c_first;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int chunk0 = blockIdx.x * kScanChunk;
  // this thread's own tokens: their loads go out together with the sweep's below
  const int base = chunk0 + threadIdx.x * kPerThread;
  bool flag[kPerThread];
  start_flags(pos, base, N, T, flag);
  // Carries from the rest of the stream in one sweep: every id outside this chunk is read once, all
  // loads of a thread issued together (the stream has at most kOnePassMaxChunks chunks), giving the
  // number of starts and the last start before the chunk and the first start after it.
  {
    constexpr int kSweep = kOnePassMaxChunks * kScanChunk / kScanThreads;
    const int chunk1 = chunk0 + kScanChunk;
    IdT id[kSweep];  // unconditional loads (index clamped), so that they are all in flight together
#pragma unroll
    for (int u = 0; u < kSweep; ++u) id[u] = pos[min(u * kScanThreads + (int)threadIdx.x, N - 1)];
    int cnt = 0, last = -1, first = N;
    int r = threadIdx.x % T;  // position inside the packed row, advanced without further divisions
    const int step = kScanThreads % T;
#pragma unroll
    for (int u = 0; u < kSweep; ++u) {
      const int t = u * kScanThreads + threadIdx.x;
      if (t < N && (t < chunk0 || t >= chunk1) && (id[u] == 0 || r == 0)) {
        if (t < chunk0) { ++cnt; last = t; } else first = min(first, t);
      }
      r += step;
      if (r >= T) r -= T;
    }
    for (int o = 32; o > 0; o >>= 1) {
      cnt += __shfl_xor(cnt, o, 64);
      last = max(last, __shfl_xor(last, o, 64));
      first = min(first, __shfl_xor(first, o, 64));
    }
    if (lane == 0) { s_cnt[w] = cnt; s_last[w] = last; s_first[w] = first; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int i = 1; i < kScanThreads / 64; ++i) {
        cnt += s_cnt[i];
        last = max(last, s_last[i]);
        first = min(first, s_first[i]);
      }
      c_cnt = cnt;
      c_last = last;
      c_first = first;
    }
  }
  __syncthreads();
  // local scan, as in scan_finalize_kernel
  int cnt = 0, last = -1, first = N;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    if (flag[e]) { ++cnt; last = t; first = min(first, t); }
  }
  const int icnt = wave_incl_add(cnt), ilast = wave_incl_max(last), sfirst = wave_suffix_min(first);
  if (lane == 63) { s_cnt[w] = icnt; s_last[w] = ilast; }
  if (lane == 0) s_first[w] = sfirst;
  __syncthreads();
  int ecnt = __shfl_up(icnt, 1, 64), elast = __shfl_up(ilast, 1, 64), efirst = __shfl_down(sfirst, 1, 64);
  if (lane == 0) { ecnt = 0; elast = -1; }
  if (lane == 63) efirst = N;
  for (int i = 0; i < w; ++i) { ecnt += s_cnt[i]; elast = max(elast, s_last[i]); }
  for (int i = w + 1; i < kScanThreads / 64; ++i) efirst = min(efirst, s_first[i]);
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
  int c = ecnt, l = elast, longest = 0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    if (t >= N) break;
    if (flag[e]) { cu[c] = t; ++c; l = t; longest = max(longest, nxt[e] - t); }
    seg_id[t] = c - 1;
    seg_start[t] = l;
    seg_end[t] = nxt[e];
  }
  for (int o = 32; o > 0; o >>= 1) longest = max(longest, __shfl_xor(longest, o, 64));
  __syncthreads();  // s_cnt free
  if (lane == 0) s_cnt[w] = longest;
  // the last thread of the last chunk knows the total number of examples
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kScanThreads - 1) {
    meta[0] = c;
    for (int i = 2; i < 8; ++i) meta[i] = 0;
    cu[c] = N;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < kScanThreads / 64; ++i) longest = max(longest, s_cnt[i]);
    chunk_longest[blockIdx.x] = longest;
  }
}

__global__ void __launch_bounds__(256)
tile_order_fused_kernel(const int32_t *__restrict__ seg_start, const int32_t *__restrict__ seg_end, int T,
                        int tiles_per_row, int ntiles, const int32_t *__restrict__ chunk_longest, int nchunks,
                        int32_t *__restrict__ meta, int32_t *__restrict__ order_q,
                        int32_t *__restrict__ order_kv) {
  __shared__ unsigned long long s_q[kFusedMaxTiles], s_kv[kFusedMaxTiles];
  for (int tile = threadIdx.x; tile < ntiles; tile += 256) {
    const int r = tile / tiles_per_row, m = tile % tiles_per_row;
    const int t0 = r * T + m * kTile;
    const int t1 = min(t0 + kTile, (r + 1) * T) - 1;
    const int ss0 = seg_start[t0], se0 = seg_end[t0], ss1 = seg_start[t1], se1 = seg_end[t1];
    s_q[tile] = tile_key(se0 - ss0, ss0, (t1 >> 6) - (ss0 >> 6) + 1);
    s_kv[tile] = tile_key(se1 - ss1, ss1, ((se1 - 1) >> 6) - (t0 >> 6) + 1);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0 && nchunks > 0) {  // nchunks == 0: max_seqlen is already in meta
    int longest = 0;
    for (int i = 0; i < nchunks; ++i) longest = max(longest, chunk_longest[i]);
    meta[1] = longest;
  }
  __syncthreads();
  const int tile = blockIdx.x * 256 + threadIdx.x;
  if (tile >= ntiles) return;
  const unsigned long long cq = s_q[tile], ckv = s_kv[tile];
  int rq = 0, rkv = 0;
  for (int o = 0; o < ntiles; ++o) {
    rq += (s_q[o] > cq) || (s_q[o] == cq && o < tile);
    rkv += (s_kv[o] > ckv) || (s_kv[o] == ckv && o < tile);
  }
  order_q[rq] = order_entry(tile, cq, rq);
  order_kv[rkv] = order_entry(tile, ckv, rkv);
}

// ---- one launch for streams of up to kSingleMaxTokens tokens -----------------------------------
// One workgroup of 1024 threads holds the whole stream: boundary scan without carries (8 consecutive
// tokens per thread), then tile keys and ranks after a barrier.  All global traffic is coalesced
// (thread i touches tokens i, i + 1024, ...): the ids' start flags go through LDS to the threads that
// scan them, and seg_id / seg_start / seg_end come back through LDS to be written out the same way --
// one compute unit cannot afford 64 cache lines per load or store instruction.  Used when the stream
// fits, because at this size every extra launch costs as much as the work.
constexpr int kSingleThreads = 1024;
constexpr int kSingleMaxTokens = kSingleThreads * kPerThread;  // 8192
constexpr int kSingleMaxTiles = 256;

template <typename IdT>
__global__ void __launch_bounds__(kSingleThreads)
pack_single_kernel(const IdT *__restrict__ pos, int N, int T, int tiles_per_row, int ntiles,
                   int32_t *__restrict__ cu, int32_t *__restrict__ seg_id, int32_t *__restrict__ seg_start,
                   int32_t *__restrict__ seg_end, int32_t *__restrict__ meta, int32_t *__restrict__ order_q,
                   int32_t *__restrict__ order_kv) {
  constexpr int kWaves = kSingleThreads / 64;
  __shared__ int s_cnt[kWaves], s_last[kWaves], s_first[kWaves];
  __shared__ int32_t s_ss[kSingleMaxTokens], s_se[kSingleMaxTokens], s_id[kSingleMaxTokens];
  __shared__ __attribute__((aligned(8))) uint8_t s_flag[kSingleMaxTokens];
  __shared__ unsigned long long s_q[kSingleMaxTiles], s_kv[kSingleMaxTiles];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  {  // start flags, coalesced; all loads in flight together
    IdT id[kPerThread];
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) id[e] = pos[min(e * kSingleThreads + (int)threadIdx.x, N - 1)];
    int r = threadIdx.x % T;
    const int step = kSingleThreads % T;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      const int t = e * kSingleThreads + threadIdx.x;
      s_flag[t] = t < N && (id[e] == 0 || r == 0);
      r += step;
      if (r >= T) r -= T;
    }
  }
  __syncthreads();
  const int base = threadIdx.x * kPerThread;
  bool flag[kPerThread];
  {
    const unsigned long long f8 = *(const unsigned long long *)(s_flag + base);
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) flag[e] = (f8 >> (8 * e)) & 1;
  }
  int cnt = 0, last = -1, first = N;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int t = base + e;
    if (flag[e]) { ++cnt; last = t; first = min(first, t); }
  }
  const int icnt = wave_incl_add(cnt), ilast = wave_incl_max(last), sfirst = wave_suffix_min(first);
  if (lane == 63) { s_cnt[w] = icnt; s_last[w] = ilast; }
  if (lane == 0) s_first[w] = sfirst;
  __syncthreads();
  int ecnt = __shfl_up(icnt, 1, 64), elast = __shfl_up(ilast, 1, 64), efirst = __shfl_down(sfirst, 1, 64);
  if (lane == 0) { ecnt = 0; elast = -1; }
  if (lane == 63) efirst = N;
  for (int i = 0; i < w; ++i) { ecnt += s_cnt[i]; elast = max(elast, s_last[i]); }
  for (int i = w + 1; i < kWaves; ++i) efirst = min(efirst, s_first[i]);
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
    if (flag[e]) { cu[c] = t; ++c; l = t; longest = max(longest, nxt[e] - t); }
    s_id[t] = c - 1;
    s_ss[t] = l;
    s_se[t] = nxt[e];
  }
  for (int o = 32; o > 0; o >>= 1) longest = max(longest, __shfl_xor(longest, o, 64));
  __syncthreads();  // s_cnt free; s_id / s_ss / s_se complete
  if (lane == 0) s_cnt[w] = longest;
  if (threadIdx.x == (N - 1) / kPerThread) {  // the thread holding the last token knows the number of examples
    meta[0] = c;
    for (int i = 2; i < 8; ++i) meta[i] = 0;
    cu[c] = N;
  }
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {  // coalesced write-out
    const int t = e * kSingleThreads + threadIdx.x;
    if (t < N) { seg_id[t] = s_id[t]; seg_start[t] = s_ss[t]; seg_end[t] = s_se[t]; }
  }
  // tile keys
  if ((int)threadIdx.x < ntiles) {
    const int tile = threadIdx.x;
    const int r = tile / tiles_per_row, m = tile % tiles_per_row;
    const int t0 = r * T + m * kTile;
    const int t1 = min(t0 + kTile, (r + 1) * T) - 1;
    const int ss0 = s_ss[t0], se0 = s_se[t0], ss1 = s_ss[t1], se1 = s_se[t1];
    s_q[tile] = tile_key(se0 - ss0, ss0, (t1 >> 6) - (ss0 >> 6) + 1);
    s_kv[tile] = tile_key(se1 - ss1, ss1, ((se1 - 1) >> 6) - (t0 >> 6) + 1);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < kWaves; ++i) longest = max(longest, s_cnt[i]);
    meta[1] = longest;
  }
  if ((int)threadIdx.x < ntiles) {
    const int tile = threadIdx.x;
    const unsigned long long cq = s_q[tile], ckv = s_kv[tile];
    int rq = 0, rkv = 0;
    for (int o = 0; o < ntiles; ++o) {
      rq += (s_q[o] > cq) || (s_q[o] == cq && o < tile);
      rkv += (s_kv[o] > ckv) || (s_kv[o] == ckv && o < tile);
    }
    order_q[rq] = order_entry(tile, cq, rq);
    order_kv[rkv] = order_entry(tile, ckv, rkv);
  }
}

}  // namespace

hipError_t launch_pack(const void *pos, va_itype it, int rows, int T, const va_segments &seg,
                       hipStream_t stream) {
  const int N = rows * T;
  const int nchunks = ceil_div(N, kScanChunk);
  const int tiles_per_row = ceil_div(T, kTile), ntiles = rows * tiles_per_row;
  if (N <= kSingleMaxTokens && ntiles <= kSingleMaxTiles) {
    if (it == VA_I64)
      pack_single_kernel<int64_t><<<1, kSingleThreads, 0, stream>>>(
          (const int64_t *)pos, N, T, tiles_per_row, ntiles, seg.cu_seqlens, seg.seg_id, seg.seg_start, seg.seg_end,
          seg.meta, seg.q_tile_order, seg.kv_tile_order);
    else
      pack_single_kernel<int32_t><<<1, kSingleThreads, 0, stream>>>(
          (const int32_t *)pos, N, T, tiles_per_row, ntiles, seg.cu_seqlens, seg.seg_id, seg.seg_start, seg.seg_end,
          seg.meta, seg.q_tile_order, seg.kv_tile_order);
    return hipGetLastError();
  }
  if (nchunks <= kOnePassMaxChunks && ntiles <= kFusedMaxTiles) {
    int32_t *chunk_longest = seg.scratch;  // [nchunks]
    if (it == VA_I64)
      scan_onepass_kernel<int64_t><<<nchunks, kScanThreads, 0, stream>>>(
          (const int64_t *)pos, N, T, seg.cu_seqlens, seg.seg_id, seg.seg_start, seg.seg_end, seg.meta, chunk_longest);
    else
      scan_onepass_kernel<int32_t><<<nchunks, kScanThreads, 0, stream>>>(
          (const int32_t *)pos, N, T, seg.cu_seqlens, seg.seg_id, seg.seg_start, seg.seg_end, seg.meta, chunk_longest);
    tile_order_fused_kernel<<<ceil_div(ntiles, 256), 256, 0, stream>>>(
        seg.seg_start, seg.seg_end, T, tiles_per_row, ntiles, chunk_longest, nchunks, seg.meta, seg.q_tile_order,
        seg.kv_tile_order);
    return hipGetLastError();
  }
  int32_t *agg = seg.scratch;                  // [3 * nchunks]
  int32_t *carry = seg.scratch + 3 * nchunks;  // [3 * nchunks]
  unsigned long long *cost_q = (unsigned long long *)(seg.scratch + 8 * nchunks);  // [ntiles] sort keys
  unsigned long long *cost_kv = cost_q + ntiles;                                   // [ntiles]
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
  if (ntiles <= kFusedMaxTiles) {  // keys of all tiles fit in LDS: keys and ranks in one launch
    tile_order_fused_kernel<<<tb, 256, 0, stream>>>(seg.seg_start, seg.seg_end, T, tiles_per_row, ntiles, nullptr, 0,
                                                    seg.meta, seg.q_tile_order, seg.kv_tile_order);
    return hipGetLastError();
  }
  tile_cost_kernel<<<tb, 256, 0, stream>>>(seg.seg_start, seg.seg_end, T, tiles_per_row, ntiles, cost_q, cost_kv);
  tile_rank_kernel<<<tb, 256, 0, stream>>>(cost_q, cost_kv, ntiles, seg.q_tile_order, seg.kv_tile_order);
  return hipGetLastError();
}

}  // namespace va
