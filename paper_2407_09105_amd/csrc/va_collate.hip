// Device-side padding-free collator (paper, Section 3.4): a minibatch held as a padded
// [n, Lp] batch with per-example lengths becomes one packed row of input_ids, labels (first
// label of every example -> -100) and position_ids (restarting at 0 in every example) --
// the three tensors Section 3.5 prints for its worked example.  Integer work only.
#include "va_internal.h"

namespace va {
namespace {

constexpr int kOffThreads = 1024;

__device__ __forceinline__ int clamp_len(int L, int Lp) { return L < 0 ? 0 : (L > Lp ? Lp : L); }

// offsets[e] = sum of the clamped lengths of examples before e; offsets[n] = total.
// One workgroup walks the lengths in slabs of kOffThreads with a running carry.
__global__ void __launch_bounds__(kOffThreads)
collate_offsets_kernel(const int32_t *__restrict__ lengths, int n, int Lp, int32_t *__restrict__ offsets) {
  __shared__ int32_t wave_sum[kOffThreads / 64];
  __shared__ int32_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { carry_s = 0; offsets[0] = 0; }
  __syncthreads();
  for (int base = 0; base < n; base += kOffThreads) {
    const int e = base + tid;
    const int L = e < n ? clamp_len(lengths[e], Lp) : 0;
    int incl = L;  // inclusive scan inside the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (e < n) offsets[e + 1] = before + incl;
    __syncthreads();
    if (tid == kOffThreads - 1) carry_s = before + incl;
    __syncthreads();
  }
}

// One thread per output token: find its example by bisection over the offsets, then copy.
template <typename IdT>
__global__ void __launch_bounds__(256)
collate_tokens_kernel(const IdT *__restrict__ ids, const IdT *__restrict__ labels_in,
                      const int32_t *__restrict__ offsets, int n, int Lp, int n_out, IdT pad_id,
                      IdT *__restrict__ input_ids, IdT *__restrict__ labels, IdT *__restrict__ position_ids) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= n_out) return;
  const int total = offsets[n];
  if (t >= total) {  // tail: one pad pseudo-example
    input_ids[t] = pad_id;
    labels[t] = (IdT)-100;
    position_ids[t] = (IdT)(t - total);
    return;
  }
  int lo = 0, hi = n;  // largest e with offsets[e] <= t (empty examples share an offset: take the last)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (offsets[mid] <= t) lo = mid; else hi = mid;
  }
  const int p = t - offsets[lo];
  const size_t src = (size_t)lo * Lp + p;
  const IdT id = ids[src];
  input_ids[t] = id;
  labels[t] = p == 0 ? (IdT)-100 : (labels_in ? labels_in[src] : id);
  position_ids[t] = (IdT)p;
}

}  // namespace

hipError_t launch_collate(const void *ids, const void *labels_in, va_itype it, const int32_t *lengths,
                          int n, int Lp, int n_out, long long pad_id, void *input_ids, void *labels,
                          void *position_ids, int32_t *offsets, hipStream_t stream) {
  collate_offsets_kernel<<<1, kOffThreads, 0, stream>>>(lengths, n, Lp, offsets);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_out == 0) return e;
  const unsigned grid = (unsigned)ceil_div(n_out, 256);
  if (it == VA_I64)
    collate_tokens_kernel<int64_t><<<grid, 256, 0, stream>>>(
        (const int64_t *)ids, (const int64_t *)labels_in, offsets, n, Lp, n_out, (int64_t)pad_id,
        (int64_t *)input_ids, (int64_t *)labels, (int64_t *)position_ids);
  else
    collate_tokens_kernel<int32_t><<<grid, 256, 0, stream>>>(
        (const int32_t *)ids, (const int32_t *)labels_in, offsets, n, Lp, n_out, (int32_t)pad_id,
        (int32_t *)input_ids, (int32_t *)labels, (int32_t *)position_ids);
  return hipGetLastError();
}

}  // namespace va
