// Per-layer, per-KV-head top-k (Eq. 3; Algorithm 1: indices <- A^l.topk(B^l, dim=-1).indices).
// One workgroup per (sequence, KV head): an LDS radix-select over the fp32 bit patterns finds the k-th
// largest score, a wavefront-ballot compaction collects the winners (ties to the lower position), and a
// bitonic sort orders them by (score descending, position ascending).
#include "dkv_internal.h"

namespace dkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

__device__ inline int wave_inclusive_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive prefix sum over the kSelThreads threads of the workgroup. `scratch` holds kSelWaves ints.
__device__ inline int block_exclusive_scan(int v, int* scratch) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int incl = wave_inclusive_scan(v);
  if (lane == 63) scratch[wv] = incl;
  __syncthreads();
  int base = 0;
  for (int i = 0; i < wv; ++i) base += scratch[i];
  __syncthreads();
  return base + incl - v;
}

// Finds the bin that holds the `rem`-th largest element, given a histogram over kRadixBins digit values.
// Returns via shared `out[0]` = bin, `out[1]` = number of elements in higher bins. Bins are scanned from the top.
__device__ inline void pick_bin_desc(const int* __restrict__ hist, int rem, int* scratch, int* out) {
  static_assert(kRadixBins == 2 * kSelThreads, "two bins per thread");
  const int hi = kRadixBins - 1 - 2 * threadIdx.x, lo = hi - 1;
  const int c_hi = hist[hi], c_lo = hist[lo];
  const int above = block_exclusive_scan(c_hi + c_lo, scratch);
  if (above < rem && rem <= above + c_hi) { out[0] = hi; out[1] = above; }
  else if (above + c_hi < rem && rem <= above + c_hi + c_lo) { out[0] = lo; out[1] = above + c_hi; }
  __syncthreads();
}

__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(int Hkv, int w, int layer_max, int L, int layer,
                                                                  const float* __restrict__ scores,
                                                                  int64_t scores_stride_head,
                                                                  const int32_t* __restrict__ cu,
                                                                  int32_t* __restrict__ idx_out,
                                                                  int32_t* __restrict__ counts) {
  __shared__ unsigned long long keys[DKV_MAX_LAYER_MAX];
  __shared__ int hist[kRadixBins];
  __shared__ int scratch[kSelWaves];
  __shared__ int picked[2];
  __shared__ int n_greater_slots;
  __shared__ int wave_eq[kSelWaves];

  const int seq = blockIdx.y, head = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int begin = cu[seq];
  const int S = cu[seq + 1] - begin;
  const int n = S > w ? S - w : 0;
  const int k = layer_max < n ? layer_max : n;
  int32_t* __restrict__ out = idx_out + ((int64_t)seq * Hkv + head) * layer_max;
  if (head == 0 && tid == 0) counts[seq * L + layer] = k;
  if (k == 0) {
    for (int j = tid; j < layer_max; j += kSelThreads) out[j] = -1;
    return;
  }
  const uint32_t* __restrict__ row = reinterpret_cast<const uint32_t*>(scores + (int64_t)head * scores_stride_head + begin);

  // ---- radix select: the k-th largest bit pattern (scores are >= 0, so patterns order like the values)
  uint32_t prefix = 0;
  int rem = k;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int hshift = pass == 0 ? 32 : (pass == 1 ? 21 : 10);   // bits above this digit
    for (int b = tid; b < kRadixBins; b += kSelThreads) hist[b] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) {
      const uint32_t u = row[i];
      const bool match = pass == 0 ? true : ((u >> hshift) == (prefix >> hshift));
      if (match) atomicAdd(&hist[(u >> shift) & (kRadixBins - 1)], 1);
    }
    __syncthreads();
    pick_bin_desc(hist, rem, scratch, picked);
    prefix |= (uint32_t)picked[0] << shift;
    rem -= picked[1];
    __syncthreads();
  }
  const uint32_t T = prefix;      // k-th largest value
  const int need_eq = rem;        // how many elements equal to T are taken (>= 1)
  const int n_gt = k - need_eq;   // elements strictly greater than T

  // ---- compaction. Each wavefront walks a contiguous segment in 64-wide coalesced steps.
  if (tid == 0) n_greater_slots = 0;
  __syncthreads();
  int seg = (n + kSelWaves - 1) / kSelWaves;
  seg = (seg + 63) / 64 * 64;
  const int seg_begin = wv * seg;
  const int seg_end = seg_begin + seg < n ? seg_begin + seg : n;
  int eq_count = 0;
  for (int i0 = seg_begin; i0 < seg_end; i0 += 64) {
    const int i = i0 + lane;
    const uint32_t u = i < seg_end ? row[i] : 0u;
    const bool gt = i < seg_end && u > T;
    const bool eq = i < seg_end && u == T;
    const unsigned long long gmask = __ballot(gt);
    eq_count += __popcll(__ballot(eq));
    if (gmask) {
      int base = 0;
      if (lane == 0) base = atomicAdd(&n_greater_slots, __popcll(gmask));
      base = __shfl(base, 0);
      if (gt) {
        const int slot = base + __popcll(gmask & ((1ull << lane) - 1ull));
        keys[slot] = ((unsigned long long)(~u) << 32) | (uint32_t)i;
      }
    }
  }
  if (lane == 0) wave_eq[wv] = eq_count;
  __syncthreads();
  int running = 0;
  for (int i = 0; i < wv; ++i) running += wave_eq[i];
  // equal elements are taken in position order until need_eq are placed
  for (int i0 = seg_begin; i0 < seg_end && running < need_eq; i0 += 64) {
    const int i = i0 + lane;
    const bool eq = i < seg_end && row[i] == T;
    const unsigned long long emask = __ballot(eq);
    if (eq) {
      const int rank = running + __popcll(emask & ((1ull << lane) - 1ull));
      if (rank < need_eq) keys[n_gt + rank] = ((unsigned long long)(~T) << 32) | (uint32_t)i;
    }
    running += __popcll(emask);
  }
  int KP = 2;
  while (KP < k) KP <<= 1;
  for (int j = k + tid; j < KP; j += kSelThreads) keys[j] = ~0ull;
  __syncthreads();

  // ---- bitonic sort of KP composite keys (ascending = score descending, position ascending)
  for (int size = 2; size <= KP; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < (KP >> 1); t += kSelThreads) {
        const int lo = 2 * t - (t & (stride - 1));
        const int hi = lo + stride;
        const bool up = (lo & size) == 0;
        const unsigned long long a = keys[lo], b = keys[hi];
        if ((a > b) == up) { keys[lo] = b; keys[hi] = a; }
      }
      __syncthreads();
    }
  }
  for (int j = tid; j < layer_max; j += kSelThreads) out[j] = j < k ? (int32_t)(uint32_t)keys[j] : -1;
}

hipError_t launch_select(const Params& p, int layer, const float* scores, int64_t scores_stride_head,
                         const int32_t* cu, int32_t* idx_out, int32_t* counts, hipStream_t st) {
  hipLaunchKernelGGL(select_topk_kernel, dim3(p.Hkv, p.n_seqs), dim3(kSelThreads), 0, st, p.Hkv, p.w, p.layer_max,
                     p.L, layer, scores, scores_stride_head, cu, idx_out, counts);
  return hipGetLastError();
}

}  // namespace dkv
