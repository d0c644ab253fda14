// Per-layer, per-KV-head top-k (Eq. 3; Algorithm 1: indices <- A^l.topk(B^l, dim=-1).indices).
// One workgroup per (sequence, KV head):
//   1. LDS radix-select (3 digits of 11/11/10 bits of the fp32 pattern; scores are >= 0 so patterns order like
//      values) finds the k-th largest score T. The digit histogram is kept in 8 interleaved copies so that
//      lanes whose scores share a digit do not serialise on one LDS word.
//   2. wavefront-ballot compaction collects the winners: everything above T, and the first (k - #above)
//      elements equal to T in position order (ties go to the lower position).
//   3. the k winners are written as 64-bit keys (~score bits, position), unordered, to the workspace.
// A second kernel orders them by (score descending, position ascending) = ascending key, by counting: the rank
// of a key is the number of smaller keys (keys are unique). That is k^2 comparisons, but they spread over the
// whole GPU (k/256 workgroups per row) instead of a sorting network on the one CU that holds the row.
#include "dkv_internal.h"

namespace dkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kHistCopies = 8;
constexpr int kSelPerThread = 32;                              // row positions a thread keeps in registers
constexpr int kSelResident = kSelPerThread * kSelThreads;      // 32768 positions

typedef unsigned long long u64;

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

// grid = (Hkv, n_seqs, layers of the call); blockIdx.z picks the layer: its scores, index list and key block lie
// blockIdx.z layer strides behind the pointers passed in.
__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(int Hkv, int w, int layer_max, int L, int layer0,
                                                                  const float* __restrict__ scores0,
                                                                  int64_t scores_stride_head,
                                                                  int64_t scores_stride_layer,
                                                                  const int32_t* __restrict__ cu,
                                                                  int32_t* __restrict__ idx_out0,
                                                                  int64_t idx_stride_layer,
                                                                  int32_t* __restrict__ counts,
                                                                  u64* __restrict__ keys_out0) {
  extern __shared__ __attribute__((aligned(16))) char sel_smem[];
  u64* keys = reinterpret_cast<u64*>(sel_smem);                               // [2048] candidates / exchange
  int* hist = reinterpret_cast<int*>(sel_smem + 2048 * sizeof(u64));          // [kRadixBins][kHistCopies]
  __shared__ int scratch[kSelWaves];
  __shared__ int picked[2];
  __shared__ int n_greater_slots;
  __shared__ int wave_eq[kSelWaves];

  const int seq = blockIdx.y, head = blockIdx.x;
  const int layer = layer0 + blockIdx.z;
  const float* __restrict__ scores = scores0 + (int64_t)blockIdx.z * scores_stride_layer;
  int32_t* __restrict__ idx_out = idx_out0 + (int64_t)blockIdx.z * idx_stride_layer;
  u64* __restrict__ keys_out = keys_out0 + (int64_t)blockIdx.z * gridDim.y * Hkv * DKV_MAX_LAYER_MAX;
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

  // The first kSelResident positions of the row live in registers for all passes: thread t holds positions
  // j * 1024 + t (coalesced loads, issued back to back). Longer rows re-read their tail from memory.
  uint32_t v[kSelPerThread];
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = j * kSelThreads + tid;
    v[j] = i < n ? row[i] : 0u;
  }
  const int n_res = n < kSelResident ? n : kSelResident;   // positions held in registers

  // ---- radix select: the k-th largest bit pattern
  uint32_t prefix = 0;
  int rem = k;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int hshift = pass == 0 ? 32 : (pass == 1 ? 21 : 10);   // bits above this digit
    // pass 0 sees every element (lanes that share a digit spread over 8 copies of the histogram); the later
    // passes only the elements that share the digits found so far: 2 copies, less to clear and to add up
    const int copies = pass == 0 ? kHistCopies : 2;
    for (int b = tid; b < kRadixBins * copies; b += kSelThreads) hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
      const uint32_t u = v[j];
      const bool match = pass == 0 ? true : ((u >> hshift) == (prefix >> hshift));
      if (j * kSelThreads + tid < n_res && match)
        atomicAdd(&hist[((u >> shift) & (kRadixBins - 1)) * copies + (lane & (copies - 1))], 1);
    }
    for (int i = kSelResident + tid; i < n; i += kSelThreads) {
      const uint32_t u = row[i];
      const bool match = pass == 0 ? true : ((u >> hshift) == (prefix >> hshift));
      if (match) atomicAdd(&hist[((u >> shift) & (kRadixBins - 1)) * copies + (lane & (copies - 1))], 1);
    }
    __syncthreads();
    // thread t owns digits 2047 - 2t and 2046 - 2t (scanned from the top)
    const int hi = kRadixBins - 1 - 2 * tid, lo = hi - 1;
    int c_hi = 0, c_lo = 0;
    if (pass == 0) {
#pragma unroll
      for (int c = 0; c < kHistCopies; ++c) { c_hi += hist[hi * kHistCopies + c]; c_lo += hist[lo * kHistCopies + c]; }
    } else {   // lo and hi are adjacent: 4 consecutive words
      const int4 q = *reinterpret_cast<const int4*>(&hist[lo * 2]);
      c_lo = q.x + q.y;
      c_hi = q.z + q.w;
    }
    const int above = block_exclusive_scan(c_hi + c_lo, scratch);
    if (above < rem && rem <= above + c_hi) { picked[0] = hi; picked[1] = above; }
    else if (above + c_hi < rem && rem <= above + c_hi + c_lo) { picked[0] = lo; picked[1] = above + c_hi; }
    __syncthreads();
    prefix |= (uint32_t)picked[0] << shift;
    rem -= picked[1];
    __syncthreads();
  }
  const uint32_t T = prefix;      // k-th largest value
  const int need_eq = rem;        // how many elements equal to T are taken (>= 1)
  const int n_gt = k - need_eq;   // elements strictly greater than T

  // ---- compaction: everything above T (any order: the sort fixes it), and the first need_eq elements equal
  // to T in position order. Position order of the resident part is (j, wavefront, lane).
  int* eq_base = hist;            // [kSelPerThread][kSelWaves] counts, then exclusive prefix sums (reuses hist)
  if (tid == 0) n_greater_slots = 0;
  for (int j = k + tid; j < 2048; j += kSelThreads) keys[j] = ~0ull;      // pads sort to the end
  __syncthreads();
  // elements above T: every thread counts its own, one scan over the threads gives it a contiguous range of
  // slots (any order will do); elements equal to T: counted per (j, wavefront) for the position-ordered pick below
  int my_gt = 0;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = j * kSelThreads + tid;
    const uint32_t u = v[j];
    my_gt += i < n_res && u > T ? 1 : 0;
    const unsigned long long emask = __ballot(i < n_res && u == T);
    if (lane == 0) eq_base[j * kSelWaves + wv] = __popcll(emask);
  }
  int slot = block_exclusive_scan(my_gt, scratch);
  if (tid == kSelThreads - 1) n_greater_slots = slot + my_gt;     // the tail of a long row continues from here
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = j * kSelThreads + tid;
    const uint32_t u = v[j];
    if (i < n_res && u > T) keys[slot++] = ((u64)(~u) << 32) | (uint32_t)i;
  }
  __syncthreads();
  {
    static_assert(kSelPerThread * kSelWaves <= kSelThreads, "one count per thread");
    const int c = tid < kSelPerThread * kSelWaves ? eq_base[tid] : 0;
    const int ex = block_exclusive_scan(c, scratch);
    if (tid < kSelPerThread * kSelWaves) eq_base[tid] = ex;
    if (tid == kSelPerThread * kSelWaves - 1) picked[0] = ex + c;   // equal elements in the resident part
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = j * kSelThreads + tid;
    const bool eq = i < n_res && v[j] == T;
    const unsigned long long emask = __ballot(eq);
    if (eq) {
      const int rank = eq_base[j * kSelWaves + wv] + __popcll(emask & ((1ull << lane) - 1ull));
      if (rank < need_eq) keys[n_gt + rank] = ((u64)(~T) << 32) | (uint32_t)i;
    }
  }
  if (n > kSelResident) {
    // tail of a long row: contiguous segments per wavefront, walked in 64-wide coalesced steps
    const int eq_resident = picked[0];
    const int tail = n - kSelResident;
    int seg = (tail + kSelWaves - 1) / kSelWaves;
    seg = (seg + 63) / 64 * 64;
    const int seg_begin = kSelResident + wv * seg;
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
        if (gt) keys[base + __popcll(gmask & ((1ull << lane) - 1ull))] = ((u64)(~u) << 32) | (uint32_t)i;
      }
    }
    if (lane == 0) wave_eq[wv] = eq_count;
    __syncthreads();
    int running = eq_resident;
    for (int i = 0; i < wv; ++i) running += wave_eq[i];
    for (int i0 = seg_begin; i0 < seg_end && running < need_eq; i0 += 64) {
      const int i = i0 + lane;
      const bool eq = i < seg_end && row[i] == T;
      const unsigned long long emask = __ballot(eq);
      if (eq) {
        const int rank = running + __popcll(emask & ((1ull << lane) - 1ull));
        if (rank < need_eq) keys[n_gt + rank] = ((u64)(~T) << 32) | (uint32_t)i;
      }
      running += __popcll(emask);
    }
  }
  __syncthreads();

  // ---- hand the k winners to the ordering kernel
  u64* __restrict__ dst = keys_out + ((int64_t)seq * Hkv + head) * DKV_MAX_LAYER_MAX;
  for (int j = tid; j < k; j += kSelThreads) dst[j] = keys[j];
}

// Orders the winners of one (layer, sequence, KV head) by counting. grid = (ceil(layer_max / 256), Hkv, n_seqs * layers),
// 256 threads: the workgroup owns candidates [blockIdx.x * 256, + 256); lane l of every wavefront holds the four
// candidates l, l + 64, l + 128, l + 192 of them in registers, and wavefront g counts, for each of the four, the
// smaller keys among a quarter of all k keys. One LDS read of a key (the same word for all lanes: a broadcast)
// thus serves 256 comparisons; the four partial counts add up to the rank = the candidate's place in idx_out.
constexpr int kOrderCand = 256;
__global__ __launch_bounds__(256) void select_order_kernel(int Hkv, int w, int layer_max, int n_seqs,
                                                           const int32_t* __restrict__ cu,
                                                           const u64* __restrict__ keys_in0,
                                                           int32_t* __restrict__ idx_out0, int64_t idx_stride_layer) {
  __shared__ __attribute__((aligned(16))) u64 keys[DKV_MAX_LAYER_MAX + 32];
  __shared__ int partial[4][kOrderCand];
  const int seq = blockIdx.z % n_seqs, lz = blockIdx.z / n_seqs;
  const int head = blockIdx.y, tid = threadIdx.x, lane = tid & 63, g = tid >> 6;
  const u64* __restrict__ keys_in = keys_in0 + (int64_t)lz * n_seqs * Hkv * DKV_MAX_LAYER_MAX;
  int32_t* __restrict__ idx_out = idx_out0 + (int64_t)lz * idx_stride_layer;
  const int S = cu[seq + 1] - cu[seq];
  const int n = S > w ? S - w : 0;
  const int k = layer_max < n ? layer_max : n;
  int32_t* __restrict__ out = idx_out + ((int64_t)seq * Hkv + head) * layer_max;
  const int e0 = blockIdx.x * kOrderCand;
  // slots past k hold -1 (each workgroup clears the ones in its own range)
  if (e0 + tid >= k && e0 + tid < layer_max) out[e0 + tid] = -1;
  if (e0 >= k) return;
  const u64* __restrict__ src = keys_in + ((int64_t)seq * Hkv + head) * DKV_MAX_LAYER_MAX;
  // every wavefront scans `quarter` keys (a multiple of 8); the pad keys are the largest value: never "smaller"
  const int quarter = ((k + 3) / 4 + 7) & ~7;
  for (int j = tid; j < 4 * quarter; j += 256) keys[j] = j < k ? src[j] : ~0ull;
  __syncthreads();
  u64 mine[4];
  int smaller[4] = {0, 0, 0, 0};
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int e = e0 + lane + 64 * c;
    mine[c] = e < k ? keys[e] : ~0ull;
  }
  const ulonglong2* __restrict__ kp = reinterpret_cast<const ulonglong2*>(keys + g * quarter);
  for (int j = 0; j < quarter / 2; j += 4) {
    ulonglong2 kk[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) kk[u] = kp[j + u];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        smaller[c] += kk[u].x < mine[c] ? 1 : 0;
        smaller[c] += kk[u].y < mine[c] ? 1 : 0;
      }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) partial[g][lane + 64 * c] = smaller[c];
  __syncthreads();
  const int e = e0 + tid;
  if (e < k) {
    const int rank = partial[0][tid] + partial[1][tid] + partial[2][tid] + partial[3][tid];
    out[rank] = (int32_t)(uint32_t)keys[e];
  }
}

hipError_t launch_select(const Params& p, int layer, int n_layers, const float* scores, int64_t scores_stride_head,
                         int64_t scores_stride_layer, const int32_t* cu, int32_t* idx_out, int64_t idx_stride_layer,
                         int32_t* counts, char* ws, const WorkspaceLayout& wl, hipStream_t st) {
  const size_t lds = 2048 * sizeof(u64) + (size_t)kRadixBins * kHistCopies * sizeof(int);
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_topk_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  u64* keys = reinterpret_cast<u64*>(ws + wl.select_keys);
  launch(DKV_KERNEL_SELECT, select_topk_kernel, dim3(p.Hkv, p.n_seqs, n_layers), dim3(kSelThreads), lds, st, p.Hkv, p.w,
         p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out, idx_stride_layer, counts,
         keys);
  launch(DKV_KERNEL_SELECT_ORDER, select_order_kernel, dim3((p.layer_max + kOrderCand - 1) / kOrderCand, p.Hkv, p.n_seqs * n_layers),
         dim3(256), 0, st, p.Hkv, p.w, p.layer_max, p.n_seqs, cu, keys, idx_out, idx_stride_layer);
  return hipGetLastError();
}

}  // namespace dkv
