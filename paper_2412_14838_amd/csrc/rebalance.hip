// Progressive cache update (Section 4.2, Eq. 4-6; Algorithm 1: Update_Buffer_Length and the truncation loop).
//
// The global top-kg over the concatenated scores of the layers processed so far only matters through its
// per-layer hit counts, so no element is ever moved: a 3-digit radix select (11 + 11 + 10 bits of the fp32
// pattern, scores are >= 0) finds the kg-th largest value T from digit histograms summed over all layers.
//
//   clear   zeroes the histograms of this call.
//   hist0   histogram of the top digit. Within one prefill a layer's scores never change once written, so a caller
//           that names its prefill (a non-zero epoch) lets the histogram stay in the workspace: a call then only
//           adds the layers that the previous call of the same epoch (layers_done - interval, same score tensor,
//           recorded in a small header) had not seen. Epoch 0, or any other history, means a full recount.
//   pick0   digit 0 of T from the top-digit histogram (one workgroup per sequence and update).
//   scan1   histograms the middle digit of the elements that share digit 0 and counts, per layer, the elements
//           whose digit 0 is larger (they are above T).
//   pick1   digit 1 of T from that histogram.
//   scan2   the same one digit down: histograms the last digit (per layer and in total), counts per layer the
//           elements that share digit 0 and have a larger middle digit.
//   final   one workgroup per sequence: digit 2, then cnt_i = #{> T in layer i} + the share of the elements
//           equal to T that the tie rule (lower layer first) gives to layer i, then Z, Z' and counts.
// The scans read the scores as 16-byte vectors, all loads of a workgroup's chunk in flight together.
//
// Several consecutive updates (layers_done, layers_done + interval, ...) can be asked for in one call: they are
// independent of each other except for the final min into `counts`, which commutes. Update u then owns slot u
// of the top-digit histogram: T[u] holds the layers that are new to update u (T[0] additionally the kept
// history), so update u's top-digit histogram is T[0] + ... + T[u]; the next call folds T[1..] into T[0] before
// it starts. The scans read every layer once per call, however many updates cover it: the updates whose
// thresholds agree in the digits found so far form a class (see class_of below), a workgroup keeps its chunk of
// scores in registers, takes it through the classes (usually one) and stores what it finds once per class.
#include "dkv_internal.h"

namespace dkv {

constexpr int kFinalThreads = 1024;
constexpr int kHist0Copies = 4;      // interleaved LDS copies of the top-digit histogram (every element lands there)
constexpr int kHist0Chunk = 8192;    // prefix positions per workgroup, top-digit histogram
constexpr int kScanChunk = 8192;     // prefix positions per workgroup, scans 1 and 2
constexpr int kLowBins = 1024;       // the last digit has 10 bits
constexpr uint32_t kHeaderMagic = 0x646b7631u;

// header[0] magic, [1] layers_done of the last completed call, [2..3] its score tensor, [4] interval, [5] n_seqs,
// [6] total_tokens, [7] updates of that call, [8] its epoch. Layers below the returned value already are in the
// top-digit histogram. Epoch 0 never matches: such a call neither uses nor leaves a history.
__device__ inline int layers_already_counted(const int32_t* __restrict__ header, const float* scores_all,
                                             int layers_done, int interval, int n_seqs, int total_tokens,
                                             uint32_t epoch) {
  const uint64_t ptr = reinterpret_cast<uint64_t>(scores_all);
  const bool same = epoch != 0u && (uint32_t)header[8] == epoch &&
                    (uint32_t)header[0] == kHeaderMagic && header[1] == layers_done - interval &&
                    (uint32_t)header[2] == (uint32_t)ptr && (uint32_t)header[3] == (uint32_t)(ptr >> 32) &&
                    header[4] == interval && header[5] == n_seqs && header[6] == total_tokens;
  return same && layers_done > interval ? layers_done - interval : 0;
}

// always: the per-class blocks of this call (n_updates of them, contiguous: there are at most as many classes as
// updates); tot0: the DKV_MAX_UPDATES slots T[v] of the top-digit histogram, tot0_words each. With a matching history the slots the previous call used (header[7])
// are folded into T[0]; without, T[0] starts from zero. The other slots are zeroed either way.
__global__ __launch_bounds__(256) void rebalance_clear_kernel(uint32_t* __restrict__ always, size_t always_words,
                                                              uint32_t* __restrict__ tot0, size_t tot0_words,
                                                              const int32_t* __restrict__ header,
                                                              const float* scores_all, int layers_done, int interval,
                                                              int n_seqs, int total_tokens, uint32_t epoch,
                                                              int32_t* __restrict__ picks, int picks_words) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < always_words; i += stride) always[i] = 0u;
  // a sequence without prefix positions has no workgroup in the scans that could record its (empty) picks
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < (size_t)picks_words; i += stride) picks[i] = 0;
  const bool keep = layers_already_counted(header, scores_all, layers_done, interval, n_seqs, total_tokens, epoch) != 0;
  int used = keep ? header[7] : 0;
  used = used < 1 ? 1 : (used > DKV_MAX_UPDATES ? DKV_MAX_UPDATES : used);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < tot0_words; i += stride) {
    uint32_t v = 0u;
    if (keep)
      for (int u = 0; u < used; ++u) v += tot0[(size_t)u * tot0_words + i];
    tot0[i] = v;
    for (int u = 1; u < DKV_MAX_UPDATES; ++u) tot0[(size_t)u * tot0_words + i] = 0u;
  }
}

// A workgroup's chunk of one (layer, head, sequence) score row as 16-byte vectors: element e of the score tensor
// is covered by vector e / 4, thread t takes vectors t, t + 256, ... counted from the first one that touches the
// chunk. ok[j] has bit q set when lane q of vector j lies inside the chunk [e_lo, e_hi): 0xf for all but the
// vectors on the chunk's two edges, which the consumers treat element by element.
template <int NV>
struct ChunkVectors {
  uint4 v[NV];
  uint32_t ok[NV];
};

// n_elems: elements of the whole score tensor; its last, partial vector (if any) is read element by element.
template <int NV>
__device__ inline void load_chunk(const float* __restrict__ scores_all, int64_t n_elems, int64_t e_lo, int64_t e_hi,
                                  ChunkVectors<NV>& cv) {
  const uint32_t* __restrict__ base = reinterpret_cast<const uint32_t*>(scores_all);
  const int64_t a_lo = e_lo & ~int64_t(3);
  const uint32_t* __restrict__ row = base + a_lo;
  const int lo_rel = (int)(e_lo - a_lo), hi_rel = (int)(e_hi - a_lo);      // chunk = [lo_rel, hi_rel) from a_lo
  const int64_t whole = (n_elems & ~int64_t(3)) - a_lo;                    // vectors below this are whole
  const int whole_rel = whole > (int64_t)0x7fffffff ? 0x7fffffff : (int)whole;
#pragma unroll
  for (int j = 0; j < NV; ++j) cv.v[j] = make_uint4(0, 0, 0, 0);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int rel = 4 * (threadIdx.x + 256 * j);
    int first = lo_rel - rel, last = hi_rel - rel;                         // valid lanes [first, last) of 0..4
    first = first < 0 ? 0 : (first > 4 ? 4 : first);
    last = last < 0 ? 0 : (last > 4 ? 4 : last);
    const uint32_t ok = last > first ? ((1u << last) - 1u) & ~((1u << first) - 1u) : 0u;
    cv.ok[j] = ok;
    if (ok) {
      if (rel + 4 <= whole_rel) {
        cv.v[j] = *reinterpret_cast<const uint4*>(row + rel);
      } else {                                                             // the tensor's last, partial vector
        uint32_t e[4] = {0, 0, 0, 0};
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (ok >> q & 1) e[q] = row[rel + q];
        cv.v[j] = make_uint4(e[0], e[1], e[2], e[3]);
      }
    }
  }
}

__device__ inline uint32_t lane_of(const uint4& v, int q) { return q == 0 ? v.x : (q == 1 ? v.y : (q == 2 ? v.z : v.w)); }

// A thread's share of a histogram of NB bins for a workgroup of NT threads: thread t owns the NB / NT bins just
// below those of thread t - 1 (thread 0 the top ones).
template <int NT, int NB>
struct Bins {
  int c[NB / NT];
};

template <int NT, int NB>
__device__ inline Bins<NT, NB> load_bins(const int32_t* __restrict__ tot) {
  constexpr int PER = NB / NT;
  Bins<NT, NB> b;
  const int base = NB - PER * ((int)threadIdx.x + 1);
#pragma unroll
  for (int i = 0; i < PER; ++i) b.c[i] = tot[base + i];
  return b;
}

// The same, summed over the first n_slots histograms (slot stride in ints).
template <int NT, int NB>
__device__ inline Bins<NT, NB> load_bins_sum(const int32_t* __restrict__ tot, int n_slots, int64_t slot_stride) {
  Bins<NT, NB> b = load_bins<NT, NB>(tot);
  for (int u = 1; u < n_slots; ++u) {
    const Bins<NT, NB> x = load_bins<NT, NB>(tot + u * slot_stride);
#pragma unroll
    for (int i = 0; i < NB / NT; ++i) b.c[i] += x.c[i];
  }
  return b;
}

// The digit that holds the rem-th largest element of the histogram, and the rank that remains inside it (both 0
// when rem <= 0). scratch: NT / 64 ints, sh: 2 ints (LDS). Starts and ends with a barrier.
template <int NT, int NB>
__device__ inline void pick_digit(const Bins<NT, NB>& bins, int rem, int* scratch, int* sh, int& digit, int& rem_out) {
  constexpr int PER = NB / NT;
  const int tid = threadIdx.x;
  const int base = NB - PER * (tid + 1);
  int sum = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) sum += bins.c[i];
  if (tid == 0) { sh[0] = 0; sh[1] = 0; }
  int all;
  const int above = block_prefix_sum(sum, scratch, all);    // two barriers: sh is cleared before the owner writes
  if (rem > 0 && above < rem && rem <= above + sum) {      // exactly one thread owns the bin
    int a = above;
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
      if (rem > a && rem <= a + bins.c[i]) { sh[0] = base + i; sh[1] = rem - a; }
      a += bins.c[i];
    }
  }
  __syncthreads();
  digit = sh[0];
  rem_out = sh[1];
  __syncthreads();                                          // scratch and sh may be reused
}

__device__ inline int global_k(const int32_t* __restrict__ cu, int seq, int w, int Hkv, int mean_budget,
                               int layers_done) {
  const int len = cu[seq + 1] - cu[seq];
  const long long n = len > w ? len - w : 0;
  const long long want = (long long)mean_budget * Hkv * layers_done;
  const long long have = n * Hkv * layers_done;
  return (int)(want < have ? want : have);                  // kg of Eq. 4, clamped to the population
}

// Top-digit histogram of the layers not yet counted. grid = (chunk upper bound, Hkv, layers_done), 256 threads.
// layers_done: of the call's first update; layers at or past it belong to the later updates' slots.
__global__ __launch_bounds__(256) void rebalance_hist0_kernel(int n_seqs, int Hkv, int w, int L, int total_tokens,
                                                              int layers_done, int interval,
                                                              const float* __restrict__ scores_all,
                                                              const int32_t* __restrict__ cu,
                                                              const int32_t* __restrict__ header, uint32_t epoch,
                                                              int32_t* __restrict__ tot0, int64_t tot0_words) {
  __shared__ int h[kRadixBins * kHist0Copies];
  const int head = blockIdx.y, layer = blockIdx.z;
  if (layer < layers_already_counted(header, scores_all, layers_done, interval, n_seqs, total_tokens, epoch)) return;
  const int slot = layer < layers_done ? 0 : 1 + (layer - layers_done) / interval;
  int seq, c, begin, len;
  if (!find_chunk(cu, n_seqs, kHist0Chunk, w, blockIdx.x, seq, c, begin, len)) return;
  const int n = len - w;
  const int i0 = c * kHist0Chunk;
  const int i1 = i0 + kHist0Chunk < n ? i0 + kHist0Chunk : n;
  constexpr int NV = kHist0Chunk / 4 / 256 + 1;
  ChunkVectors<NV> cv;
  const int64_t e_lo = ((int64_t)layer * Hkv + head) * total_tokens + begin + i0;
  load_chunk<NV>(scores_all, (int64_t)L * Hkv * total_tokens, e_lo, e_lo + (i1 - i0), cv);
  for (int b = threadIdx.x; b < kRadixBins * kHist0Copies; b += 256) h[b] = 0;
  __syncthreads();
  int* __restrict__ hc = h + (threadIdx.x & (kHist0Copies - 1));
  // Scores crowd into a few top digits (a quarter of an octave each) and pooling repeats values along a row, so a
  // thread mostly meets the digit it met last: runs of equal digits are counted in a register and cost one LDS
  // atomic per run instead of one per element.
  uint32_t run_digit = 0;
  int run = 0;
  auto count = [&](uint32_t u) {
    const uint32_t d = u >> 21;
    if (d != run_digit) {
      if (run) atomicAdd(&hc[run_digit * kHist0Copies], run);
      run_digit = d;
      run = 0;
    }
    ++run;
  };
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    if (cv.ok[j] == 0xf) {
      count(cv.v[j].x);
      count(cv.v[j].y);
      count(cv.v[j].z);
      count(cv.v[j].w);
    } else if (cv.ok[j]) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (cv.ok[j] >> q & 1) count(lane_of(cv.v[j], q));
    }
  }
  if (run) atomicAdd(&hc[run_digit * kHist0Copies], run);
  __syncthreads();
  int32_t* __restrict__ g = tot0 + slot * tot0_words + (int64_t)seq * kRadixBins;
  for (int b = threadIdx.x; b < kRadixBins; b += 256) {
    int v = 0;
#pragma unroll
    for (int c2 = 0; c2 < kHist0Copies; ++c2) v += h[b * kHist0Copies + c2];
    if (v) atomicAdd(&g[b], v);
  }
}

// Classes. Update u of a call covers the layers [0, layers_done + u * interval); a layer is new to update
// f = first_update(layer) and is covered by the updates f .. n_updates - 1. Among those, the updates whose
// thresholds agree in the digits found so far (`key`) see exactly the same elements of the layer: they form a
// class, named by its first member, class_of(key, f, u) = min {v in [f, u] : key[v] == key[u]}. What a scan
// finds for a class is stored once, under the class's name (block `class * always_words`) and the slot f (sums
// over layers) or the layer itself; whoever needs update u's figures asks for class_of(.., f, u) again.
__device__ inline int class_of(const uint32_t* key, int f, int u) {
  const uint32_t k = key[u];
  for (int v = f; v < u; ++v)
    if (key[v] == k) return v;
  return u;
}

__device__ inline int first_update_of(int layer, int layers_done, int interval) {
  return layer < layers_done ? 0 : (layer - layers_done) / interval + 1;
}

// picks[(update * n_seqs + seq) * 4 + ..]: digit 0 of the update's threshold, rank left inside it, digit 1, rank
// left inside that. grid = (n_seqs, n_updates), kFinalThreads threads; layers_done comes in as the first update's.
//   LEVEL 0 (after hist0): from the top-digit histograms; LEVEL 1 (after scan 1): from the classes' tot1 slots.
template <int LEVEL>
__global__ __launch_bounds__(kFinalThreads) void rebalance_pick_kernel(int n_seqs, int w, int Hkv, int mean_budget,
                                                                       int layers_done, int interval,
                                                                       const int32_t* __restrict__ cu,
                                                                       const int32_t* __restrict__ tot0, int64_t tot0_words,
                                                                       const int32_t* __restrict__ tot1, int64_t always_words,
                                                                       int32_t* __restrict__ picks) {
  __shared__ int scratch[kFinalThreads / 64];
  __shared__ int sh[2];
  __shared__ uint32_t key[DKV_MAX_UPDATES];
  const int seq = blockIdx.x, update = blockIdx.y, n_updates = gridDim.y;
  int32_t* __restrict__ mine = picks + ((int64_t)update * n_seqs + seq) * 4;
  Bins<kFinalThreads, kRadixBins> bins;
  int rem;
  if (LEVEL == 0) {
    bins = load_bins_sum<kFinalThreads, kRadixBins>(tot0 + (int64_t)seq * kRadixBins, update + 1, tot0_words);
    rem = global_k(cu, seq, w, Hkv, mean_budget, layers_done + update * interval);
  } else {
    if (threadIdx.x < n_updates) key[threadIdx.x] = (uint32_t)picks[((int64_t)threadIdx.x * n_seqs + seq) * 4];
    __syncthreads();
    // the layers new to update f, as the class of this update saw them; all slots are requested before the first wait
    Bins<kFinalThreads, kRadixBins> x[DKV_MAX_UPDATES];
#pragma unroll
    for (int f = 0; f < DKV_MAX_UPDATES; ++f)
      if (f <= update)
        x[f] = load_bins<kFinalThreads, kRadixBins>(tot1 + class_of(key, f, update) * always_words +
                                                    ((int64_t)seq * DKV_MAX_UPDATES + f) * kRadixBins);
    rem = mine[1];
#pragma unroll
    for (int i = 0; i < kRadixBins / kFinalThreads; ++i) bins.c[i] = 0;
#pragma unroll
    for (int f = 0; f < DKV_MAX_UPDATES; ++f)
      if (f <= update)
#pragma unroll
        for (int i = 0; i < kRadixBins / kFinalThreads; ++i) bins.c[i] += x[f].c[i];
  }
  int digit, left;
  pick_digit<kFinalThreads, kRadixBins>(bins, rem, scratch, sh, digit, left);
  if (threadIdx.x == 0) { mine[2 * LEVEL] = digit; mine[2 * LEVEL + 1] = left; }
}

// Scans 1 and 2. grid = (chunk upper bound, Hkv, layers of the call's last update), 256 threads. A workgroup reads
// its chunk of one layer's scores once and takes it through the classes of the updates that cover the layer
// (usually one: T moves little from one update to the next):
//   PASS 1: histogram of the middle digit over elements with digit 0 == d0 -> tot1 (slot of the layer);
//           above[0][layer] += #{digit 0 > d0}
//   PASS 2: histogram of the last digit over elements with digits (0, 1) == (d0, d1) -> tot2 (slot of the layer) and
//           hist2[layer]; above[1][layer] += #{digit 0 == d0, digit 1 > d1}
// with (d0, d1) of the updates from `picks`. tot1 .. above point at class 0's block.
// PICKS_HERE (calls of a single update): no pick kernel ran; every workgroup finds the digit this scan needs by itself
// from the histogram the kernel before completed (the top digit from tot0, the middle digit from tot1: 8 KB from
// the L2, while its scores are on their way), and the sequence's first workgroup records it in `picks` for the
// kernels behind.
template <int PASS, bool PICKS_HERE>
__global__ __launch_bounds__(256) void rebalance_scan_kernel(int n_seqs, int Hkv, int w, int L, int total_tokens,
                                                             int layers_done, int interval, int n_updates,
                                                             int mean_budget, const int32_t* __restrict__ tot0,
                                                             const float* __restrict__ scores_all,
                                                             const int32_t* __restrict__ cu,
                                                             int32_t* __restrict__ picks,
                                                             int32_t* __restrict__ tot1, int32_t* __restrict__ tot2,
                                                             int32_t* __restrict__ hist2, int32_t* __restrict__ above,
                                                             int64_t always_words) {
  constexpr int BINS = PASS == 1 ? kRadixBins : kLowBins;
  // classes taken through the chunk together: PASS 1 usually has one (the top digit of T rarely moves between the
  // updates of a call), PASS 2 often one per update (the middle digit does), and its histograms are small
  constexpr int ROUND = PASS == 1 ? 1 : DKV_MAX_UPDATES;
  __shared__ int h[ROUND * BINS];
  __shared__ uint32_t key_of[DKV_MAX_UPDATES];        // the digits of the updates' thresholds found so far
  __shared__ int cls_update[DKV_MAX_UPDATES];         // the classes of the updates that cover this layer (first members)
  __shared__ int n_cls;
  __shared__ int n_above[ROUND];
  int seq, c, begin, len;
  if (!find_chunk(cu, n_seqs, kScanChunk, w, blockIdx.x, seq, c, begin, len)) return;
  const int head = blockIdx.y, layer = blockIdx.z;
  const int first_update = first_update_of(layer, layers_done, interval);   // < n_updates by the grid
  const int n = len - w;
  const int i0 = c * kScanChunk;
  const int i1 = i0 + kScanChunk < n ? i0 + kScanChunk : n;
  constexpr int NV = kScanChunk / 4 / 256 + 1;
  ChunkVectors<NV> cv;
  const int64_t e_lo = ((int64_t)layer * Hkv + head) * total_tokens + begin + i0;
  load_chunk<NV>(scores_all, (int64_t)L * Hkv * total_tokens, e_lo, e_lo + (i1 - i0), cv);
  if (PICKS_HERE) {                                      // n_updates == 1: update 0, class 0, slot 0
    __shared__ int pick_scratch[256 / 64];
    __shared__ int pick_sh[2];
    int32_t* __restrict__ pk = picks + (int64_t)seq * 4;
    const Bins<256, kRadixBins> bins = load_bins<256, kRadixBins>(
        PASS == 1 ? tot0 + (int64_t)seq * kRadixBins : tot1 + (int64_t)seq * DKV_MAX_UPDATES * kRadixBins);
    const int rem = PASS == 1 ? global_k(cu, seq, w, Hkv, mean_budget, layers_done) : pk[1];
    const int d_top = PASS == 1 ? 0 : pk[0];
    int digit, left;
    pick_digit<256, kRadixBins>(bins, rem, pick_scratch, pick_sh, digit, left);
    if (threadIdx.x == 0) {
      key_of[0] = PASS == 1 ? (uint32_t)digit : (((uint32_t)d_top << 11) | (uint32_t)digit);
      if (c == 0 && head == 0 && layer == 0) { pk[2 * (PASS - 1)] = digit; pk[2 * (PASS - 1) + 1] = left; }
    }
  } else if (threadIdx.x < n_updates) {
    const int32_t* __restrict__ pk = picks + ((int64_t)threadIdx.x * n_seqs + seq) * 4;
    key_of[threadIdx.x] = PASS == 1 ? (uint32_t)pk[0] : (((uint32_t)pk[0] << 11) | (uint32_t)pk[2]);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int k = 0;
    for (int update = first_update; update < n_updates; ++update)
      if (class_of(key_of, first_update, update) == update) cls_update[k++] = update;
    n_cls = k;
  }
  __syncthreads();
  const int classes = n_cls;
  // PASS 1 looks at the top digit p = u >> 21, PASS 2 at the top two p = u >> 10; an element is "above" when
  // p lies in (key, end): PASS 1 any larger top digit, PASS 2 a larger middle digit under the same top digit.
  constexpr int SH = PASS == 1 ? 21 : 10;
  auto bin_of = [](uint32_t u) { return PASS == 1 ? ((u >> 10) & (uint32_t)(kRadixBins - 1)) : (u & (uint32_t)(kLowBins - 1)); };
  for (int c0 = 0; c0 < classes; c0 += ROUND) {
    const int in_round = classes - c0 < ROUND ? classes - c0 : ROUND;
    for (int b = threadIdx.x; b < in_round * BINS; b += 256) h[b] = 0;
    if (threadIdx.x < ROUND) n_above[threadIdx.x] = 0;
    __syncthreads();
    int mine[ROUND];
#pragma unroll
    for (int r = 0; r < ROUND; ++r) mine[r] = 0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (cv.ok[j] == 0xf) {
        const uint32_t p0 = cv.v[j].x >> SH, p1 = cv.v[j].y >> SH, p2 = cv.v[j].z >> SH, p3 = cv.v[j].w >> SH;
#pragma unroll
        for (int r = 0; r < ROUND; ++r) {
          if (r >= in_round) break;
          const uint32_t key = key_of[cls_update[c0 + r]];
          const uint32_t end = PASS == 1 ? (uint32_t)kRadixBins : (((key >> 11) + 1u) << 11);
          const uint32_t span = end - key - 1u;   // p in (key, end)  <=>  p - key - 1 < span (unsigned)
          mine[r] += (p0 - key - 1u < span) + (p1 - key - 1u < span) + (p2 - key - 1u < span) + (p3 - key - 1u < span);
          if (p0 == key || p1 == key || p2 == key || p3 == key) {       // one branch per vector and class
            int* __restrict__ hr = h + r * BINS;
            if (p0 == key) atomicAdd(&hr[bin_of(cv.v[j].x)], 1);
            if (p1 == key) atomicAdd(&hr[bin_of(cv.v[j].y)], 1);
            if (p2 == key) atomicAdd(&hr[bin_of(cv.v[j].z)], 1);
            if (p3 == key) atomicAdd(&hr[bin_of(cv.v[j].w)], 1);
          }
        }
      } else if (cv.ok[j]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (!(cv.ok[j] >> q & 1)) continue;
          const uint32_t u = lane_of(cv.v[j], q), pq = u >> SH;
#pragma unroll
          for (int r = 0; r < ROUND; ++r) {
            if (r >= in_round) break;
            const uint32_t key = key_of[cls_update[c0 + r]];
            const uint32_t end = PASS == 1 ? (uint32_t)kRadixBins : (((key >> 11) + 1u) << 11);
            mine[r] += pq - key - 1u < end - key - 1u;
            if (pq == key) atomicAdd(&h[r * BINS + bin_of(u)], 1);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < ROUND; ++r) {
      if (r >= in_round) break;
      const int m = wave_sum(mine[r]);
      if ((threadIdx.x & 63) == 0 && m) atomicAdd(&n_above[r], m);
    }
    __syncthreads();
    const int64_t slot = (int64_t)seq * DKV_MAX_UPDATES + first_update;
    for (int r = 0; r < in_round; ++r) {
      const int64_t cls = (int64_t)cls_update[c0 + r] * always_words;   // the class's block
      if (threadIdx.x == 0 && n_above[r])
        atomicAdd(&above[cls + ((int64_t)(PASS - 1) * n_seqs + seq) * L + layer], n_above[r]);
      for (int b = threadIdx.x; b < BINS; b += 256) {
        const int v = h[r * BINS + b];
        if (!v) continue;
        if (PASS == 1) {
          atomicAdd(&tot1[cls + slot * kRadixBins + b], v);
        } else {
          atomicAdd(&tot2[cls + slot * kLowBins + b], v);
          atomicAdd(&hist2[cls + ((int64_t)seq * L + layer) * kLowBins + b], v);
        }
      }
    }
    __syncthreads();                                                    // h and n_above are reused by the next round
  }
}

// Exclusive prefix sum and total of one int per thread over the kFinalThreads threads.
__device__ inline int block_exclusive_scan_final(int v, int* scratch, int& total) {
  return block_prefix_sum(v, scratch, total);
}

// Last digit, per-layer hit counts and the budget arithmetic of Eq. 5-6, one workgroup per sequence.
// grid = (n_seqs, n_updates): blockIdx.y is the update, layers_done comes in as the first update's.
__global__ __launch_bounds__(kFinalThreads) void rebalance_final_kernel(
    int n_seqs, int L, int layers_done, int interval, int w, int Hkv, int mean_budget, int layer_max, int total_tokens,
    const float* scores_all, const int32_t* __restrict__ cu, const int32_t* __restrict__ picks,
    const int32_t* __restrict__ tot2, const int32_t* __restrict__ hist2, const int32_t* __restrict__ above,
    int64_t always_words, int32_t* __restrict__ header, uint32_t epoch, int32_t* __restrict__ counts,
    int32_t* __restrict__ budgets_out, int32_t* __restrict__ hits_out, int64_t out_stride_update) {
  const int update = blockIdx.y, n_updates = gridDim.y;
  const int first_done = layers_done;                  // of the call's first update: it fixes the slots of the layers
  layers_done += update * interval;
  if (budgets_out) budgets_out += update * out_stride_update;
  if (hits_out) hits_out += update * out_stride_update;
  static_assert(DKV_MAX_LAYERS <= kFinalThreads, "one layer per thread");
  __shared__ int scratch[kFinalThreads / 64];
  __shared__ int sh[2];
  __shared__ int gt[DKV_MAX_LAYERS];
  __shared__ int eq[DKV_MAX_LAYERS];
  __shared__ int wave_max_s[kFinalThreads / 64];
  __shared__ uint32_t key1[DKV_MAX_UPDATES], key2[DKV_MAX_UPDATES];   // digit 0, digits (0, 1) of the updates' thresholds
  const int seq = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int kg = global_k(cu, seq, w, Hkv, mean_budget, layers_done);
  if (tid < n_updates) {
    const int32_t* __restrict__ pk = picks + ((int64_t)tid * n_seqs + seq) * 4;
    key1[tid] = (uint32_t)pk[0];
    key2[tid] = ((uint32_t)pk[0] << 11) | (uint32_t)pk[2];
  }
  __syncthreads();
  // last-digit histogram of this update: the slots of the layers it covers, each from the class this update is in
  // (all reads are requested before the first wait)
  Bins<kFinalThreads, kLowBins> slot2[DKV_MAX_UPDATES];
#pragma unroll
  for (int f = 0; f < DKV_MAX_UPDATES; ++f)
    if (f <= update)
      slot2[f] = load_bins<kFinalThreads, kLowBins>(tot2 + class_of(key2, f, update) * always_words +
                                                    ((int64_t)seq * DKV_MAX_UPDATES + f) * kLowBins);
  constexpr int kWaves = kFinalThreads / 64, kPerLane = kLowBins / 64;
  // the first layer of this wavefront, requested before the first wait: lane l holds last-digit bins l, l + 64, ...
  // (later layers are read in the loop)
  int first[kPerLane];
  {
    const int i = wv < layers_done ? wv : 0;
    const int cls = class_of(key2, first_update_of(i, first_done, interval), update);
    const int32_t* __restrict__ g = hist2 + cls * always_words + ((int64_t)seq * L + i) * kLowBins;
#pragma unroll
    for (int r = 0; r < kPerLane; ++r) first[r] = g[lane + 64 * r];
  }
  int above_mine = 0;
  if (tid < layers_done) {
    const int f = first_update_of(tid, first_done, interval);
    above_mine = above[class_of(key1, f, update) * always_words + ((int64_t)0 * n_seqs + seq) * L + tid] +
                 above[class_of(key2, f, update) * always_words + ((int64_t)1 * n_seqs + seq) * L + tid];
  }
  int rem = picks[((int64_t)update * n_seqs + seq) * 4 + 3], d2;      // rank left inside the digits (0, 1)
  Bins<kFinalThreads, kLowBins> bins2;
#pragma unroll
  for (int i = 0; i < kLowBins / kFinalThreads; ++i) bins2.c[i] = 0;
#pragma unroll
  for (int f = 0; f < DKV_MAX_UPDATES; ++f)
    if (f <= update)
#pragma unroll
      for (int i = 0; i < kLowBins / kFinalThreads; ++i) bins2.c[i] += slot2[f].c[i];
  pick_digit<kFinalThreads, kLowBins>(bins2, rem, scratch, sh, d2, rem);
  const int need_eq = rem;   // elements equal to T that belong to the top-kg
  // per layer: elements above T = those counted by the scans (a higher digit is larger) + the last-digit bins
  // above the chosen one; equal to T = the chosen last-digit bin
  for (int i = wv; i < layers_done; i += kWaves) {
    int acc = 0, at = 0;
    const int cls = class_of(key2, first_update_of(i, first_done, interval), update);
    const int32_t* __restrict__ g = hist2 + cls * always_words + ((int64_t)seq * L + i) * kLowBins;
#pragma unroll
    for (int r = 0; r < kPerLane; ++r) {
      const int b = lane + 64 * r;
      const int v = i == wv ? first[r] : g[b];
      acc += b > d2 ? v : 0;
      at += b == d2 ? v : 0;
    }
    acc = wave_sum(acc);
    at = wave_sum(at);
    if (lane == 0) { gt[i] = acc; eq[i] = at; }
  }
  __syncthreads();
  // Phi: ties go to the lower flat index, i.e. earlier layers first: layer i takes what the earlier layers left
  const bool live = tid < layers_done;
  const int my_eq = live ? eq[tid] : 0;
  int eq_total;
  const int eq_before = block_exclusive_scan_final(my_eq, scratch, eq_total);
  int left = need_eq - eq_before;
  left = left > 0 ? left : 0;
  const int cnt = live && kg > 0 ? gt[tid] + above_mine + (my_eq < left ? my_eq : left) : 0;
  const int m = wave_max(cnt);   // max over layers
  if (lane == 0) wave_max_s[wv] = m;
  __syncthreads();
  int cmax = 0;
  for (int i = 0; i < kFinalThreads / 64; ++i) cmax = wave_max_s[i] > cmax ? wave_max_s[i] : cmax;
  const int z = cmax > 0 ? (int)(((long long)layer_max * cnt) / cmax) : 0;          // Eq. 5, exact floor
  int zsum_i;
  (void)block_exclusive_scan_final(z, scratch, zsum_i);                               // <= layer_max * layers: fits
  const long long zsum = zsum_i;
  const long long B = (long long)mean_budget * L;                                     // Eq. 6: B = (wt - ws) * L
  if (live) {
    const long long zp = zsum > 0 ? ((long long)z * B) / zsum : 0;                    // exact floor
    const int zpi = zp > 0x7fffffffLL ? 0x7fffffff : (int)zp;
    if (budgets_out) budgets_out[seq * L + tid] = zpi;
    if (hits_out) hits_out[seq * L + tid] = cnt;
    atomicMin(&counts[seq * L + tid], zpi);       // truncation never grows a layer; the updates of a call commute
  }
  if (seq == 0 && tid == 0 && update == n_updates - 1) {   // this call's layers are in the top-digit histograms now
    const uint64_t ptr = reinterpret_cast<uint64_t>(scores_all);
    header[0] = (int32_t)kHeaderMagic; header[1] = layers_done;
    header[2] = (int32_t)(uint32_t)ptr; header[3] = (int32_t)(uint32_t)(ptr >> 32);
    header[4] = interval; header[5] = n_seqs; header[6] = total_tokens; header[7] = n_updates;
    header[8] = (int32_t)epoch;
  }
}

// layers_done: of the first update; update u of the n_updates covers layers [0, layers_done + u * interval).
// budgets_out / hits_out (may be null): update u writes its block out_stride_update ints after update u - 1's.
hipError_t launch_rebalance(const Params& p, int layers_done, int n_updates, uint32_t epoch, const float* scores_all,
                            const int32_t* cu, int32_t* counts, int32_t* budgets_out, int32_t* hits_out,
                            int64_t out_stride_update, char* ws, const WorkspaceLayout& wl, hipStream_t st) {
  int32_t* header = reinterpret_cast<int32_t*>(ws + wl.header);
  int32_t* tot0 = reinterpret_cast<int32_t*>(ws + wl.tot0);
  int32_t* tot1 = reinterpret_cast<int32_t*>(ws + wl.tot1);
  int32_t* tot2 = reinterpret_cast<int32_t*>(ws + wl.tot2);
  int32_t* hist2 = reinterpret_cast<int32_t*>(ws + wl.hist2);
  int32_t* above = reinterpret_cast<int32_t*>(ws + wl.above);
  int32_t* picks = reinterpret_cast<int32_t*>(ws + wl.picks);
  // tot1 .. above of a class of updates are one contiguous block, the blocks follow each other: as many as the call
  // has updates are cleared; the top-digit slots are folded or cleared according to the history
  const int64_t always_words = (int64_t)(wl.update_block_bytes / 4), tot0_words = (int64_t)(wl.tot0_slot_bytes / 4);
  const size_t clear_words = (size_t)always_words * n_updates;
  size_t blocks = (clear_words + 255) / 256;
  blocks = blocks > 1024 ? 1024 : blocks;
  launch(DKV_KERNEL_FILL, rebalance_clear_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
         reinterpret_cast<uint32_t*>(tot1), clear_words, reinterpret_cast<uint32_t*>(tot0), (size_t)tot0_words, header,
         scores_all, layers_done, p.interval, p.n_seqs, p.total_tokens, epoch, picks, n_updates * p.n_seqs * 4);
  const int last_done = layers_done + (n_updates - 1) * p.interval;
  const dim3 grid0(p.total_tokens / kHist0Chunk + p.n_seqs, p.Hkv, last_done);
  launch(DKV_KERNEL_REBALANCE_HIST, rebalance_hist0_kernel, grid0, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L,
         p.total_tokens, layers_done, p.interval, scores_all, cu, header, epoch, tot0, tot0_words);
  const dim3 grid_pick(p.n_seqs, n_updates);
  const dim3 grid(p.total_tokens / kScanChunk + p.n_seqs, p.Hkv, last_done);
  if (n_updates == 1) {     // the scans pick their digits themselves: two launches less
    launch(DKV_KERNEL_REBALANCE_SCAN, (rebalance_scan_kernel<1, true>), grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L,
           p.total_tokens, layers_done, p.interval, n_updates, p.mean_budget, tot0, scores_all, cu, picks, tot1, tot2, hist2,
           above, always_words);
    launch(DKV_KERNEL_REBALANCE_SCAN, (rebalance_scan_kernel<2, true>), grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L,
           p.total_tokens, layers_done, p.interval, n_updates, p.mean_budget, tot0, scores_all, cu, picks, tot1, tot2, hist2,
           above, always_words);
  } else {
    launch(DKV_KERNEL_REBALANCE_PICK, rebalance_pick_kernel<0>, grid_pick, dim3(kFinalThreads), 0, st, p.n_seqs, p.w, p.Hkv,
           p.mean_budget, layers_done, p.interval, cu, tot0, tot0_words, tot1, always_words, picks);
    launch(DKV_KERNEL_REBALANCE_SCAN, (rebalance_scan_kernel<1, false>), grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L,
           p.total_tokens, layers_done, p.interval, n_updates, p.mean_budget, tot0, scores_all, cu, picks, tot1, tot2, hist2,
           above, always_words);
    launch(DKV_KERNEL_REBALANCE_PICK, rebalance_pick_kernel<1>, grid_pick, dim3(kFinalThreads), 0, st, p.n_seqs, p.w, p.Hkv,
           p.mean_budget, layers_done, p.interval, cu, tot0, tot0_words, tot1, always_words, picks);
    launch(DKV_KERNEL_REBALANCE_SCAN, (rebalance_scan_kernel<2, false>), grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L,
           p.total_tokens, layers_done, p.interval, n_updates, p.mean_budget, tot0, scores_all, cu, picks, tot1, tot2, hist2,
           above, always_words);
  }
  launch(DKV_KERNEL_REBALANCE_FINAL, rebalance_final_kernel, dim3(p.n_seqs, n_updates), dim3(kFinalThreads), 0, st,
         p.n_seqs, p.L, layers_done, p.interval, p.w, p.Hkv, p.mean_budget, p.layer_max, p.total_tokens, scores_all, cu,
         picks, tot2, hist2, above, always_words, header, epoch, counts, budgets_out, hits_out, out_stride_update);
  return hipGetLastError();
}

}  // namespace dkv
