// Per-layer, per-KV-head top-k (Eq. 3; Algorithm 1: indices <- A^l.topk(B^l, dim=-1).indices).
// One workgroup per (layer, sequence, KV head):
//   1. LDS radix-select (3 digits of 11/11/10 bits of the fp32 pattern; scores are >= 0 so patterns order like
//      values) finds the k-th largest score T. The digit histogram is kept in 8 interleaved copies so that
//      lanes whose scores share a digit do not serialise on one LDS word.
//   2. wavefront-ballot compaction collects the winners as 64-bit keys (~score bits, position) in LDS: everything
//      above T, and the first (k - #above) elements equal to T in position order (ties go to the lower position).
//   3. the k winners are ordered by (score descending, position ascending) = ascending key: bucketed by the
//      leading bits of their scores, the buckets laid out by a scan, the few keys of a bucket ranked by counting.
// Short path (rows that fit the registers, final lists): after two digits the elements that can still win are the
// ones above those 22 bits plus the few that share them; when they fit (4096), steps 1-2 stop there, all of them
// become keys, step 3 orders them and writes the first k. The result is the same list bit for bit.
// Prefix sums and reductions over the workgroup go through DPP moves (see dkv_internal.h).
//
// Rows longer than the 32768 positions a workgroup keeps in registers are selected in two levels, each the same
// kernel: level 1 cuts the row into segments of 32768 positions, one workgroup per segment, and leaves every
// segment's own top-k (score and position, in POSITION order) in the workspace; level 2 selects the top-k of those
// candidates with one workgroup per row. Every element of a row's top-k is in its segment's top-k, and both levels
// break ties toward the lower position (the candidates lie in position order), so the result is the single-level
// one bit for bit; a row of a million positions costs its segments' parallel passes plus one pass over 63 488
// candidates instead of a serial walk over the whole row by one workgroup.
#include "dkv_internal.h"

namespace dkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kHistCopies = 8;
constexpr int kSelPerThread = 32;                              // row positions a thread keeps in registers
constexpr int kSelResident = kSelPerThread * kSelThreads;      // 32768 positions
static_assert(kSelResident == kSelectSegment, "the workspace is sized for segments of what one workgroup holds");

constexpr int kShortCap = 4096;                                // candidates the short path orders (see below)
constexpr int kOrderPerThread = kShortCap / kSelThreads;       // keys a thread takes through the ordering step

typedef unsigned long long u64;

// Exclusive prefix sum over the kSelThreads threads of the workgroup. `scratch` holds kSelWaves ints.
__device__ inline int block_exclusive_scan(int v, int* scratch) {
  int total;
  return block_prefix_sum(v, scratch, total);
}

// Minimum and maximum of one value per lane over the wavefront (DPP inside the rows of 16 lanes, then the four rows).
template <int CTRL>
__device__ inline uint32_t dpp_lane_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
__device__ inline void wave_min_max(uint32_t& lo, uint32_t& hi) {
#define DKV_MINMAX_STEP(CTRL)                                  \
  {                                                            \
    const uint32_t l2 = dpp_lane_u32<CTRL>(lo), h2 = dpp_lane_u32<CTRL>(hi); \
    lo = l2 < lo ? l2 : lo;                                    \
    hi = h2 > hi ? h2 : hi;                                    \
  }
  DKV_MINMAX_STEP(0xB1) DKV_MINMAX_STEP(0x4E) DKV_MINMAX_STEP(0x141) DKV_MINMAX_STEP(0x140)
#undef DKV_MINMAX_STEP
  uint32_t l = (uint32_t)__builtin_amdgcn_readlane((int)lo, 0), h = (uint32_t)__builtin_amdgcn_readlane((int)hi, 0);
#pragma unroll
  for (int r = 16; r < 64; r += 16) {
    const uint32_t l2 = (uint32_t)__builtin_amdgcn_readlane((int)lo, r), h2 = (uint32_t)__builtin_amdgcn_readlane((int)hi, r);
    l = l2 < l ? l2 : l;
    h = h2 > h ? h2 : h;
  }
  lo = l;
  hi = h;
}

// Candidates of the two-level selection: segment g of row r (r = (layer of the call * n_seqs + seq) * Hkv + head) owns
// entries [r * cand_stride + g * layer_max, + its k) of cand_val (score bit patterns) and cand_pos (positions).
struct SelectCandidates {
  uint32_t* val;
  int32_t* pos;
  int64_t stride;      // entries per row: segments_max * layer_max
  int segments_max;    // segments of the longest row the descriptor admits
};

enum { kSelDirect = 0, kSelSegments = 1, kSelMerge = 2 };

// Candidates a row of n positions leaves behind level 1: layer_max per full segment, min(layer_max, rest) for the last.
__host__ __device__ inline int candidates_of(int n, int layer_max) {
  const int full = n / kSelResident, rest = n - full * kSelResident;
  return full * (layer_max < kSelResident ? layer_max : kSelResident) + (rest < layer_max ? rest : layer_max);
}

// grid = (Hkv, n_seqs [x segments_max for MODE == kSelSegments], layers of the call); blockIdx.z picks the layer: its
// scores, index list and key block lie blockIdx.z layer strides behind the pointers passed in.
// PER: row positions a thread keeps in registers: 32 (rows and segments of up to 32768 positions), or 16 / 8 when no
// row of the call is longer than 16384 / 8192 (the passes over the registers are that much shorter).
template <int MODE, int PER>
__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(int Hkv, int w, int layer_max, int L, int layer0,
                                                                  const float* __restrict__ scores0,
                                                                  int64_t scores_stride_head,
                                                                  int64_t scores_stride_layer,
                                                                  const int32_t* __restrict__ cu,
                                                                  int32_t* __restrict__ idx_out0,
                                                                  int64_t idx_stride_layer,
                                                                  int32_t* __restrict__ counts, SelectCandidates cand) {
  constexpr int RES = PER * kSelThreads;                    // positions held in registers
  static_assert(MODE != kSelSegments || RES == kSelectSegment, "a segment is what one workgroup holds");
  extern __shared__ __attribute__((aligned(16))) char sel_smem[];
  u64* keys = reinterpret_cast<u64*>(sel_smem);                               // [2048] candidates / exchange
  int* hist = reinterpret_cast<int*>(sel_smem + 2048 * sizeof(u64));          // [kRadixBins][kHistCopies]
  __shared__ int scratch[kSelWaves];
  __shared__ int picked[3];
  __shared__ int n_greater_slots;
  __shared__ int wave_eq[kSelWaves];

  const int seq = MODE == kSelSegments ? blockIdx.y / cand.segments_max : blockIdx.y, head = blockIdx.x;
  const int segment = MODE == kSelSegments ? blockIdx.y % cand.segments_max : 0;
  const int layer = layer0 + blockIdx.z;
  const float* __restrict__ scores = scores0 + (int64_t)blockIdx.z * scores_stride_layer;
  int32_t* __restrict__ idx_out = idx_out0 + (int64_t)blockIdx.z * idx_stride_layer;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int begin = cu[seq];
  const int S = cu[seq + 1] - begin;
  const int n_row = S > w ? S - w : 0;                       // candidate positions of the whole row
  const int n_seqs = MODE == kSelSegments ? gridDim.y / cand.segments_max : gridDim.y;
  const int64_t cand_row = (((int64_t)blockIdx.z * n_seqs + seq) * Hkv + head) * cand.stride;
  // what this workgroup selects from: the row, one segment of it, or the row's candidates
  int n, k;
  const uint32_t* __restrict__ row;
  if (MODE == kSelSegments) {
    const int seg_begin = segment * RES;
    n = n_row - seg_begin;
    if (n <= 0) return;                                       // the row has fewer segments
    n = n < RES ? n : RES;
    k = layer_max < n ? layer_max : n;
    row = reinterpret_cast<const uint32_t*>(scores + (int64_t)head * scores_stride_head + begin) + seg_begin;
  } else if (MODE == kSelMerge) {
    n = candidates_of(n_row, layer_max);
    k = layer_max < n_row ? layer_max : n_row;
    row = cand.val + cand_row;
  } else {
    n = n_row;
    k = layer_max < n ? layer_max : n;
    row = reinterpret_cast<const uint32_t*>(scores + (int64_t)head * scores_stride_head + begin);
  }
  int32_t* __restrict__ out = idx_out + ((int64_t)seq * Hkv + head) * layer_max;
  if (MODE != kSelSegments) {
    if (head == 0 && tid == 0) counts[seq * L + layer] = k;
    if (k == 0) {
      for (int j = tid; j < layer_max; j += kSelThreads) out[j] = -1;
      return;
    }
  }
  // 64-bit key of element i with bit pattern u; ascending keys are the order the winners are written in:
  // (score descending, position ascending) for a final list, position ascending for a segment's candidates
  auto make_key = [](uint32_t u, int i) -> u64 {
    return MODE == kSelSegments ? ((u64)(uint32_t)i << 32) | u : ((u64)(~u) << 32) | (uint32_t)i;
  };

  // The first RES positions of the row live in registers for all passes: thread t holds positions
  // j * 1024 + t (coalesced loads, issued back to back). Longer rows re-read their tail from memory.
  uint32_t v[PER];
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int i = j * kSelThreads + tid;
    v[j] = i < n ? row[i] : 0u;
  }
  const int n_res = n < RES ? n : RES;   // positions held in registers

  // ---- radix select: the k-th largest bit pattern
  uint32_t prefix = 0;
  int rem = k;
  auto radix_pass = [&](auto pass_c) {
    constexpr int pass = decltype(pass_c)::value;
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int hshift = pass == 1 ? 21 : 10;                      // bits above this digit (passes 1 and 2)
    auto matches = [&](uint32_t u) { return pass == 0 ? true : ((u >> hshift) == (prefix >> hshift)); };
    // pass 0 sees every element (lanes that share a digit spread over 8 copies of the histogram); the later
    // passes only the elements that share the digits found so far: 2 copies, less to clear and to add up
    const int copies = pass == 0 ? kHistCopies : 2;
    for (int b = tid; b < kRadixBins * copies; b += kSelThreads) hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const uint32_t u = v[j];
      if (j * kSelThreads + tid < n_res && matches(u))
        atomicAdd(&hist[((u >> shift) & (kRadixBins - 1)) * copies + (lane & (copies - 1))], 1);
    }
    // the tail of a long row, eight loads in flight per thread
    for (int i0 = RES + tid; i0 < n; i0 += 8 * kSelThreads) {
      uint32_t u8[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int i = i0 + q * kSelThreads;
        u8[q] = i < n ? row[i] : 0u;
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t u = u8[q];
        if (i0 + q * kSelThreads < n && matches(u))
          atomicAdd(&hist[((u >> shift) & (kRadixBins - 1)) * copies + (lane & (copies - 1))], 1);
      }
    }
    __syncthreads();
    // thread t owns digits 2047 - 2t and 2046 - 2t (scanned from the top)
    const int hi = kRadixBins - 1 - 2 * tid, lo = hi - 1;
    int c_hi = 0, c_lo = 0;
    if (pass == 0) {   // lo and hi are adjacent: 16 consecutive words
      static_assert(kHistCopies == 8, "four 16-byte reads cover the copies of two digits");
      const int4* q = reinterpret_cast<const int4*>(&hist[lo * kHistCopies]);
      const int4 a = q[0], b = q[1], c = q[2], d = q[3];
      c_lo = a.x + a.y + a.z + a.w + b.x + b.y + b.z + b.w;
      c_hi = c.x + c.y + c.z + c.w + d.x + d.y + d.z + d.w;
    } else {   // lo and hi are adjacent: 4 consecutive words
      const int4 q = *reinterpret_cast<const int4*>(&hist[lo * 2]);
      c_lo = q.x + q.y;
      c_hi = q.z + q.w;
    }
    const int above = block_exclusive_scan(c_hi + c_lo, scratch);
    if (above < rem && rem <= above + c_hi) { picked[0] = hi; picked[1] = above; picked[2] = c_hi; }
    else if (above + c_hi < rem && rem <= above + c_hi + c_lo) { picked[0] = lo; picked[1] = above + c_hi; picked[2] = c_lo; }
    __syncthreads();
    prefix |= (uint32_t)picked[0] << shift;     // picked is next written two barriers further on
    rem -= picked[1];
  };
  radix_pass(std::integral_constant<int, 0>{});
  radix_pass(std::integral_constant<int, 1>{});
  // Short path. After the upper two digits (22 bits) the winners are known up to the elements that share them:
  // `sure` elements have larger upper digits, picked[2] share them (a handful, unless many scores are equal). When
  // all of those together fit, they go to LDS as keys in any order and the ordering step below sorts them ALL: the
  // first k of the ascending keys are the answer, ties already broken by the position in the key - no third
  // digit, no position-ordered pick of the elements equal to the threshold. Not for a segment's candidates (they
  // are left in position order) nor for rows with a tail outside the registers.
  // (One histogram over the upper 16 bits in place of the two digits was measured and is slower: 16384 single bins
  // collide on the LDS banks more than 8 copies of a few hot 11-bit digits collide on their addresses.)
  const int sure = k - rem;
  const int m_short = sure + picked[2];
  const bool short_path = MODE != kSelSegments && n <= RES && m_short <= kShortCap;
  int m_keys = k;                                     // keys the ordering step sorts
  const u64* order_src = keys;
  if (short_path) {
    u64* __restrict__ cand_keys = reinterpret_cast<u64*>(hist);      // [kShortCap]: the histogram is spent
    const uint32_t bound = prefix;                                   // every pattern whose upper two digits are not below the threshold's
    int mine_n = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine_n += (j * kSelThreads + tid < n_res && v[j] >= bound) ? 1 : 0;
    int slot = block_exclusive_scan(mine_n, scratch);               // its first barrier: all reads of the histogram are done
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int i = j * kSelThreads + tid;
      if (i < n_res && v[j] >= bound) cand_keys[slot++] = make_key(v[j], i);
    }
    m_keys = m_short;
    order_src = cand_keys;
  } else {
  radix_pass(std::integral_constant<int, 2>{});
  const uint32_t T = prefix;      // k-th largest value
  const int need_eq = rem;        // how many elements equal to T are taken (>= 1)
  const int n_gt = k - need_eq;   // elements strictly greater than T

  // ---- compaction: everything above T (any order: the sort fixes it), and the first need_eq elements equal
  // to T in position order. Position order of the resident part is (j, wavefront, lane).
  int* eq_base = hist;            // [PER][kSelWaves] counts, then exclusive prefix sums (reuses hist)
  if (tid == 0) n_greater_slots = 0;
  for (int j = k + tid; j < 2048; j += kSelThreads) keys[j] = ~0ull;      // pads sort to the end
  __syncthreads();
  // elements above T: every thread counts its own, one scan over the threads gives it a contiguous range of
  // slots (any order will do); elements equal to T: counted per (j, wavefront) for the position-ordered pick below
  int my_gt = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int i = j * kSelThreads + tid;
    const uint32_t u = v[j];
    my_gt += i < n_res && u > T ? 1 : 0;
    const unsigned long long emask = __ballot(i < n_res && u == T);
    if (lane == 0) eq_base[j * kSelWaves + wv] = __popcll(emask);
  }
  int slot = block_exclusive_scan(my_gt, scratch);
  if (tid == kSelThreads - 1) n_greater_slots = slot + my_gt;     // the tail of a long row continues from here
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int i = j * kSelThreads + tid;
    const uint32_t u = v[j];
    if (i < n_res && u > T) keys[slot++] = make_key(u, i);
  }
  __syncthreads();
  {
    static_assert(PER * kSelWaves <= kSelThreads, "one count per thread");
    const int c = tid < PER * kSelWaves ? eq_base[tid] : 0;
    const int ex = block_exclusive_scan(c, scratch);
    if (tid < PER * kSelWaves) eq_base[tid] = ex;
    if (tid == PER * kSelWaves - 1) picked[0] = ex + c;   // equal elements in the resident part
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int i = j * kSelThreads + tid;
    const bool eq = i < n_res && v[j] == T;
    const unsigned long long emask = __ballot(eq);
    if (eq) {
      const int rank = eq_base[j * kSelWaves + wv] + __popcll(emask & ((1ull << lane) - 1ull));
      if (rank < need_eq) keys[n_gt + rank] = make_key(T, i);
    }
  }
  if (n > RES) {
    // tail of a long row: contiguous segments per wavefront, walked in 64-wide coalesced steps
    const int eq_resident = picked[0];
    const int tail = n - RES;
    int seg = (tail + kSelWaves - 1) / kSelWaves;
    seg = (seg + 63) / 64 * 64;
    const int seg_begin = RES + wv * seg;
    const int seg_end = seg_begin + seg < n ? seg_begin + seg : n;
    int eq_count = 0;
    for (int i00 = seg_begin; i00 < seg_end; i00 += 4 * 64) {   // four loads in flight per lane
      uint32_t u4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i00 + q * 64 + lane;
        u4[q] = i < seg_end ? row[i] : 0u;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i00 + q * 64 + lane;
        const uint32_t u = u4[q];
        const bool gt = i < seg_end && u > T;
        const bool eq = i < seg_end && u == T;
        const unsigned long long gmask = __ballot(gt);
        eq_count += __popcll(__ballot(eq));
        if (gmask) {
          int base = 0;
          if (lane == 0) base = atomicAdd(&n_greater_slots, __popcll(gmask));
          base = __shfl(base, 0);
          if (gt) keys[base + __popcll(gmask & ((1ull << lane) - 1ull))] = make_key(u, i);
        }
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
        if (rank < need_eq) keys[n_gt + rank] = make_key(T, i);
      }
      running += __popcll(emask);
    }
  }
  }   // long path
  __syncthreads();

  // ---- order the keys (the k winners, or the short path's candidates) by (score descending, position ascending) =
  // ascending 64-bit key, here in LDS: buckets by the leading bits of the keys' score halves (2048 linear bins
  // between the smallest and the largest one), a scan over the buckets, and a rank inside the bucket by counting.
  // The keys are the upper tail of the row, a few per bucket; keys that all share one bucket (all scores equal)
  // cost their number squared in comparisons. Only ranks below k are written.
  int* bcount = reinterpret_cast<int*>(sel_smem);               // [kRadixBins] keys per bucket
  int* bstart = bcount + kRadixBins;                            // [kRadixBins] first place of the bucket
  u64* sorted = reinterpret_cast<u64*>(hist + 2 * kShortCap);   // [kShortCap] keys in bucket order (behind the candidates)
  static_assert(2 * kRadixBins * sizeof(int) <= 2048 * sizeof(u64), "the bucket arrays take the place of the winners' keys");
  static_assert(2 * kShortCap * sizeof(u64) <= (size_t)kRadixBins * kHistCopies * sizeof(int), "candidates and their sorted copy fit the histogram");
  u64 mine[kOrderPerThread];
  uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
  for (int c = 0; c < kOrderPerThread; ++c) {
    const int j = tid + c * kSelThreads;
    mine[c] = j < m_keys ? order_src[j] : ~0ull;
    if (j < m_keys) {
      const uint32_t h = (uint32_t)(mine[c] >> 32);
      lo = h < lo ? h : lo;
      hi = h > hi ? h : hi;
    }
  }
  wave_min_max(lo, hi);
  __shared__ uint32_t wave_lo[kSelWaves], wave_hi[kSelWaves];
  if (lane == 0) { wave_lo[wv] = lo; wave_hi[wv] = hi; }
  __syncthreads();                                             // every key is in registers: its place in LDS is free
  for (int bI = tid; bI < kRadixBins; bI += kSelThreads) bcount[bI] = 0;
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i) {
    lo = wave_lo[i] < lo ? wave_lo[i] : lo;
    hi = wave_hi[i] > hi ? wave_hi[i] : hi;
  }
  __syncthreads();
  const uint32_t range = hi - lo;                              // m_keys >= 1 here: lo <= hi
  const int shift = range < (uint32_t)kRadixBins ? 0 : (32 - __builtin_clz(range)) - 11;   // (range >> shift) < 2048
  int bin[kOrderPerThread], place[kOrderPerThread];
#pragma unroll
  for (int c = 0; c < kOrderPerThread; ++c) {
    const int j = tid + c * kSelThreads;
    bin[c] = j < m_keys ? (int)((((uint32_t)(mine[c] >> 32)) - lo) >> shift) : 0;
    place[c] = j < m_keys ? atomicAdd(&bcount[bin[c]], 1) : 0;  // order of arrival inside the bucket: any order will do
  }
  __syncthreads();
  {
    const int c0 = bcount[2 * tid], c1 = bcount[2 * tid + 1];  // thread t owns buckets 2t and 2t + 1
    const int ex = block_exclusive_scan(c0 + c1, scratch);
    bstart[2 * tid] = ex;
    bstart[2 * tid + 1] = ex + c0;
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < kOrderPerThread; ++c) {
    const int j = tid + c * kSelThreads;
    if (j < m_keys) sorted[bstart[bin[c]] + place[c]] = mine[c];
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < kOrderPerThread; ++c) {
    const int j = tid + c * kSelThreads;
    if (j < m_keys) {
      const int first = bstart[bin[c]], n_in = bcount[bin[c]];
      int rank = first;
      for (int i = 0; i < n_in; ++i) rank += sorted[first + i] < mine[c] ? 1 : 0;
      if (rank >= k) continue;                 // a candidate of the short path that is not among the k winners
      if (MODE == kSelSegments) {            // the segment's candidates, in position order
        const int64_t e = cand_row + (int64_t)segment * layer_max + rank;
        cand.val[e] = (uint32_t)mine[c];
        cand.pos[e] = segment * RES + (int32_t)(mine[c] >> 32);
      } else if (MODE == kSelMerge) {        // the key's low half is a place in the candidate list
        out[rank] = cand.pos[cand_row + (uint32_t)mine[c]];
      } else {
        out[rank] = (int32_t)(uint32_t)mine[c];
      }
    }
  }
  if (MODE != kSelSegments)
    for (int j = k + tid; j < layer_max; j += kSelThreads) out[j] = -1;
}

hipError_t launch_select(const Params& p, int layer, int n_layers, const float* scores, int64_t scores_stride_head,
                         int64_t scores_stride_layer, const int32_t* cu, int32_t* idx_out, int64_t idx_stride_layer,
                         int32_t* counts, char* ws, const WorkspaceLayout& wl, hipStream_t st) {
  const size_t lds = 2048 * sizeof(u64) + (size_t)kRadixBins * kHistCopies * sizeof(int);
  static bool attr_set = false;
  if (!attr_set) {
    for (const void* f : {reinterpret_cast<const void*>(&select_topk_kernel<kSelDirect, 32>),
                          reinterpret_cast<const void*>(&select_topk_kernel<kSelDirect, 16>),
                          reinterpret_cast<const void*>(&select_topk_kernel<kSelDirect, 8>),
                          reinterpret_cast<const void*>(&select_topk_kernel<kSelSegments, 32>),
                          reinterpret_cast<const void*>(&select_topk_kernel<kSelMerge, 32>),
                          reinterpret_cast<const void*>(&select_topk_kernel<kSelMerge, 16>),
                          reinterpret_cast<const void*>(&select_topk_kernel<kSelMerge, 8>)}) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    attr_set = true;
  }
  SelectCandidates cand{};
  if (wl.select_segments <= 1) {      // every row fits the registers of one workgroup
    // the fewest registers per thread that hold the longest row the descriptor admits
    const int longest = p.max_seq_len - p.w;
    if (longest <= 8 * kSelThreads)
      launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelDirect, 8>), dim3(p.Hkv, p.n_seqs, n_layers), dim3(kSelThreads), lds,
             st, p.Hkv, p.w, p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out,
             idx_stride_layer, counts, cand);
    else if (longest <= 16 * kSelThreads)
      launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelDirect, 16>), dim3(p.Hkv, p.n_seqs, n_layers), dim3(kSelThreads), lds,
             st, p.Hkv, p.w, p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out,
             idx_stride_layer, counts, cand);
    else
      launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelDirect, 32>), dim3(p.Hkv, p.n_seqs, n_layers), dim3(kSelThreads), lds,
             st, p.Hkv, p.w, p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out,
             idx_stride_layer, counts, cand);
    return hipGetLastError();
  }
  cand.val = reinterpret_cast<uint32_t*>(ws + wl.select_cand_val);
  cand.pos = reinterpret_cast<int32_t*>(ws + wl.select_cand_pos);
  cand.segments_max = wl.select_segments;
  cand.stride = (int64_t)wl.select_segments * p.layer_max;
  launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelSegments, 32>), dim3(p.Hkv, p.n_seqs * wl.select_segments, n_layers),
         dim3(kSelThreads), lds, st, p.Hkv, p.w, p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer,
         cu, idx_out, idx_stride_layer, counts, cand);
  // level 2: the fewest registers per thread that hold a row's candidates (a longer list keeps its tail in memory)
  const int64_t most = (int64_t)wl.select_segments * p.layer_max;
  const dim3 grid_merge(p.Hkv, p.n_seqs, n_layers);
  if (most <= 8 * kSelThreads)
    launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelMerge, 8>), grid_merge, dim3(kSelThreads), lds, st, p.Hkv, p.w,
           p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out, idx_stride_layer, counts, cand);
  else if (most <= 16 * kSelThreads)
    launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelMerge, 16>), grid_merge, dim3(kSelThreads), lds, st, p.Hkv, p.w,
           p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out, idx_stride_layer, counts, cand);
  else
    launch(DKV_KERNEL_SELECT, (select_topk_kernel<kSelMerge, 32>), grid_merge, dim3(kSelThreads), lds, st, p.Hkv, p.w,
           p.layer_max, p.L, layer, scores, scores_stride_head, scores_stride_layer, cu, idx_out, idx_stride_layer, counts, cand);
  return hipGetLastError();
}

}  // namespace dkv
