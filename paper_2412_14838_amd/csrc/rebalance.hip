// Progressive cache update (Section 4.2, Eq. 4-6; Algorithm 1: Update_Buffer_Length and the truncation loop).
//
// The global top-kg over the concatenated scores of the layers processed so far only matters through its
// per-layer hit counts, so no element is ever moved: a 3-digit radix select (11 + 11 + 10 bits of the fp32
// pattern, scores are >= 0) finds the kg-th largest value T from per-(sequence, layer) digit histograms.
// Many workgroups build the histograms (the scan of all scores is bandwidth work) and, from the second pass on,
// also count per layer the elements that the digits found so far already place above T; a single workgroup per
// sequence takes every decision: the digit of T after each pass, then cnt_i = #{> T in layer i} + the share
// of the elements equal to T that the tie rule (lower layer first) gives to layer i, then Z, Z' and counts.
#include "dkv_internal.h"

namespace dkv {

constexpr int kDecThreads = 1024;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kScanCopies = 4;   // interleaved copies of the LDS histogram: lanes sharing a digit spread over 4 words

// state[seq][8]: 0 prefix bits of T found so far, 1 remaining rank, 2..4 chosen digit of pass 0..2, 5 kg
__device__ inline int digit_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }

// grid = (chunk upper bound, Hkv, layers_done); block 256. Adds the digit histogram of one chunk of one
// (sequence, head, layer) row into hist[pass][seq][layer][*]. Elements whose higher bits differ from the
// prefix found by the earlier passes are skipped.
template <int PASS>
__global__ __launch_bounds__(256) void rebalance_hist_kernel(int n_seqs, int Hkv, int w, int L, int total_tokens,
                                                             const float* __restrict__ scores_all,
                                                             const int32_t* __restrict__ cu, int32_t* __restrict__ hist,
                                                             const int32_t* __restrict__ state,
                                                             int32_t* __restrict__ above) {
  __shared__ int h[kRadixBins * kScanCopies];
  __shared__ int n_above;
  int seq, c, begin, len;
  if (!find_chunk(cu, n_seqs, kRebalanceChunk, w, blockIdx.x, seq, c, begin, len)) return;
  const int head = blockIdx.y, layer = blockIdx.z;
  const int n = len - w;
  const int i0 = c * kRebalanceChunk;
  const int i1 = i0 + kRebalanceChunk < n ? i0 + kRebalanceChunk : n;
  uint32_t prefix = 0;
  if (PASS > 0) {
    if (state[seq * 8 + 5] == 0) return;   // kg == 0: nothing to select
    prefix = (uint32_t)state[seq * 8 + 0];
  }
  for (int b = threadIdx.x; b < kRadixBins * kScanCopies; b += 256) h[b] = 0;
  if (threadIdx.x == 0) n_above = 0;
  __syncthreads();
  const uint32_t* __restrict__ row =
      reinterpret_cast<const uint32_t*>(scores_all + ((int64_t)layer * Hkv + head) * total_tokens + begin);
  constexpr int shift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
  constexpr int ushift = PASS == 0 ? 0 : (PASS == 1 ? 21 : 10);
  constexpr uint32_t dmask = PASS == 2 ? 1023u : (uint32_t)(kRadixBins - 1);   // the last digit has 10 bits only
  int mine = 0;   // elements of this thread that the digits found so far place above T
  for (int i = i0 + threadIdx.x; i < i1; i += 256) {
    const uint32_t u = row[i];
    const bool match = PASS == 0 ? true : ((u >> ushift) == (prefix >> ushift));
    if (match) atomicAdd(&h[((u >> shift) & dmask) * kScanCopies + (threadIdx.x & (kScanCopies - 1))], 1);
    if (PASS > 0) {
      // the digit chosen by the previous pass sits just above this pass's digit: equal higher bits, larger digit
      constexpr int pshift = PASS == 1 ? 21 : 10;
      const bool higher_equal = PASS == 1 ? true : ((u >> 21) == (prefix >> 21));
      if (higher_equal && (u >> pshift) > (prefix >> pshift)) ++mine;
    }
  }
  if (PASS > 0) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&n_above, mine);
  }
  __syncthreads();
  if (PASS > 0 && threadIdx.x == 0 && n_above) atomicAdd(&above[seq * L + layer], n_above);
  int32_t* __restrict__ g = hist + (((int64_t)PASS * n_seqs + seq) * L + layer) * kRadixBins;
  for (int b = threadIdx.x; b < kRadixBins; b += 256) {
    int v = 0;
#pragma unroll
    for (int c2 = 0; c2 < kScanCopies; ++c2) v += h[b * kScanCopies + c2];
    if (v) atomicAdd(&g[b], v);
  }
}

__device__ inline int wave_inclusive_scan_i(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
}

// Single workgroup per sequence: sums the per-layer histograms of `pass`, finds the digit that holds the
// remaining rank and records it in state[] (for later kernels) and in sh[] (for this workgroup):
// sh[0] digit, sh[1] remaining rank after this pass, sh[2] kg. Shared by the decide and the final kernel.
__device__ inline void decide_digit(int pass, int seq, int n_seqs, int L, int layers_done, int w, int Hkv,
                                    int mean_budget, const int32_t* __restrict__ cu,
                                    const int32_t* __restrict__ hist, int32_t* __restrict__ state, int* scratch,
                                    int* sh) {
  static_assert(kRadixBins == 2 * kDecThreads, "two bins per thread");
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int rem, kg;
  uint32_t prefix = 0;
  if (pass == 0) {
    const int len = cu[seq + 1] - cu[seq];
    const long long n = len > w ? len - w : 0;
    const long long want = (long long)mean_budget * Hkv * layers_done;
    const long long have = n * Hkv * layers_done;
    kg = (int)(want < have ? want : have);
    rem = kg;
  } else {   // written by the previous kernel of this call
    prefix = (uint32_t)state[seq * 8 + 0];
    rem = state[seq * 8 + 1];
    kg = state[seq * 8 + 5];
  }
  const int hi = kRadixBins - 1 - 2 * tid, lo = hi - 1;
  int c_hi = 0, c_lo = 0;
  const int32_t* __restrict__ g = hist + ((int64_t)pass * n_seqs + seq) * L * kRadixBins;
#pragma unroll 8
  for (int i = 0; i < layers_done; ++i) {   // bins lo, hi are adjacent: one 8-byte load per layer
    const int2 v = *reinterpret_cast<const int2*>(g + (int64_t)i * kRadixBins + lo);
    c_lo += v.x;
    c_hi += v.y;
  }
  const int v = c_hi + c_lo;
  const int incl = wave_inclusive_scan_i(v);
  if (lane == 63) scratch[wv] = incl;
  if (tid == 0) { sh[0] = 0; sh[1] = 0; sh[2] = kg; }
  __syncthreads();
  int above = incl - v;
  for (int i = 0; i < wv; ++i) above += scratch[i];
  if (rem > 0) {   // exactly one thread owns the bin that holds the rem-th largest element
    if (above < rem && rem <= above + c_hi) { sh[0] = hi; sh[1] = rem - above; }
    else if (above + c_hi < rem && rem <= above + v) { sh[0] = lo; sh[1] = rem - above - c_hi; }
  }
  __syncthreads();
  if (tid == 0) {
    state[seq * 8 + 0] = (int32_t)(prefix | ((uint32_t)sh[0] << digit_shift(pass)));
    state[seq * 8 + 1] = sh[1];
    state[seq * 8 + 2 + pass] = sh[0];
    state[seq * 8 + 5] = kg;
  }
}

__global__ __launch_bounds__(kDecThreads) void rebalance_decide_kernel(int pass, int n_seqs, int L, int layers_done,
                                                                       int w, int Hkv, int mean_budget,
                                                                       const int32_t* __restrict__ cu,
                                                                       const int32_t* __restrict__ hist,
                                                                       int32_t* __restrict__ state) {
  __shared__ int scratch[kDecWaves];
  __shared__ int sh[3];
  decide_digit(pass, blockIdx.x, n_seqs, L, layers_done, w, Hkv, mean_budget, cu, hist, state, scratch, sh);
}

// Last pass decision, per-layer hit counts and the budget arithmetic of Eq. 5-6, one workgroup per sequence.
__global__ __launch_bounds__(kDecThreads) void rebalance_final_kernel(int n_seqs, int L, int layers_done, int w, int Hkv,
                                                                      int mean_budget, int layer_max,
                                                                      const int32_t* __restrict__ cu,
                                                                      const int32_t* __restrict__ hist,
                                                                      int32_t* __restrict__ state,
                                                                      const int32_t* __restrict__ above,
                                                                      int32_t* __restrict__ counts,
                                                                      int32_t* __restrict__ budgets_out,
                                                                      int32_t* __restrict__ hits_out) {
  __shared__ int scratch[kDecWaves];
  __shared__ int sh[3];
  __shared__ int gt[DKV_MAX_LAYERS];
  __shared__ int eq[DKV_MAX_LAYERS];
  const int seq = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  // digits of passes 0 and 1 were recorded by earlier kernels of this call
  const int digit0 = state[seq * 8 + 2], digit1 = state[seq * 8 + 3];
  decide_digit(2, seq, n_seqs, L, layers_done, w, Hkv, mean_budget, cu, hist, state, scratch, sh);
  const int digit[3] = {digit0, digit1, sh[0]};
  (void)digit0; (void)digit1;
  const int need_eq = sh[1];   // elements equal to T that belong to the top-kg
  const int kg = sh[2];
  // per layer: elements above T = those counted by the scan kernels of passes 1 and 2 (higher digits larger)
  // + the last-digit bins above the chosen one; equal to T = the chosen last-digit bin
  for (int i = wv; i < layers_done; i += kDecWaves) {
    int acc = 0;
    const int32_t* __restrict__ g = hist + (((int64_t)2 * n_seqs + seq) * L + i) * kRadixBins;
    for (int b = digit[2] + 1 + lane; b < 1024; b += 64) acc += g[b];     // the last digit has 10 bits
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) {
      gt[i] = acc + above[seq * L + i];
      eq[i] = g[digit[2]];
    }
  }
  __shared__ int cur[DKV_MAX_LAYERS];
  for (int i = tid; i < layers_done; i += kDecThreads) cur[i] = counts[seq * L + i];
  __syncthreads();
  __shared__ long long red[2];   // max cnt, sum Z
  if (tid == 0) {   // Phi: ties go to the lower flat index, i.e. earlier layers first (a serial prefix over L ints)
    long long cmax = 0;
    int left = need_eq;
    for (int i = 0; i < layers_done; ++i) {
      int take = 0;
      if (kg > 0) { take = eq[i] < left ? eq[i] : left; left -= take; }
      const int c = kg > 0 ? gt[i] + take : 0;
      gt[i] = c;
      cmax = c > cmax ? c : cmax;
    }
    red[0] = cmax;
  }
  __syncthreads();
  const long long cmax = red[0];
  for (int i = tid; i < layers_done; i += kDecThreads)
    eq[i] = cmax > 0 ? (int)(((long long)layer_max * gt[i]) / cmax) : 0;          // Eq. 5, exact floor
  __syncthreads();
  if (tid == 0) {
    long long zsum = 0;
    for (int i = 0; i < layers_done; ++i) zsum += eq[i];
    red[1] = zsum;
  }
  __syncthreads();
  const long long zsum = red[1];
  const long long B = (long long)mean_budget * L;                                 // Eq. 6: B = (wt - ws) * L
  for (int i = tid; i < layers_done; i += kDecThreads) {
    const long long zp = zsum > 0 ? ((long long)eq[i] * B) / zsum : 0;            // exact floor
    const int zpi = zp > 0x7fffffffLL ? 0x7fffffff : (int)zp;
    if (budgets_out) budgets_out[seq * L + i] = zpi;
    if (hits_out) hits_out[seq * L + i] = gt[i];
    counts[seq * L + i] = cur[i] < zpi ? cur[i] : zpi;                            // truncation never grows a layer
  }
}

hipError_t launch_rebalance(const Params& p, int layers_done, const float* scores_all, const int32_t* cu,
                            int32_t* counts, int32_t* budgets_out, int32_t* hits_out, char* ws,
                            const WorkspaceLayout& wl, hipStream_t st) {
  int32_t* hist = reinterpret_cast<int32_t*>(ws + wl.hist);
  int32_t* state = reinterpret_cast<int32_t*>(ws + wl.state);
  int32_t* above = reinterpret_cast<int32_t*>(ws + wl.above);
  hipError_t e = launch_fill_zero(ws + wl.hist, wl.total - wl.hist, st);
  if (e != hipSuccess) return e;
  const int chunks = p.total_tokens / kRebalanceChunk + p.n_seqs;
  const dim3 grid(chunks, p.Hkv, layers_done);
  launch(DKV_KERNEL_REBALANCE_HIST, rebalance_hist_kernel<0>, grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L, p.total_tokens,
                     scores_all, cu, hist, state, above);
  launch(DKV_KERNEL_REBALANCE_DECIDE, rebalance_decide_kernel, dim3(p.n_seqs), dim3(kDecThreads), 0, st, 0, p.n_seqs, p.L, layers_done,
                     p.w, p.Hkv, p.mean_budget, cu, hist, state);
  launch(DKV_KERNEL_REBALANCE_HIST, rebalance_hist_kernel<1>, grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L, p.total_tokens,
                     scores_all, cu, hist, state, above);
  launch(DKV_KERNEL_REBALANCE_DECIDE, rebalance_decide_kernel, dim3(p.n_seqs), dim3(kDecThreads), 0, st, 1, p.n_seqs, p.L, layers_done,
                     p.w, p.Hkv, p.mean_budget, cu, hist, state);
  launch(DKV_KERNEL_REBALANCE_HIST, rebalance_hist_kernel<2>, grid, dim3(256), 0, st, p.n_seqs, p.Hkv, p.w, p.L, p.total_tokens,
                     scores_all, cu, hist, state, above);
  launch(DKV_KERNEL_REBALANCE_FINAL, rebalance_final_kernel, dim3(p.n_seqs), dim3(kDecThreads), 0, st, p.n_seqs, p.L, layers_done, p.w,
                     p.Hkv, p.mean_budget, p.layer_max, cu, hist, state, above, counts, budgets_out, hits_out);
  return hipGetLastError();
}

}  // namespace dkv
