// Fixed-pattern retention schedules: the comparison methods of the paper's Section 5.1 ("Baselines") and Figure 1
// (b), (c), as alternative producers of the per-layer counts that dkv_gather_kv, dkv_pack_cache and
// dkv_decode_attention consume. The paper names the patterns without formulas; the readings are stated in
// include/dkv.h next to each call.
#include "dkv_internal.h"

namespace dkv {

// counts[q][i] <- min(counts[q][i], budgets[i]) for i < n_layers: the truncation loop of Algorithm 1 with preset
// budgets. grid = ceil(n_seqs * n_layers / 256).
__global__ __launch_bounds__(256) void apply_budgets_kernel(int n_seqs, int L, int n_layers,
                                                            const int32_t* __restrict__ budgets,
                                                            int32_t* __restrict__ counts) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n_seqs * n_layers) return;
  const int q = i / n_layers, l = i % n_layers;
  const int b = budgets[l] > 0 ? budgets[l] : 0;
  const int c = counts[q * L + l];
  counts[q * L + l] = c < b ? c : b;
}

// Recency pattern: per (sequence, KV head) the first `sinks` prefix positions, then the newest prefix positions from
// the last one down, k = min(layer_max, S') entries in all; entries past k are -1. grid = (ceil(layer_max / 256), Hkv,
// n_seqs folded into x), 256 threads.
__global__ __launch_bounds__(256) void select_recent_kernel(int n_seqs, int Hkv, int L, int layer, int w, int layer_max,
                                                            int n_sink, int blocks_per_row,
                                                            const int32_t* __restrict__ cu, int32_t* __restrict__ idx_out,
                                                            int32_t* __restrict__ counts) {
  const int seq = blockIdx.x / blocks_per_row, head = blockIdx.y;
  const int j = (blockIdx.x % blocks_per_row) * 256 + threadIdx.x;
  const int S = cu[seq + 1] - cu[seq];
  const int prefix = S > w ? S - w : 0;
  const int k = layer_max < prefix ? layer_max : prefix;
  const int sinks = n_sink < k ? n_sink : k;
  if (j < layer_max)
    idx_out[((int64_t)seq * Hkv + head) * layer_max + j] = j >= k ? -1 : (j < sinks ? j : prefix - 1 - (j - sinks));
  if (j == 0 && head == 0) counts[seq * L + layer] = k;
}

hipError_t launch_apply_budgets(const Params& p, int n_layers, const int32_t* budgets, int32_t* counts, hipStream_t st) {
  const int n = p.n_seqs * n_layers;
  launch(DKV_KERNEL_SCHEDULE, apply_budgets_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p.n_seqs, p.L, n_layers,
         budgets, counts);
  return hipGetLastError();
}

hipError_t launch_select_recent(const Params& p, int layer, int n_sink, const int32_t* cu, int32_t* idx_out,
                                int32_t* counts, hipStream_t st) {
  const int blocks_per_row = (p.layer_max + 255) / 256;
  launch(DKV_KERNEL_SCHEDULE, select_recent_kernel, dim3(blocks_per_row * p.n_seqs, p.Hkv), dim3(256), 0, st, p.n_seqs,
         p.Hkv, p.L, layer, p.w, p.layer_max, n_sink, blocks_per_row, cu, idx_out, counts);
  return hipGetLastError();
}

}  // namespace dkv
