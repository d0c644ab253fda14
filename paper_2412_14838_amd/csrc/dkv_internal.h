// Internal declarations shared by the translation units of libdkv.so (host side + device helpers).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>
#include "../../include/dkv.h"

namespace dkv {

// ----------------------------------------------------------------------------------------------
// Tiling constants
// ----------------------------------------------------------------------------------------------
constexpr int kGenericKeys = 256;      // keys per workgroup in the generic (VALU) score kernels
constexpr int kMfmaMinChunk = 256;     // smallest chunk of keys per workgroup in the MFMA score kernels
constexpr int kRadixBins = 2048;       // 11-bit digits; 3 passes cover bits 31..21, 20..10, 9..0
constexpr int kSelectSegment = 32768;  // row positions one selection workgroup keeps in registers

// ----------------------------------------------------------------------------------------------
// Workspace layout (byte offsets, all 256-byte aligned)
// ----------------------------------------------------------------------------------------------
constexpr int kDecodeMaxGroup = 16;    // query heads per KV head the decode kernel handles
constexpr int kDecodeMaxSlabs = (DKV_MAX_LAYER_MAX + DKV_MAX_ROWS + 31) / 32;   // slabs of one cache block at most
// cache rows per workgroup of the decode kernel, by element size
constexpr int decode_slab_rows(size_t elt_bytes) { return elt_bytes == 2 ? 128 : 64; }

struct WorkspaceLayout {
  size_t partials;     // float2 [DKV_MAX_SELECT_LAYERS][chunks_max][Hkv][rows_pad] per-chunk row statistics (max, sum of exponentials)
  size_t partials_layer_bytes;   // one layer's share of it
  size_t lse_rows;     // float [DKV_MAX_SELECT_LAYERS][n_seqs][Hkv][rows_pad] merged row normalisers (log2) of a multi-layer scoring call
  size_t edges;        // float [DKV_MAX_SELECT_LAYERS][chunks_max][Hkv][64] column sums next to the chunk borders of a multi-layer emit launch
  size_t edges_layer_bytes;      // one layer's share of it
  // progressive update: digit histograms summed over layers (tot0 persists from call to call, see header)
  size_t header;       // int32 [16]                     which layers tot0 covers, for which score tensor and prefill epoch
  size_t tot0;         // int32 [DKV_MAX_UPDATES][n_seqs][kRadixBins]  top digit: slot 0 kept from call to call, slot u the layers new to update u
  // per class of updates of a call (updates whose thresholds share the digits found so far see the same elements;
  // a class is named by its first update), DKV_MAX_UPDATES blocks of:
  size_t tot1;         // int32 [n_seqs][DKV_MAX_UPDATES][kRadixBins]  middle digit of the elements sharing the threshold's top digit, summed over the layers new to update f (slot f)
  size_t tot2;         // int32 [n_seqs][DKV_MAX_UPDATES][1024]        last digit of the elements sharing the two digits above, same slots
  size_t hist2;        // int32 [n_seqs][L][1024]        the same per layer
  size_t above;        // int32 [2][n_seqs][L]           per-layer counts of elements known to be above the threshold (by the top digit; by the middle digit)
  size_t tot0_slot_bytes;      // one of the DKV_MAX_UPDATES slots of the top-digit histogram
  size_t update_block_bytes;   // tot1 .. above of one class; DKV_MAX_UPDATES such blocks follow each other
  size_t picks;        // int32 [DKV_MAX_UPDATES][n_seqs][4]  per update: digit 0 of its threshold, rank left inside it, digit 1, rank left inside that
  size_t decode_partials;  // float [DKV_MAX_SELECT_LAYERS][n_seqs][Hq][slabs][d + 2]    per-slab (max, sum, unnormalised output) of the decode attention
  size_t decode_partials_layer_bytes;   // one layer's share of it
  // two-level selection of rows longer than one workgroup keeps in registers (absent when no row can be that long)
  size_t select_cand_val;  // uint32 [DKV_MAX_SELECT_LAYERS][n_seqs][Hkv][select_segments][layer_max]  candidates' score bits
  size_t select_cand_pos;  // int32, same shape: their positions
  int select_segments;     // segments of the longest row the descriptor admits (1: single-level selection)
  size_t total;
  int rows_pad;        // padded_rows(G*w)
  int chunks_max;      // upper bound on statistics chunks over all sequences
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Rows of the per-(chunk, head) statistics blocks: G*w rounded up to what the widest kernel writes (the MFMA
// kernels work on 64, 128 or 256 rows), so that a block never reaches into its neighbour's.
inline int padded_rows(int rows) { return rows <= 64 ? 64 : rows <= 128 ? 128 : (rows + 255) / 256 * 256; }

inline int min_stats_keys() { return kGenericKeys < kMfmaMinChunk ? kGenericKeys : kMfmaMinChunk; }

inline WorkspaceLayout workspace_layout(const dkv_desc& d) {
  WorkspaceLayout w{};
  const int rows = (d.n_q_heads / d.n_kv_heads) * d.window;
  w.rows_pad = padded_rows(rows);
  w.chunks_max = d.total_tokens / min_stats_keys() + d.n_seqs;
  size_t off = 0;
  w.partials = off;
  w.partials_layer_bytes = align256(size_t(w.chunks_max) * d.n_kv_heads * w.rows_pad * 2 * sizeof(float));
  off += w.partials_layer_bytes * DKV_MAX_SELECT_LAYERS;
  w.lse_rows = off; off += align256(size_t(DKV_MAX_SELECT_LAYERS) * d.n_seqs * d.n_kv_heads * w.rows_pad * sizeof(float));
  w.edges = off;
  w.edges_layer_bytes = align256(size_t(w.chunks_max) * d.n_kv_heads * 64 * sizeof(float));
  off += w.edges_layer_bytes * DKV_MAX_SELECT_LAYERS;
  w.decode_partials = off;
  w.decode_partials_layer_bytes =
      align256(size_t(d.n_seqs) * d.n_q_heads * ((d.window + d.layer_max + 31) / 32) * (d.head_dim + 2) * sizeof(float));
  off += w.decode_partials_layer_bytes * DKV_MAX_SELECT_LAYERS;
  {
    const int longest = d.max_seq_len > d.window ? d.max_seq_len - d.window : 0;
    w.select_segments = longest > kSelectSegment ? (longest + kSelectSegment - 1) / kSelectSegment : 1;
    const size_t entries = w.select_segments > 1
        ? size_t(DKV_MAX_SELECT_LAYERS) * d.n_seqs * d.n_kv_heads * w.select_segments * d.layer_max : 0;
    w.select_cand_val = off; off += align256(entries * sizeof(uint32_t));
    w.select_cand_pos = off; off += align256(entries * sizeof(int32_t));
  }
  w.header = off;   off += align256(16 * sizeof(int32_t));
  w.tot0_slot_bytes = align256(size_t(d.n_seqs) * kRadixBins * sizeof(int32_t));
  w.tot0 = off;     off += w.tot0_slot_bytes * DKV_MAX_UPDATES;
  const size_t block = off;                                                             // tot1 .. above: one class's block
  w.tot1 = off;     off += align256(size_t(d.n_seqs) * DKV_MAX_UPDATES * kRadixBins * sizeof(int32_t));
  w.tot2 = off;     off += align256(size_t(d.n_seqs) * DKV_MAX_UPDATES * 1024 * sizeof(int32_t));
  w.hist2 = off;    off += align256(size_t(d.n_seqs) * d.n_layers * 1024 * sizeof(int32_t));
  w.above = off;    off += align256(size_t(2) * d.n_seqs * d.n_layers * sizeof(int32_t));
  w.update_block_bytes = off - block;
  off = block + w.update_block_bytes * DKV_MAX_UPDATES;                                 // at most one class per update of a call
  w.picks = off;    off += align256(size_t(DKV_MAX_UPDATES) * d.n_seqs * 4 * sizeof(int32_t));
  w.total = off;
  return w;
}

// ----------------------------------------------------------------------------------------------
// Kernel launch: every kernel of the library goes through launch(), so that dkv_profile_begin() can attach a
// start/stop event pair to each launch (hipExtLaunchKernelGGL) and dkv_profile_end() can report true kernel
// durations on the launch stream. Outside a profiling session this is a plain hipLaunchKernelGGL.
// ----------------------------------------------------------------------------------------------
struct ProfileSession {
  hipEvent_t* start = nullptr;
  hipEvent_t* stop = nullptr;
  int32_t* kernel_id = nullptr;
  std::atomic<int> capacity{0};   // 0: no session (the only thing a launch outside a session reads)
  std::atomic<int> count{0};      // launches that asked for a slot (may pass capacity: those are not recorded)
};
extern ProfileSession g_profile;

template <typename Kernel, typename... Args>
inline void launch(int kernel_id, Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st, Args... args) {
  const int capacity = g_profile.capacity.load(std::memory_order_acquire);
  if (capacity > 0) {                                  // slots are handed out atomically: stage calls from several
    const int i = g_profile.count.fetch_add(1, std::memory_order_relaxed);   // threads may launch during a session
    if (i < capacity) {
      g_profile.kernel_id[i] = kernel_id;
      hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, st, g_profile.start[i], g_profile.stop[i], 0, args...);
      return;
    }
  }
  hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, args...);
}

// Host-side descriptor validation shared by every entry point. Returns DKV_OK or a negative status.
int validate_desc(const dkv_desc* d);

// Resolved launch parameters handed to the kernels by value.
struct Params {
  int L, Hq, Hkv, G, d, w, P, half;   // half = (P-1)/2
  int layer_max, mean_budget, interval;
  int n_seqs, total_tokens, max_seq_len;
  int rows;        // G*w
  int rows_pad;
  float scale;     // softmax scale
  float row_scale;
};

Params make_params(const dkv_desc& d);

// Stage launchers (defined next to their kernels). Each returns hipGetLastError() of its launches.
// `phases` of the score launchers: bit 0 = row-statistics kernel, bit 1 = score kernel.
constexpr int kPhaseStats = 1, kPhaseEmit = 2, kPhaseLse = 4;   // kPhaseLse: export the row normalisers
hipError_t launch_score_generic(const Params& p, int phases, int dtype, const void* q_win, const void* k, int64_t k_stride_token,
                                int64_t k_stride_head, const int32_t* cu, float* scores, int64_t scores_stride_head,
                                char* ws, const WorkspaceLayout& wl, const float* lse_in, float* lse_out, hipStream_t st);
bool score_mfma_supported(const Params& p, int dtype, int64_t k_stride_token);
hipError_t launch_score_mfma(const Params& p, int phases, int n_layers, const void* const* q_layers,
                             const void* const* k_layers, int64_t k_stride_token, int64_t k_stride_head,
                             const int32_t* cu, float* scores, int64_t scores_stride_head, int64_t scores_stride_layer,
                             char* ws, const WorkspaceLayout& wl, const float* lse_in, const float* const* lse_layers,
                             float* lse_out, hipStream_t st);
hipError_t launch_select(const Params& p, int layer, int n_layers, const float* scores, int64_t scores_stride_head,
                         int64_t scores_stride_layer, const int32_t* cu, int32_t* idx_out, int64_t idx_stride_layer,
                         int32_t* counts, char* ws, const WorkspaceLayout& wl, hipStream_t st);
hipError_t launch_pack_cache(const Params& p, int elt_bytes, const int32_t* cu, const int32_t* counts, const void* kb,
                             const void* vb, int64_t stride_layer, int64_t stride_seq, int64_t stride_head,
                             void* k_packed, void* v_packed, int64_t capacity_rows, int64_t* row_offsets,
                             hipStream_t st);
hipError_t launch_decode(const Params& p, int dtype, int layer, int n_layers, const void* q_new, const void* kb,
                         const void* vb, int64_t stride_layer, int64_t stride_seq, int64_t stride_head, const int32_t* cu,
                         const int32_t* counts, float* out, float* lse_out, char* ws, const WorkspaceLayout& wl,
                         hipStream_t st);
hipError_t launch_rebalance(const Params& p, int layers_done, int n_updates, uint32_t epoch, const float* scores_all,
                            const int32_t* cu, int32_t* counts, int32_t* budgets_out, int32_t* hits_out,
                            int64_t out_stride_update, char* ws, const WorkspaceLayout& wl, hipStream_t st);
hipError_t launch_gather(const Params& p, int elt_bytes, int layer, int n_layers, const void* const* k_layers,
                         const void* const* v_layers, int64_t stride_token, int64_t stride_head, const int32_t* cu,
                         const int32_t* idx, int64_t idx_stride_layer, const int32_t* counts, void* k_out, void* v_out,
                         int64_t out_stride_layer, int64_t out_stride_seq, int64_t out_stride_head, hipStream_t st);

hipError_t launch_apply_budgets(const Params& p, int n_layers, const int32_t* budgets, int32_t* counts, hipStream_t st);
hipError_t launch_select_recent(const Params& p, int layer, int n_sink, const int32_t* cu, int32_t* idx_out,
                                int32_t* counts, hipStream_t st);

// ----------------------------------------------------------------------------------------------
// Device helpers
// ----------------------------------------------------------------------------------------------
#if defined(__HIPCC__)
// Maps a linear chunk index to (sequence, chunk within the sequence) when every sequence is cut into
// chunks of `chunk` items and `window_off` is subtracted from each length first (0: all S keys,
// w: the S' prefix positions). Returns false for indices past the last chunk (grids are sized by an
// upper bound). A sequence whose item count is 0 owns no chunk.
__device__ inline bool find_chunk(const int32_t* __restrict__ cu, int n_seqs, int chunk, int window_off, int b,
                                  int& seq, int& c, int& seq_begin, int& seq_len) {
  int begin = cu[0];
  for (int s = 0; s < n_seqs; ++s) {
    const int end = cu[s + 1];
    const int len = end - begin;
    int items = len - window_off;
    items = items > 0 ? items : 0;
    const int n = (items + chunk - 1) / chunk;
    if (b < n) {
      seq = s; c = b; seq_begin = begin; seq_len = len;
      return true;
    }
    b -= n;
    begin = end;
  }
  return false;
}

// ---- wavefront and workgroup prefix sums on DPP moves (a few cycles each; a shuffle through LDS costs a round trip
// per step). All of these must be called by every lane of the wavefront (workgroup), outside divergent branches.

// v + the value of the lane CTRL names, where the rows of ROW_MASK have one; v elsewhere.
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_add_from(int v) {
  return v + __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes.
__device__ inline int wave_prefix_sum(int v) {
  v = dpp_add_from<0x111, 0xf>(v);   // row_shr:1
  v = dpp_add_from<0x112, 0xf>(v);   // row_shr:2
  v = dpp_add_from<0x114, 0xf>(v);   // row_shr:4
  v = dpp_add_from<0x118, 0xf>(v);   // row_shr:8: every row of 16 lanes holds its own prefix sums
  v = dpp_add_from<0x142, 0xa>(v);   // row_bcast:15: rows 1 and 3 add the total of the row before
  v = dpp_add_from<0x143, 0xc>(v);   // row_bcast:31: rows 2 and 3 add the total of the first two
  return v;
}

// Sum over the 16 lanes of a row; every lane of the row gets it.
__device__ inline int row_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);    // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);    // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);   // row_half_mirror
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);   // row_mirror
  return v;
}

// Sum / maximum over the 64 lanes, the same value in every lane.
__device__ inline int wave_sum(int v) {
  v = row_sum(v);
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}
__device__ inline int wave_max(int v) {
#define DKV_MAX_STEP(CTRL)                                                       \
  {                                                                              \
    const int t = __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);       \
    v = t > v ? t : v;                                                           \
  }
  DKV_MAX_STEP(0xB1) DKV_MAX_STEP(0x4E) DKV_MAX_STEP(0x141) DKV_MAX_STEP(0x140)
#undef DKV_MAX_STEP
  const int a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
  const int c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
  const int ab = a > b ? a : b, cd = c > d ? c : d;
  return ab > cd ? ab : cd;
}

// Exclusive prefix sum of one int per thread over a workgroup of up to 16 wavefronts, and the sum over all of them.
// scratch: one int per wavefront (LDS). Two barriers; scratch may be reused after the call.
__device__ inline int block_prefix_sum(int v, int* scratch, int& total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, waves = (blockDim.x + 63) >> 6;
  const int incl = wave_prefix_sum(v);
  if (lane == 63) scratch[wv] = incl;
  __syncthreads();
  const int t = lane < waves ? scratch[lane] : 0;                   // lanes 0..15: the wavefronts' totals
  const int before = __builtin_amdgcn_readfirstlane(row_sum(lane < wv ? t : 0));
  total = __builtin_amdgcn_readfirstlane(row_sum(t));
  __syncthreads();
  return before + incl - v;
}

__device__ inline int chunks_of(int len, int window_off, int chunk) {
  int items = len - window_off;
  items = items > 0 ? items : 0;
  return (items + chunk - 1) / chunk;
}
#endif

}  // namespace dkv
