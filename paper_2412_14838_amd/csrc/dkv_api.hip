// C ABI entry points of libdkv.so: host-side validation, then the stage launchers.
// The operations are those of Algorithm 1 of the paper (DynamicKV in Prefill Phase); see include/dkv.h.
#include <math.h>
#include <mutex>
#include "dkv_internal.h"

namespace dkv {

ProfileSession g_profile;

// Scratch memory of dkv_score_window_static: the row statistics that go from the first sweep to the second live in
// this array instead of a caller's workspace. Every GPU the library runs on holds its own copy at its own address
// until the process ends; host code reaches it only through the address hipGetSymbolAddress returns for the
// current device (the array's name is a host-side stand-in, not a device address).
constexpr size_t kStaticScratchBytes = size_t(8) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (resolved once per device), or nullptr.
static void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

int validate_desc(const dkv_desc* d) {
  if (d == nullptr) return DKV_ERR_INVALID_ARG;
  if (d->n_layers < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->window < 1 || d->n_seqs < 1) return DKV_ERR_INVALID_ARG;
  if (d->n_q_heads % d->n_kv_heads != 0) return DKV_ERR_INVALID_ARG;
  if (d->pool_kernel < 1 || d->pool_kernel % 2 == 0) return DKV_ERR_INVALID_ARG;
  if (d->layer_max < 1 || d->mean_budget < 1 || d->interval < 1) return DKV_ERR_INVALID_ARG;
  if (d->total_tokens < 0 || d->max_seq_len < 0 || d->max_seq_len > d->total_tokens) return DKV_ERR_INVALID_ARG;
  if (!(d->softmax_scale >= 0.0f) || !(d->row_scale >= 0.0f)) return DKV_ERR_INVALID_ARG;
  if (d->dtype != DKV_F32 && d->dtype != DKV_BF16) return DKV_ERR_UNSUPPORTED;
  if (d->head_dim != 64 && d->head_dim != 128) return DKV_ERR_UNSUPPORTED;
  if (d->layer_max > DKV_MAX_LAYER_MAX || d->pool_kernel > DKV_MAX_POOL) return DKV_ERR_UNSUPPORTED;
  if ((d->n_q_heads / d->n_kv_heads) * (int64_t)d->window > DKV_MAX_ROWS) return DKV_ERR_UNSUPPORTED;
  if (d->n_seqs > DKV_MAX_SEQS || d->n_layers > DKV_MAX_LAYERS || d->n_kv_heads > DKV_MAX_KV_HEADS) return DKV_ERR_UNSUPPORTED;
  // 64-bit budget arithmetic must not overflow: layer_max * (L * Hkv * S') and Z * B
  if ((int64_t)d->n_layers * d->n_kv_heads * (int64_t)d->max_seq_len > (int64_t)1 << 31) return DKV_ERR_UNSUPPORTED;
  return DKV_OK;
}

Params make_params(const dkv_desc& d) {
  Params p{};
  p.L = d.n_layers; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  p.d = d.head_dim; p.w = d.window; p.P = d.pool_kernel; p.half = (d.pool_kernel - 1) / 2;
  p.layer_max = d.layer_max; p.mean_budget = d.mean_budget; p.interval = d.interval;
  p.n_seqs = d.n_seqs; p.total_tokens = d.total_tokens; p.max_seq_len = d.max_seq_len;
  p.rows = p.G * p.w; p.rows_pad = padded_rows(p.rows);
  p.scale = d.softmax_scale > 0.0f ? d.softmax_scale : 1.0f / sqrtf((float)d.head_dim);
  p.row_scale = d.row_scale > 0.0f ? d.row_scale : 1.0f;
  return p;
}

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

static int check_workspace(const dkv_desc& d, const void* ws, size_t bytes, WorkspaceLayout& wl) {
  wl = workspace_layout(d);
  if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255) != 0 || bytes < wl.total) return DKV_ERR_WORKSPACE;
  return DKV_OK;
}

static int check_kv_strides(const dkv_desc& d, int64_t stride_token, int64_t stride_head) {
  const int64_t elt = d.dtype == DKV_BF16 ? 2 : 4;
  if (stride_token < d.head_dim || stride_head < d.head_dim) return DKV_ERR_INVALID_ARG;
  if ((stride_token * elt) % 16 != 0 || (stride_head * elt) % 16 != 0) return DKV_ERR_INVALID_ARG;
  return DKV_OK;
}

}  // namespace dkv

using namespace dkv;

extern "C" {

int dkv_version(void) { return DKV_VERSION; }

const char* dkv_status_string(int status) {
  switch (status) {
    case DKV_OK: return "ok";
    case DKV_ERR_INVALID_ARG: return "invalid argument";
    case DKV_ERR_UNSUPPORTED: return "unsupported head_dim, dtype or size";
    case DKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DKV_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

static std::mutex g_profile_mutex;   // begin / end exclude each other; launches take their slots atomically

static void profile_release(int created) {
  for (int j = 0; j < created; ++j) { (void)hipEventDestroy(g_profile.start[j]); (void)hipEventDestroy(g_profile.stop[j]); }
  delete[] g_profile.start; delete[] g_profile.stop; delete[] g_profile.kernel_id;
  g_profile.start = g_profile.stop = nullptr;
  g_profile.kernel_id = nullptr;
  g_profile.count.store(0);
}

int dkv_profile_begin(int32_t capacity) {
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  if (capacity < 1 || g_profile.capacity.load() != 0) return DKV_ERR_INVALID_ARG;
  g_profile.start = new hipEvent_t[capacity];
  g_profile.stop = new hipEvent_t[capacity];
  g_profile.kernel_id = new int32_t[capacity];
  for (int i = 0; i < capacity; ++i) {
    const bool a = hipEventCreate(&g_profile.start[i]) == hipSuccess;
    const bool b = a && hipEventCreate(&g_profile.stop[i]) == hipSuccess;
    if (!b) {
      if (a) (void)hipEventDestroy(g_profile.start[i]);
      profile_release(i);
      return DKV_ERR_LAUNCH;
    }
  }
  g_profile.count.store(0);
  g_profile.capacity.store(capacity, std::memory_order_release);   // from here on launches record
  return DKV_OK;
}

int dkv_profile_end(int32_t* kernel_ids_out, float* microseconds_out, int32_t max_out) {
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  const int capacity = g_profile.capacity.exchange(0);              // launches stop recording first
  if (capacity == 0) return DKV_ERR_INVALID_ARG;
  const int asked = g_profile.count.load();
  const int n = asked < capacity ? asked : capacity;
  int status = DKV_OK;
  for (int i = 0; i < n; ++i) {
    float ms = 0.0f;
    if (hipEventSynchronize(g_profile.stop[i]) != hipSuccess ||
        hipEventElapsedTime(&ms, g_profile.start[i], g_profile.stop[i]) != hipSuccess) status = DKV_ERR_LAUNCH;
    if (i < max_out && kernel_ids_out && microseconds_out) {
      kernel_ids_out[i] = g_profile.kernel_id[i];
      microseconds_out[i] = ms * 1000.0f;
    }
  }
  profile_release(capacity);
  return status == DKV_OK ? n : status;
}

int dkv_score_path(const dkv_desc* desc, int64_t k_stride_token) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  st = check_kv_strides(*desc, k_stride_token, desc->head_dim);
  if (st != DKV_OK) return st;
  return score_mfma_supported(make_params(*desc), desc->dtype, k_stride_token) ? 1 : 0;
}

size_t dkv_workspace_bytes(const dkv_desc* desc) {
  if (validate_desc(desc) != DKV_OK) return 0;
  return workspace_layout(*desc).total;
}

// Common body of the score entry points: n_layers layers (q_layers / k_layers: host arrays of device pointers),
// scores of layer i at scores_out + i * scores_stride_layer.
static int score_window_phases(int phases, const dkv_desc* desc, int n_layers, const void* const* q_layers,
                               const void* const* k_layers, int64_t k_stride_token, int64_t k_stride_head,
                               const int32_t* cu_seqlens, float* scores_out, int64_t scores_stride_head,
                               int64_t scores_stride_layer, void* workspace, size_t workspace_bytes,
                               const float* lse_in, float* lse_out, void* stream,
                               const float* const* lse_layers = nullptr, bool static_scratch = false) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  const bool sweeps = (phases & (kPhaseStats | kPhaseEmit)) != 0;       // reads Q and K
  if (!cu_seqlens) return DKV_ERR_INVALID_ARG;
  if (sweeps) {
    if (!q_layers || !k_layers) return DKV_ERR_INVALID_ARG;
    for (int i = 0; i < n_layers; ++i)
      if (!q_layers[i] || !k_layers[i] || !aligned16(q_layers[i]) || !aligned16(k_layers[i])) return DKV_ERR_INVALID_ARG;
  }
  if ((phases & kPhaseEmit) && !scores_out) return DKV_ERR_INVALID_ARG;
  if ((phases & kPhaseLse) && !lse_out) return DKV_ERR_INVALID_ARG;
  st = check_kv_strides(*desc, k_stride_token, k_stride_head);
  if (st != DKV_OK) return st;
  if ((phases & kPhaseEmit) && scores_stride_head < desc->total_tokens) return DKV_ERR_INVALID_ARG;
  WorkspaceLayout wl{};
  if (lse_layers)
    for (int i = 0; i < n_layers; ++i)
      if (!lse_layers[i]) return DKV_ERR_INVALID_ARG;
  const bool needs_workspace = phases != kPhaseEmit || lse_in == nullptr;   // everything but the single-layer single sweep
  if (static_scratch) {
    // one layer, both sweeps: only the first layer's share of the row statistics is used
    wl = workspace_layout(*desc);
    if (n_layers != 1 || wl.partials + wl.partials_layer_bytes > kStaticScratchBytes) return DKV_ERR_UNSUPPORTED;
    workspace = static_scratch_ptr();
    if (workspace == nullptr) return DKV_ERR_LAUNCH;
  } else if (needs_workspace) {
    st = check_workspace(*desc, workspace, workspace_bytes, wl);
    if (st != DKV_OK) return st;
  } else {
    workspace = nullptr;
  }
  if (desc->total_tokens == 0) return DKV_OK;
  const Params p = make_params(*desc);
  const hipStream_t hs = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  if (score_mfma_supported(p, desc->dtype, k_stride_token)) {
    e = launch_score_mfma(p, phases, n_layers, q_layers, k_layers, k_stride_token, k_stride_head, cu_seqlens, scores_out,
                          scores_stride_head, scores_stride_layer, static_cast<char*>(workspace), wl, lse_in, lse_layers,
                          lse_out, hs);
  } else {
    // the vector-ALU kernels take one layer at a time (both sweeps of a layer before the next layer's)
    for (int i = 0; i < (sweeps ? n_layers : 1) && e == hipSuccess; ++i)
      e = launch_score_generic(p, phases, desc->dtype, sweeps ? q_layers[i] : nullptr, sweeps ? k_layers[i] : nullptr,
                               k_stride_token, k_stride_head, cu_seqlens,
                               scores_out ? scores_out + i * scores_stride_layer : nullptr, scores_stride_head,
                               static_cast<char*>(workspace), wl, lse_layers ? lse_layers[i] : lse_in, lse_out, hs);
  }
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_score_window(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                     int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                     int64_t scores_stride_head, void* workspace, size_t workspace_bytes, void* stream) {
  return score_window_phases(kPhaseStats | kPhaseEmit, desc, 1, &q_win, &k, k_stride_token, k_stride_head, cu_seqlens,
                             scores_out, scores_stride_head, 0, workspace, workspace_bytes, nullptr, nullptr, stream);
}

int dkv_score_window_static(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                            int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                            int64_t scores_stride_head, void* stream) {
  return score_window_phases(kPhaseStats | kPhaseEmit, desc, 1, &q_win, &k, k_stride_token, k_stride_head, cu_seqlens,
                             scores_out, scores_stride_head, 0, nullptr, 0, nullptr, nullptr, stream, nullptr, true);
}

size_t dkv_static_scratch_limit(void) { return kStaticScratchBytes; }

int dkv_score_window_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const void* const* h_q_layers,
                            const void* const* h_k_layers, int64_t k_stride_token, int64_t k_stride_head,
                            const int32_t* cu_seqlens, float* scores_all, void* workspace, size_t workspace_bytes,
                            void* stream) {
  const int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!scores_all) return DKV_ERR_INVALID_ARG;
  if (n_layers < 1 || n_layers > DKV_MAX_SELECT_LAYERS) return DKV_ERR_INVALID_ARG;
  if (layer_begin < 0 || layer_begin + n_layers > desc->n_layers) return DKV_ERR_INVALID_ARG;
  const int64_t stride_layer = (int64_t)desc->n_kv_heads * desc->total_tokens;
  return score_window_phases(kPhaseStats | kPhaseEmit, desc, n_layers, h_q_layers, h_k_layers, k_stride_token,
                             k_stride_head, cu_seqlens, scores_all + layer_begin * stride_layer, desc->total_tokens,
                             stride_layer, workspace, workspace_bytes, nullptr, nullptr, stream);
}

int dkv_score_window_stats(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                           int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                           int64_t scores_stride_head, void* workspace, size_t workspace_bytes, void* stream) {
  return score_window_phases(kPhaseStats, desc, 1, &q_win, &k, k_stride_token, k_stride_head, cu_seqlens, scores_out,
                             scores_stride_head, 0, workspace, workspace_bytes, nullptr, nullptr, stream);
}

int dkv_score_window_emit(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                          int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                          int64_t scores_stride_head, void* workspace, size_t workspace_bytes, void* stream) {
  return score_window_phases(kPhaseEmit, desc, 1, &q_win, &k, k_stride_token, k_stride_head, cu_seqlens, scores_out,
                             scores_stride_head, 0, workspace, workspace_bytes, nullptr, nullptr, stream);
}

int dkv_score_window_lse(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                         int64_t k_stride_head, const int32_t* cu_seqlens, const float* lse, float* scores_out,
                         int64_t scores_stride_head, void* stream) {
  if (!lse) return DKV_ERR_INVALID_ARG;
  return score_window_phases(kPhaseEmit, desc, 1, &q_win, &k, k_stride_token, k_stride_head, cu_seqlens, scores_out,
                             scores_stride_head, 0, nullptr, 0, lse, nullptr, stream);
}

int dkv_score_window_lse_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers,
                                const void* const* h_q_layers, const void* const* h_k_layers, int64_t k_stride_token,
                                int64_t k_stride_head, const int32_t* cu_seqlens, const float* const* h_lse_layers,
                                float* scores_all, void* workspace, size_t workspace_bytes, void* stream) {
  const int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!scores_all || !h_lse_layers) return DKV_ERR_INVALID_ARG;
  if (n_layers < 1 || n_layers > DKV_MAX_SELECT_LAYERS) return DKV_ERR_INVALID_ARG;
  if (layer_begin < 0 || layer_begin + n_layers > desc->n_layers) return DKV_ERR_INVALID_ARG;
  const int64_t stride_layer = (int64_t)desc->n_kv_heads * desc->total_tokens;
  return score_window_phases(kPhaseEmit, desc, n_layers, h_q_layers, h_k_layers, k_stride_token, k_stride_head,
                             cu_seqlens, scores_all + layer_begin * stride_layer, desc->total_tokens, stride_layer,
                             workspace, workspace_bytes, nullptr, nullptr, stream, h_lse_layers);
}

int dkv_row_lse(const dkv_desc* desc, int64_t k_stride_token, const int32_t* cu_seqlens, float* lse_out,
                void* workspace, size_t workspace_bytes, void* stream) {
  if (!desc) return DKV_ERR_INVALID_ARG;
  return score_window_phases(kPhaseLse, desc, 1, nullptr, nullptr, k_stride_token, (int64_t)desc->head_dim, cu_seqlens,
                             nullptr, 0, 0, workspace, workspace_bytes, nullptr, lse_out, stream);
}

int dkv_select_topk(const dkv_desc* desc, int32_t layer, const float* scores, int64_t scores_stride_head,
                    const int32_t* cu_seqlens, int32_t* idx_out, int32_t* counts, void* workspace,
                    size_t workspace_bytes, void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!scores || !cu_seqlens || !idx_out || !counts) return DKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= desc->n_layers) return DKV_ERR_INVALID_ARG;
  if (scores_stride_head < desc->total_tokens) return DKV_ERR_INVALID_ARG;
  WorkspaceLayout wl;
  st = check_workspace(*desc, workspace, workspace_bytes, wl);
  if (st != DKV_OK) return st;
  const Params p = make_params(*desc);
  const hipError_t e = launch_select(p, layer, 1, scores, scores_stride_head, 0, cu_seqlens, idx_out, 0, counts,
                                     static_cast<char*>(workspace), wl, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_select_topk_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const float* scores_all,
                           const int32_t* cu_seqlens, int32_t* idx_all, int32_t* counts, void* workspace,
                           size_t workspace_bytes, void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!scores_all || !cu_seqlens || !idx_all || !counts) return DKV_ERR_INVALID_ARG;
  if (n_layers < 1 || n_layers > DKV_MAX_SELECT_LAYERS) return DKV_ERR_INVALID_ARG;
  if (layer_begin < 0 || layer_begin + n_layers > desc->n_layers) return DKV_ERR_INVALID_ARG;
  WorkspaceLayout wl;
  st = check_workspace(*desc, workspace, workspace_bytes, wl);
  if (st != DKV_OK) return st;
  const Params p = make_params(*desc);
  const int64_t scores_stride_layer = (int64_t)desc->n_kv_heads * desc->total_tokens;
  const int64_t idx_stride_layer = (int64_t)desc->n_seqs * desc->n_kv_heads * desc->layer_max;
  const hipError_t e = launch_select(p, layer_begin, n_layers, scores_all + layer_begin * scores_stride_layer,
                                     desc->total_tokens, scores_stride_layer, cu_seqlens,
                                     idx_all + layer_begin * idx_stride_layer, idx_stride_layer, counts,
                                     static_cast<char*>(workspace), wl, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_rebalance_batch(const dkv_desc* desc, int32_t layers_done, int32_t n_updates, uint32_t epoch,
                        const float* scores_all, const int32_t* cu_seqlens, int32_t* counts, int32_t* budgets_out,
                        int32_t* hits_out, int64_t out_stride_update, void* workspace, size_t workspace_bytes,
                        void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!scores_all || !cu_seqlens || !counts || !aligned16(scores_all)) return DKV_ERR_INVALID_ARG;
  if (n_updates < 1 || n_updates > DKV_MAX_UPDATES) return DKV_ERR_INVALID_ARG;
  if (layers_done < 1 || layers_done % desc->interval != 0) return DKV_ERR_INVALID_ARG;
  if ((int64_t)layers_done + (int64_t)(n_updates - 1) * desc->interval > desc->n_layers) return DKV_ERR_INVALID_ARG;
  if (n_updates > 1 && (budgets_out || hits_out) && out_stride_update < (int64_t)desc->n_seqs * desc->n_layers)
    return DKV_ERR_INVALID_ARG;
  WorkspaceLayout wl;
  st = check_workspace(*desc, workspace, workspace_bytes, wl);
  if (st != DKV_OK) return st;
  const Params p = make_params(*desc);
  const hipError_t e = launch_rebalance(p, layers_done, n_updates, epoch, scores_all, cu_seqlens, counts, budgets_out, hits_out,
                                        out_stride_update, static_cast<char*>(workspace), wl,
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_rebalance(const dkv_desc* desc, int32_t layers_done, uint32_t epoch, const float* scores_all,
                  const int32_t* cu_seqlens, int32_t* counts, int32_t* budgets_out, int32_t* hits_out, void* workspace,
                  size_t workspace_bytes, void* stream) {
  return dkv_rebalance_batch(desc, layers_done, 1, epoch, scores_all, cu_seqlens, counts, budgets_out, hits_out, 0,
                             workspace, workspace_bytes, stream);
}

int dkv_gather_kv(const dkv_desc* desc, int32_t layer, const void* k, const void* v, int64_t stride_token,
                  int64_t stride_head, const int32_t* cu_seqlens, const int32_t* idx, const int32_t* counts,
                  void* k_out, void* v_out, int64_t out_stride_seq, int64_t out_stride_head, void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!k || !v || !cu_seqlens || !idx || !counts || !k_out || !v_out) return DKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= desc->n_layers) return DKV_ERR_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out)) return DKV_ERR_INVALID_ARG;
  st = check_kv_strides(*desc, stride_token, stride_head);
  if (st != DKV_OK) return st;
  const int64_t elt = desc->dtype == DKV_BF16 ? 2 : 4;
  const int64_t block = (int64_t)(desc->window + desc->layer_max) * desc->head_dim;
  if (out_stride_head < block || out_stride_seq < out_stride_head * desc->n_kv_heads) return DKV_ERR_INVALID_ARG;
  if ((out_stride_head * elt) % 16 != 0 || (out_stride_seq * elt) % 16 != 0) return DKV_ERR_INVALID_ARG;
  const Params p = make_params(*desc);
  const hipError_t e = launch_gather(p, (int)elt, layer, 1, &k, &v, stride_token, stride_head, cu_seqlens, idx, 0,
                                     counts, k_out, v_out, 0, out_stride_seq, out_stride_head,
                                     static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_gather_kv_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const void* const* h_k_layers,
                         const void* const* h_v_layers, int64_t stride_token, int64_t stride_head,
                         const int32_t* cu_seqlens, const int32_t* idx_all, const int32_t* counts, void* k_out_all,
                         void* v_out_all, int64_t out_stride_layer, int64_t out_stride_seq, int64_t out_stride_head,
                         void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!h_k_layers || !h_v_layers || !cu_seqlens || !idx_all || !counts || !k_out_all || !v_out_all)
    return DKV_ERR_INVALID_ARG;
  if (n_layers < 1 || n_layers > DKV_MAX_SELECT_LAYERS) return DKV_ERR_INVALID_ARG;
  if (layer_begin < 0 || layer_begin + n_layers > desc->n_layers) return DKV_ERR_INVALID_ARG;
  for (int i = 0; i < n_layers; ++i)
    if (!h_k_layers[i] || !h_v_layers[i] || !aligned16(h_k_layers[i]) || !aligned16(h_v_layers[i]))
      return DKV_ERR_INVALID_ARG;
  if (!aligned16(k_out_all) || !aligned16(v_out_all)) return DKV_ERR_INVALID_ARG;
  st = check_kv_strides(*desc, stride_token, stride_head);
  if (st != DKV_OK) return st;
  const int64_t elt = desc->dtype == DKV_BF16 ? 2 : 4;
  const int64_t block = (int64_t)(desc->window + desc->layer_max) * desc->head_dim;
  if (out_stride_head < block || out_stride_seq < out_stride_head * desc->n_kv_heads) return DKV_ERR_INVALID_ARG;
  if (out_stride_layer < out_stride_seq * desc->n_seqs) return DKV_ERR_INVALID_ARG;
  if ((out_stride_head * elt) % 16 != 0 || (out_stride_seq * elt) % 16 != 0 || (out_stride_layer * elt) % 16 != 0)
    return DKV_ERR_INVALID_ARG;
  const Params p = make_params(*desc);
  const int64_t idx_stride_layer = (int64_t)desc->n_seqs * desc->n_kv_heads * desc->layer_max;
  const hipError_t e = launch_gather(
      p, (int)elt, layer_begin, n_layers, h_k_layers, h_v_layers, stride_token, stride_head, cu_seqlens,
      idx_all + layer_begin * idx_stride_layer, idx_stride_layer, counts,
      static_cast<char*>(k_out_all) + layer_begin * out_stride_layer * elt,
      static_cast<char*>(v_out_all) + layer_begin * out_stride_layer * elt, out_stride_layer, out_stride_seq,
      out_stride_head, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_pack_cache(const dkv_desc* desc, const int32_t* cu_seqlens, const int32_t* counts, const void* kb_all,
                   const void* vb_all, int64_t stride_layer, int64_t stride_seq, int64_t stride_head, void* k_packed,
                   void* v_packed, int64_t capacity_rows, int64_t* row_offsets, void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!cu_seqlens || !counts || !kb_all || !vb_all || !k_packed || !v_packed || !row_offsets) return DKV_ERR_INVALID_ARG;
  if (!aligned16(kb_all) || !aligned16(vb_all) || !aligned16(k_packed) || !aligned16(v_packed)) return DKV_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(row_offsets) % 8 != 0 || capacity_rows < 0) return DKV_ERR_INVALID_ARG;
  const int64_t elt = desc->dtype == DKV_BF16 ? 2 : 4;
  const int64_t block = (int64_t)(desc->window + desc->layer_max) * desc->head_dim;
  if (stride_head < block || stride_seq < stride_head * desc->n_kv_heads || stride_layer < stride_seq * desc->n_seqs)
    return DKV_ERR_INVALID_ARG;
  if ((stride_head * elt) % 16 != 0 || (stride_seq * elt) % 16 != 0 || (stride_layer * elt) % 16 != 0)
    return DKV_ERR_INVALID_ARG;
  const Params p = make_params(*desc);
  const hipError_t e = launch_pack_cache(p, (int)elt, cu_seqlens, counts, kb_all, vb_all, stride_layer, stride_seq,
                                         stride_head, k_packed, v_packed, capacity_rows, row_offsets,
                                         static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_decode_attention(const dkv_desc* desc, int32_t layer, const void* q_new, const void* kb, const void* vb,
                         int64_t stride_seq, int64_t stride_head, const int32_t* cu_seqlens, const int32_t* counts,
                         float* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!q_new || !kb || !vb || !cu_seqlens || !counts || !out) return DKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= desc->n_layers) return DKV_ERR_INVALID_ARG;
  if (!aligned16(kb) || !aligned16(vb)) return DKV_ERR_INVALID_ARG;
  if (desc->n_q_heads / desc->n_kv_heads > DKV_MAX_DECODE_GROUP) return DKV_ERR_UNSUPPORTED;
  const int64_t elt = desc->dtype == DKV_BF16 ? 2 : 4;
  const int64_t block = (int64_t)(desc->window + desc->layer_max) * desc->head_dim;
  if (stride_head < block || stride_seq < stride_head * desc->n_kv_heads) return DKV_ERR_INVALID_ARG;
  if ((stride_head * elt) % 16 != 0 || (stride_seq * elt) % 16 != 0) return DKV_ERR_INVALID_ARG;
  WorkspaceLayout wl;
  st = check_workspace(*desc, workspace, workspace_bytes, wl);
  if (st != DKV_OK) return st;
  const Params p = make_params(*desc);
  const hipError_t e = launch_decode(p, desc->dtype, layer, 1, q_new, kb, vb, 0, stride_seq, stride_head, cu_seqlens,
                                     counts, out, lse_out, static_cast<char*>(workspace), wl,
                                     static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_decode_attention_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const void* q_new_all,
                                const void* kb_all, const void* vb_all, int64_t stride_layer, int64_t stride_seq,
                                int64_t stride_head, const int32_t* cu_seqlens, const int32_t* counts, float* out_all,
                                float* lse_all, void* workspace, size_t workspace_bytes, void* stream) {
  int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!q_new_all || !kb_all || !vb_all || !cu_seqlens || !counts || !out_all) return DKV_ERR_INVALID_ARG;
  if (n_layers < 1 || n_layers > DKV_MAX_SELECT_LAYERS) return DKV_ERR_INVALID_ARG;
  if (layer_begin < 0 || layer_begin + n_layers > desc->n_layers) return DKV_ERR_INVALID_ARG;
  if (!aligned16(kb_all) || !aligned16(vb_all)) return DKV_ERR_INVALID_ARG;
  if (desc->n_q_heads / desc->n_kv_heads > DKV_MAX_DECODE_GROUP) return DKV_ERR_UNSUPPORTED;
  const int64_t elt = desc->dtype == DKV_BF16 ? 2 : 4;
  const int64_t block = (int64_t)(desc->window + desc->layer_max) * desc->head_dim;
  if (stride_head < block || stride_seq < stride_head * desc->n_kv_heads || stride_layer < stride_seq * desc->n_seqs)
    return DKV_ERR_INVALID_ARG;
  if ((stride_head * elt) % 16 != 0 || (stride_seq * elt) % 16 != 0 || (stride_layer * elt) % 16 != 0)
    return DKV_ERR_INVALID_ARG;
  WorkspaceLayout wl;
  st = check_workspace(*desc, workspace, workspace_bytes, wl);
  if (st != DKV_OK) return st;
  const Params p = make_params(*desc);
  const hipError_t e = launch_decode(
      p, desc->dtype, layer_begin, n_layers, q_new_all, static_cast<const char*>(kb_all) + layer_begin * stride_layer * elt,
      static_cast<const char*>(vb_all) + layer_begin * stride_layer * elt, stride_layer, stride_seq, stride_head, cu_seqlens,
      counts, out_all, lse_all, static_cast<char*>(workspace), wl, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_layer_budgets(const dkv_desc* desc, int32_t schedule, int32_t beta, int32_t* h_budgets_out) {
  const int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!h_budgets_out || beta < 1) return DKV_ERR_INVALID_ARG;
  const int64_t L = desc->n_layers, mean = desc->mean_budget;
  if (schedule == DKV_SCHEDULE_FIXED || L == 1) {
    if (schedule != DKV_SCHEDULE_FIXED && schedule != DKV_SCHEDULE_PYRAMID) return DKV_ERR_INVALID_ARG;
    for (int64_t i = 0; i < L; ++i) h_budgets_out[i] = (int32_t)mean;
    return DKV_OK;
  }
  if (schedule != DKV_SCHEDULE_PYRAMID) return DKV_ERR_INVALID_ARG;
  int64_t lo = mean / beta, hi = 2 * mean - lo;
  if (hi > desc->layer_max) {
    lo += hi - desc->layer_max;
    hi = desc->layer_max;
  }
  for (int64_t i = 0; i < L; ++i) h_budgets_out[i] = (int32_t)(((L - 1 - i) * hi + i * lo) / (L - 1));
  return DKV_OK;
}

int dkv_apply_budgets(const dkv_desc* desc, int32_t n_layers, const int32_t* budgets, int32_t* counts, void* stream) {
  const int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!budgets || !counts || n_layers < 1 || n_layers > desc->n_layers) return DKV_ERR_INVALID_ARG;
  const Params p = make_params(*desc);
  const hipError_t e = launch_apply_budgets(p, n_layers, budgets, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

int dkv_select_recent(const dkv_desc* desc, int32_t layer, int32_t n_sink, const int32_t* cu_seqlens, int32_t* idx_out,
                      int32_t* counts, void* stream) {
  const int st = validate_desc(desc);
  if (st != DKV_OK) return st;
  if (!cu_seqlens || !idx_out || !counts || n_sink < 0) return DKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= desc->n_layers) return DKV_ERR_INVALID_ARG;
  const Params p = make_params(*desc);
  const hipError_t e = launch_select_recent(p, layer, n_sink, cu_seqlens, idx_out, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DKV_OK : DKV_ERR_LAUNCH;
}

}  // extern "C"
