/*
 * dkv.h - C ABI of the DynamicKV prefill-time KV-cache compression path for AMD MI355X (gfx950).
 *
 * The four stage calls follow the problem statement of the paper (arxiv 2412.14838), Algorithm 1
 * "DynamicKV in Prefill Phase": per layer, score the cached keys against the last ws queries
 * (Eq. 1-2), keep the top B^l positions per KV head (Eq. 3), copy their K/V rows next to the window
 * rows, and every m layers shrink all layers processed so far to the global budget (Section 4.2,
 * Eq. 4-6, function Update_Buffer_Length).
 *
 * Conventions
 *   - plain C; every stage call returns an int status (DKV_OK or a negative DKV_ERR_*); nothing throws.
 *   - every pointer is a DEVICE pointer unless the parameter comment says "host"; the descriptor is host.
 *   - the caller owns every buffer; the library allocates no device memory, keeps no state between
 *     calls except what it writes into the caller's workspace, and never synchronises the stream.
 *   - all work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - arguments are validated on the host before anything is launched; on a negative status nothing
 *     was enqueued.
 *   - sequences are packed along the token axis: sequence s owns tokens [cu_seqlens[s], cu_seqlens[s+1]),
 *     cu_seqlens[0] = 0 and cu_seqlens[n_seqs] = total_tokens;
 *     its length S_s must be >= window for its scores to be meaningful; a sequence with S_s <= window
 *     has no candidate positions (count 0) and only its existing window rows are copied.
 *   - "prefix" of a sequence = its first S' = S - window positions: the candidates for retention.
 */
#ifndef DKV_H
#define DKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DKV_VERSION 1

enum { DKV_F32 = 0, DKV_BF16 = 1 };

enum {
  DKV_OK = 0,
  DKV_ERR_INVALID_ARG = -1, /* null pointer, inconsistent descriptor, misaligned pointer or stride   */
  DKV_ERR_UNSUPPORTED = -2, /* head_dim / dtype / size outside what the kernels are built for        */
  DKV_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or smaller than dkv_workspace_bytes()   */
  DKV_ERR_LAUNCH = -4       /* the HIP runtime refused a launch (hipGetLastError)                    */
};

/* Limits of this build (checked by every call). */
#define DKV_MAX_LAYER_MAX 2048 /* B^l                                        */
#define DKV_MAX_POOL 63        /* pooling kernel size                        */
#define DKV_MAX_ROWS 256       /* G * window: score rows per KV head         */
#define DKV_MAX_SEQS 4096
#define DKV_MAX_LAYERS 512
#define DKV_MAX_KV_HEADS 1024      /* KV heads (a grid dimension of every stage) */
#define DKV_MAX_DECODE_GROUP 16   /* query heads per KV head dkv_decode_attention handles */
#define DKV_MAX_SELECT_LAYERS 32  /* layers one dkv_*_layers call may cover */
#define DKV_MAX_UPDATES 8         /* progressive updates per dkv_rebalance_batch call */

/* Problem descriptor (host memory, read during the call only). Symbols as in Algorithm 1. */
typedef struct dkv_desc {
  int32_t n_layers;     /* L                                                                         */
  int32_t n_q_heads;    /* query heads Hq                                                            */
  int32_t n_kv_heads;   /* KV heads Hkv; Hq % Hkv == 0, G = Hq / Hkv query heads share one KV head   */
  int32_t head_dim;     /* d_k: 64 or 128                                                            */
  int32_t window;       /* ws: observation window = last ws tokens, always retained; >= 1            */
  int32_t pool_kernel;  /* P: size of the 1-D max pooling of Eq. 2 (odd, stride 1, same length)      */
  int32_t layer_max;    /* B^l = (wt - ws) * r_max: per-layer maximum budget per KV head             */
  int32_t mean_budget;  /* wt - ws: mean retained prefix rows per layer per KV head                  */
  int32_t interval;     /* m: layers between two progressive updates                                 */
  int32_t dtype;        /* DKV_F32 or DKV_BF16: element type of q_win, k, v and the gathered copies  */
  int32_t n_seqs;       /* sequences in this launch (ragged lengths allowed)                         */
  int32_t total_tokens; /* T = cu_seqlens[n_seqs]                                                    */
  int32_t max_seq_len;  /* an upper bound on every sequence length (sizes grids and the workspace)   */
  float softmax_scale;  /* 0 => 1/sqrt(d_k) (Eq. 1)                                                  */
  float row_scale;      /* 0 => 1: scores are SUMS over the window rows; 1/ws gives the listing's mean */
} dkv_desc;

/* Kernel identifiers reported by dkv_profile_end(). */
enum {
  DKV_KERNEL_SCORE_STATS = 0,     /* first sweep over K: row statistics              */
  DKV_KERNEL_SCORE_EMIT = 1,      /* second sweep over K: scores, window sum, pooling */
  DKV_KERNEL_SELECT = 2,
  DKV_KERNEL_GATHER = 3,
  DKV_KERNEL_REBALANCE_HIST = 4,
  DKV_KERNEL_REBALANCE_SCAN = 5,
  DKV_KERNEL_REBALANCE_FINAL = 6,
  DKV_KERNEL_FILL = 7,
  DKV_KERNEL_SCORE_BORDERS = 8,   /* pooled scores next to the chunk borders of a multi-layer scoring call */
  DKV_KERNEL_SCORE_LSE = 9,       /* export of the row normalisers                    */
  DKV_KERNEL_PACK = 10,           /* tight packing of the final cache                 */
  DKV_KERNEL_DECODE = 11,         /* decode attention over the compressed cache       */
  DKV_KERNEL_SCORE_MERGE = 12,    /* row normalisers of a multi-layer scoring call    */
  DKV_KERNEL_REBALANCE_PICK = 13, /* digits of the updates' thresholds, between the scans */
  DKV_KERNEL_SCHEDULE = 14        /* fixed-pattern schedules: preset budgets, recency candidates */
};

/* Library version (DKV_VERSION it was built with). Host only. */
int dkv_version(void);

/* Static text for a status code. Host only. */
const char* dkv_status_string(int status);

/* Bytes of device workspace the stage calls need for this descriptor (0 if the descriptor is invalid).
 * Host only, launches nothing. The workspace must be 256-byte aligned; it needs no initialisation and carries
 * nothing from one stage call to the next, except from dkv_score_window_stats to dkv_score_window_emit and, when
 * the caller asks for it with a non-zero epoch, from one dkv_rebalance call of a prefill to the next. */
size_t dkv_workspace_bytes(const dkv_desc* desc);

/*
 * Which kernels a scoring call (Eq. 1-2) with this descriptor and key token stride (elements) runs on: 1 = the bf16
 * matrix-core kernels (bf16, head_dim 128, and a token stride short enough for their 32-bit row offsets: at most
 * about 485 000 elements), 0 = the vector-ALU kernels (everything else the library accepts), negative = a status.
 * Host only, launches nothing.
 */
int dkv_score_path(const dkv_desc* desc, int64_t k_stride_token);

/*
 * Per-kernel timing (a measurement aid, not part of the method). Between dkv_profile_begin(capacity) and
 * dkv_profile_end(...) every kernel the library launches (up to `capacity`) carries a start/stop HIP event pair
 * on its launch stream; dkv_profile_end waits for them, writes the kernel identifiers and durations of the
 * first min(n, max_out) launches in launch order and returns n, the number of launches recorded (or a negative
 * status). The session is the one piece of process-wide state in the library: one session at a time (a second begin
 * returns DKV_ERR_INVALID_ARG), not during stream capture. Stage calls from other threads may run during a session
 * (they take their slots atomically); outside a session a launch reads one integer and is otherwise untouched.
 */
int dkv_profile_begin(int32_t capacity);
int dkv_profile_end(int32_t* kernel_ids_out /* host */, float* microseconds_out /* host */, int32_t max_out);

/*
 * Observation-window scoring of ONE layer (Eq. 1-2; Algorithm 1, the softmax(...).mean(dim=-2).pooling(dim=-1) line).
 * For every sequence and KV head h and prefix position s:
 *     x[g,i,t]  = softmax_scale * <q_win[g,i,:], k[h,t,:]>   for the G query heads g of h, window rows i,
 *                 masked causally (window row i is the token at position S - ws + i);
 *     p[g,i,:]  = softmax over all S keys;
 *     a[h,t]    = row_scale * sum_g sum_i p[g,i,t];
 *     A[h,s]    = max over t in [s - (P-1)/2, s + (P-1)/2] intersected with [0, S') of a[h,t].
 * q_win      [n_seqs][Hq][ws][d], contiguous.
 * k          element (seq s, token t, head h, j) at k[(cu_seqlens[s] + t) * k_stride_token + h * k_stride_head + j];
 *            strides in elements, rows 16-byte aligned.
 * scores_out fp32; A[h,s] of sequence q is written to scores_out[h * scores_stride_head + cu_seqlens[q] + s]
 *            for s < S'; the window slots [S', S) of each sequence longer than the window receive -inf (a
 *            sequence without a prefix has no candidates and its slots are left alone). Candidate scores are >= 0.
 * Accumulation is fp32 (bf16 products are exact in fp32). Two kernels are enqueued (row statistics, then scores).
 */
int dkv_score_window(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                     int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                     int64_t scores_stride_head, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dkv_score_window for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and bit-identical
 * output, but the row statistics that go from the first sweep to the second live in a fixed array inside the
 * library (8 MiB of device memory per GPU the library runs on, held until the process ends) instead of a
 * caller's workspace. The call allocates and frees nothing; the first call on a device looks up the array's device
 * address (the runtime loads the code object that holds the array at that point, if it has not yet), so a caller
 * under stream capture makes one call outside the capture first.
 * Limit: the statistics of one layer, (total_tokens / 256 + n_seqs) * n_kv_heads * rows_pad * 8 bytes with
 * rows_pad = G * ws rounded up to 64, 128 or 256, must fit dkv_static_scratch_limit() (e.g. 8 KV heads, 128 rows:
 * about 260 000 tokens per call); a larger problem returns DKV_ERR_UNSUPPORTED and launches nothing.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams or threads) race
 * on it; calls on one stream are ordered. Nothing in it needs clearing between calls (the first sweep writes
 * every entry the second one reads).
 */
int dkv_score_window_static(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                            int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                            int64_t scores_stride_head, void* stream);
size_t dkv_static_scratch_limit(void);   /* host only: bytes of the fixed array */

/*
 * dkv_score_window (Eq. 1-2) for the n_layers consecutive layers [layer_begin, layer_begin + n_layers) in one call,
 * for a caller that holds the window queries and the keys of a few layers (see dkv_select_topk_layers): a layer's
 * scores depend on that layer's Q and K only. One launch per sweep covers all the layers; a workgroup takes its
 * chunk of keys through the layers one after the other and fetches the next layer's first tiles while it finishes
 * the current one, so the start-up cost of a launch is paid once per call instead of once per layer. Results are
 * identical to n_layers dkv_score_window calls.
 * h_q_layers, h_k_layers  HOST arrays of n_layers DEVICE pointers (Q_win and K of layer layer_begin + i), all with the
 *                         strides given; read during the call only.
 * scores_all              fp32 [L][Hkv][total_tokens] contiguous; the blocks of the layers of the call are written.
 * n_layers                1 .. DKV_MAX_SELECT_LAYERS, layer_begin + n_layers <= L.
 */
int dkv_score_window_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const void* const* h_q_layers,
                            const void* const* h_k_layers, int64_t k_stride_token, int64_t k_stride_head,
                            const int32_t* cu_seqlens, float* scores_all, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * The two kernels of dkv_score_window as separate calls with the same arguments (Eq. 1-2): first the per-row
 * softmax normalisers (log-sum-exp of every window row over all keys, kept in the workspace), then the scores.
 * dkv_score_window(...) is exactly dkv_score_window_stats(...) followed by dkv_score_window_emit(...) on the same
 * stream; the split lets a caller time the two sweeps over K separately or place other work between them.
 * dkv_score_window_emit reads the normalisers the last dkv_score_window_stats call left in `workspace`.
 */
int dkv_score_window_stats(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                           int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                           int64_t scores_stride_head, void* workspace, size_t workspace_bytes, void* stream);
int dkv_score_window_emit(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                          int64_t k_stride_head, const int32_t* cu_seqlens, float* scores_out,
                          int64_t scores_stride_head, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Eq. 1-2 in ONE sweep over K, for a caller that already holds the softmax normalisers of the window rows: the
 * prefill attention of the same layer computes, for every query row, lse = log sum_s exp(scale * <q, k_s>) over
 * the keys the row may see (causal); for the last ws rows that is exactly the denominator of Eq. 1. With it the
 * probabilities are p = exp(scale * <q, k_s> - lse[row]) and the statistics sweep of dkv_score_window is not
 * needed. Same arguments and output as dkv_score_window, plus
 * lse   fp32 [n_seqs][Hq][ws], natural log, row (q, g, i) = window query i of query head g of sequence q.
 * No workspace. The result equals dkv_score_window's up to the rounding of the supplied lse.
 */
int dkv_score_window_lse(const dkv_desc* desc, const void* q_win, const void* k, int64_t k_stride_token,
                         int64_t k_stride_head, const int32_t* cu_seqlens, const float* lse, float* scores_out,
                         int64_t scores_stride_head, void* stream);

/*
 * dkv_score_window_lse for the n_layers consecutive layers [layer_begin, layer_begin + n_layers) in one call (see
 * dkv_score_window_layers): h_lse_layers is a HOST array of n_layers device pointers, one lse tensor per layer in
 * the layout above. Writes the layers' blocks of scores_all. Unlike the single-layer call this one uses the
 * workspace (the normalisers of all layers are first brought into the kernels' own layout by a small kernel).
 */
int dkv_score_window_lse_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers,
                                const void* const* h_q_layers, const void* const* h_k_layers, int64_t k_stride_token,
                                int64_t k_stride_head, const int32_t* cu_seqlens, const float* const* h_lse_layers,
                                float* scores_all, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The normalisers themselves (the denominator of Eq. 1 in log form), from the row statistics that the last
 * dkv_score_window_stats or dkv_score_window call left in `workspace`: lse_out fp32 [n_seqs][Hq][ws], natural log,
 * in the layout dkv_score_window_lse takes. k_stride_token must be the value passed to that call (it selects the
 * kernel family whose statistics are read). After dkv_score_window_layers it is that call's FIRST layer whose
 * normalisers are exported. One small kernel.
 */
int dkv_row_lse(const dkv_desc* desc, int64_t k_stride_token, const int32_t* cu_seqlens, float* lse_out,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-layer, per-KV-head top-k (Eq. 3; Algorithm 1, the A^l.topk(B^l).indices line) for layer index `layer`.
 * For every (sequence, KV head): the k = min(layer_max, S') prefix positions with the largest scores,
 * ORDERED by (score descending, position ascending) - ties go to the lower position - so that a later
 * truncation to the first n entries is again a top-n set.
 * scores     as written by dkv_score_window for this layer.
 * idx_out    int32 [n_seqs][Hkv][layer_max], sequence-local positions; entries >= k are set to -1.
 * counts     int32 [n_seqs][L]; counts[q][layer] = k is written.
 * One kernel (selection of the winners and their ordering, one workgroup per sequence and KV head); the workspace
 * arguments are validated like those of the other calls but the kernel needs no scratch memory.
 */
int dkv_select_topk(const dkv_desc* desc, int32_t layer, const float* scores, int64_t scores_stride_head,
                    const int32_t* cu_seqlens, int32_t* idx_out, int32_t* counts, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * The same selection (Eq. 3) for the n_layers consecutive layers [layer_begin, layer_begin + n_layers) in one
 * call: the selection of a layer depends on that layer's scores only, so a caller that keeps the scores of a
 * few layers (the progressive update needs them anyway) can select them together; one row per (layer,
 * sequence, KV head) then gives the GPU layers-times more workgroups than a single layer does. Results are
 * identical to n_layers dkv_select_topk calls.
 * n_layers    1 .. DKV_MAX_SELECT_LAYERS, layer_begin + n_layers <= L.
 * scores_all  fp32 [L][Hkv][total_tokens] contiguous, as for dkv_rebalance.
 * idx_all     int32 [L][n_seqs][Hkv][layer_max]; the blocks of the selected layers are written.
 * counts      int32 [n_seqs][L]; counts[q][layer] = k is written for the selected layers.
 */
int dkv_select_topk_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const float* scores_all,
                           const int32_t* cu_seqlens, int32_t* idx_all, int32_t* counts, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * Progressive cache update after `layers_done` layers (Section 4.2, Eq. 4-6; Update_Buffer_Length and the
 * truncation loop of Algorithm 1). Per sequence: the kg = min(mean_budget * Hkv * l, l * Hkv * S') largest
 * entries of the scores of layers [0, l) (ties to the lower (layer, head, position)) are counted per layer
 * (cnt_i), then Z_i = floor(layer_max * cnt_i / max cnt), Z'_i = floor(Z_i * mean_budget * L / sum Z)
 * (exact integers), and counts[q][i] <- min(counts[q][i], Z'_i) for i < l.
 * layers_done  l: a positive multiple of desc->interval, <= L.
 * scores_all   fp32 [L][Hkv][total_tokens] contiguous (layer i at scores_all + i * Hkv * total_tokens), 16-byte
 *              aligned.
 * counts       int32 [n_seqs][L], updated in place for layers < l.
 * budgets_out  int32 [n_seqs][L]: Z' for layers < l (others untouched). May be NULL.
 * hits_out     int32 [n_seqs][L]: cnt for layers < l. May be NULL.
 * epoch        names the prefill this call belongs to. 0: the call scans all layers [0, l) and leaves nothing behind.
 *              Non-zero: within one prefill a layer's scores do not change once written, so the call leaves a
 *              histogram of the layers it has scanned in the workspace, and the next call with the SAME epoch,
 *              layers_done + interval, the same scores_all and the same workspace extends it instead of
 *              recounting. A call whose epoch, predecessor or tensors differ, and every call with
 *              layers_done == interval, recounts from scratch. The caller's side of the contract: give every
 *              prefill its own epoch (a counter will do), do not rewrite the scores of layers < l between the
 *              calls of one epoch, and do not share one workspace between prefills that are in flight together.
 */
int dkv_rebalance(const dkv_desc* desc, int32_t layers_done, uint32_t epoch, const float* scores_all,
                  const int32_t* cu_seqlens, int32_t* counts, int32_t* budgets_out, int32_t* hits_out, void* workspace,
                  size_t workspace_bytes, void* stream);

/*
 * The n_updates consecutive updates after layers_done, layers_done + interval, ... layers in one call (Section 4.2
 * as above, once per update): for a caller that has scored and selected the layers of several update intervals
 * before it updates (see dkv_score_window_layers). The updates read the scores only and meet in
 * counts[q][i] <- min(counts[q][i], Z'_i), which commutes, so the result equals n_updates dkv_rebalance calls in
 * order; every kernel of the update takes the updates side by side, and a layer's scores are read once per scan
 * whatever the number of updates that cover the layer.
 * n_updates          1 .. DKV_MAX_UPDATES; layers_done + (n_updates - 1) * interval <= L.
 * budgets_out, hits_out   as for dkv_rebalance, one [n_seqs][L] block per update: update u writes at
 *                    out + u * out_stride_update (ints; >= n_seqs * L when n_updates > 1). May be NULL.
 * The epoch rule of dkv_rebalance applies with the last update's layers_done.
 */
int dkv_rebalance_batch(const dkv_desc* desc, int32_t layers_done, int32_t n_updates, uint32_t epoch,
                        const float* scores_all, const int32_t* cu_seqlens, int32_t* counts, int32_t* budgets_out,
                        int32_t* hits_out, int64_t out_stride_update, void* workspace, size_t workspace_bytes,
                        void* stream);

/*
 * Compaction of the retained K/V rows of layer index `layer` (Algorithm 1, the two cat(gather(...), window) lines).
 * For every (sequence q, KV head h) the output block holds ws + layer_max row slots:
 *     slots [0, ws)              the window rows (positions S - ws .. S - 1, in position order),
 *     slots [ws, ws + count)     the rows at idx[q][h][0 .. count), in that order (count = counts[q][layer]).
 * The window comes first so that truncating a layer to n rows is the prefix [0, ws + n) of its block: the
 * compressed cache is a view of this buffer (attention is invariant to the order of cached rows).
 * k, v       same addressing as k of dkv_score_window (v uses the same strides).
 * k_out,v_out element (q, h, slot, j) at out[q * out_stride_seq + h * out_stride_head + slot * d + j] (elements).
 * Slots >= ws + count are left untouched. Entries of idx outside [0, S') are skipped.
 */
int dkv_gather_kv(const dkv_desc* desc, int32_t layer, const void* k, const void* v, int64_t stride_token,
                  int64_t stride_head, const int32_t* cu_seqlens, const int32_t* idx, const int32_t* counts,
                  void* k_out, void* v_out, int64_t out_stride_seq, int64_t out_stride_head, void* stream);

/*
 * The same compaction (Algorithm 1, the two cat(gather(...), window) lines) for the n_layers consecutive layers
 * [layer_begin, layer_begin + n_layers) in one call, for a caller that selected them together
 * (dkv_select_topk_layers) and still holds their K and V. Results are identical to n_layers dkv_gather_kv calls.
 * h_k_layers, h_v_layers  HOST arrays of n_layers DEVICE pointers: K and V of layer layer_begin + i, all with the
 *                         strides given; the arrays are read during the call only.
 * idx_all                 int32 [L][n_seqs][Hkv][layer_max], as written by dkv_select_topk_layers.
 * k_out_all, v_out_all    element (layer, q, h, slot, j) at
 *                         out[layer * out_stride_layer + q * out_stride_seq + h * out_stride_head + slot * d + j].
 * n_layers                1 .. DKV_MAX_SELECT_LAYERS, layer_begin + n_layers <= L.
 */
int dkv_gather_kv_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const void* const* h_k_layers,
                         const void* const* h_v_layers, int64_t stride_token, int64_t stride_head,
                         const int32_t* cu_seqlens, const int32_t* idx_all, const int32_t* counts, void* k_out_all,
                         void* v_out_all, int64_t out_stride_layer, int64_t out_stride_seq, int64_t out_stride_head,
                         void* stream);

/*
 * The final compressed cache as one tight tensor (Algorithm 1, last line: K^c, V^c <- K^b, V^b after the
 * truncations). The cache dkv_gather_kv builds is already usable in place (block (l, q, h) holds ws + counts[q][l]
 * valid rows); this call copies the valid rows of every block next to each other for a consumer that wants no
 * padding. For block i = q * L + l (sequence q, layer l), n = counts[q][l]:
 *     row_offsets[i]            first packed row of the block (int64, [n_seqs * L + 1], written by the call;
 *                               row_offsets[n_seqs * L] = total rows),
 *     rows of head h            [row_offsets[i] + h * (w_q + n), + w_q + n): the n retained rows in selection
 *                               order, then the w_q window rows in position order (the listing's cat order);
 *                               w_q = min(ws, S_q).
 * kb_all, vb_all   the buffers dkv_gather_kv wrote: element (l, q, h, slot, j) at
 *                  kb[l * stride_layer + q * stride_seq + h * stride_head + slot * d + j] (elements).
 * k_packed, v_packed  [capacity_rows][d]; a block that would end past capacity_rows is not written (its offsets
 *                  still are). n_seqs * L * Hkv * (ws + layer_max) rows always suffice; after the last update
 *                  of a model with L % interval == 0, n_seqs * Hkv * L * (ws + mean_budget) do.
 * Two kernels (offsets by one workgroup, then the copy).
 */
int dkv_pack_cache(const dkv_desc* desc, const int32_t* cu_seqlens, const int32_t* counts, const void* kb_all,
                   const void* vb_all, int64_t stride_layer, int64_t stride_seq, int64_t stride_head, void* k_packed,
                   void* v_packed, int64_t capacity_rows, int64_t* row_offsets, void* stream);

/*
 * Decode-phase attention of one new token per sequence over the compressed cache of layer `layer` (Section 4.3:
 * the decoding phase is unchanged, i.e. ordinary softmax attention over the keys and values the prefill
 * retained). For sequence q and query head g (KV head h = g / G):
 *     out[q][g][:] = sum_r softmax_r(softmax_scale * <q_new[q][g], K_r>) * V_r
 * over the valid rows r of cache block (layer, q, h): its w_q = min(ws, S_q) window rows and its counts[q][layer]
 * retained rows (the new token's own key and value are the caller's to append; they are not part of this sum).
 * q_new    [n_seqs][Hq][d], element type of the descriptor.
 * kb, vb   the layer's block of the cache dkv_gather_kv wrote: element (q, h, slot, j) at
 *          kb[q * stride_seq + h * stride_head + slot * d + j] (elements).
 * out      fp32 [n_seqs][Hq][d]; lse_out fp32 [n_seqs][Hq] (natural log of the softmax denominator) or NULL.
 *          A sequence without any cached row gets zeros and lse = -inf.
 * Hq / Hkv must not exceed DKV_MAX_DECODE_GROUP. All sums in fp32 (for bf16 caches the products run on the matrix
 * cores: bf16 x bf16 is exact there, and the softmax weights enter as two bf16 terms, hi + lo, whose residue is
 * below 2^-17 of the weight). Two kernels (the cache rows are split over workgroups, then merged); the split
 * results live in the workspace.
 */
int dkv_decode_attention(const dkv_desc* desc, int32_t layer, const void* q_new, const void* kb, const void* vb,
                         int64_t stride_seq, int64_t stride_head, const int32_t* cu_seqlens, const int32_t* counts,
                         float* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dkv_decode_attention (Section 4.3) for the n_layers consecutive layers [layer_begin, layer_begin + n_layers) in one
 * call, for a caller that holds the new token's queries of several layers at once (layers evaluated side by side:
 * verification of drafted tokens against stored queries, parallel-attention blocks, a benchmark of the kernel); an
 * ordinary decoder produces layer l+1's query from layer l's output and uses the single-layer call. One layer's
 * cache is a few megabytes and one launch per layer is bound by launch latency; one launch over all layers streams
 * the whole compressed cache. Results are identical to n_layers dkv_decode_attention calls.
 * q_new_all  [n_layers][n_seqs][Hq][d] contiguous: the queries of layer layer_begin + i at index i.
 * kb_all, vb_all  the whole cache dkv_gather_kv wrote: layer l at kb_all + l * stride_layer (elements).
 * out_all    fp32 [n_layers][n_seqs][Hq][d]; lse_all fp32 [n_layers][n_seqs][Hq] or NULL.
 * n_layers   1 .. DKV_MAX_SELECT_LAYERS, layer_begin + n_layers <= L.
 */
int dkv_decode_attention_layers(const dkv_desc* desc, int32_t layer_begin, int32_t n_layers, const void* q_new_all,
                                const void* kb_all, const void* vb_all, int64_t stride_layer, int64_t stride_seq,
                                int64_t stride_head, const int32_t* cu_seqlens, const int32_t* counts, float* out_all,
                                float* lse_all, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fixed-pattern schedules: the comparison methods of Section 5.1 ("Baselines") and Figure 1 (b), (c) as alternative
 * producers of `counts`, through the same scoring, selection and compaction calls. The paper names the patterns
 * and gives no formulas; the readings:
 *   DKV_SCHEDULE_FIXED    Figure 1 (b): every layer keeps mean_budget rows per KV head (with Eq. 1-3 as the
 *                         selection this is the SnapKV-style baseline; no update ever runs).
 *   DKV_SCHEDULE_PYRAMID  Figure 1 (c): retention falls with depth along a straight line from hi rows (layer 0) to
 *                         lo rows (layer L-1), lo = floor(mean_budget / beta), hi = 2 * mean_budget - lo; a hi above
 *                         layer_max is lowered to layer_max and lo raised by the same amount. Layer i gets
 *                         floor(((L-1-i) * hi + i * lo) / (L-1)); L = 1 gets mean_budget. The sum is at most
 *                         mean_budget * L and misses it by less than L.
 * dkv_layer_budgets   HOST only, launches nothing: writes the L budgets of `schedule` to h_budgets_out (host memory).
 *                     beta >= 1 (ignored by DKV_SCHEDULE_FIXED).
 * dkv_apply_budgets   counts[q][i] <- min(counts[q][i], budgets[i]) for i < n_layers and every sequence q: the
 *                     truncation lines of Algorithm 1 with preset budgets. budgets: DEVICE int32 [n_layers].
 *                     Negative budgets count as 0. One kernel.
 * Recipe: per layer dkv_score_window, dkv_select_topk (counts = min(layer_max, S')), dkv_apply_budgets, dkv_gather_kv
 * (or the *_layers forms); nothing else differs from the DynamicKV loop, which calls dkv_rebalance instead.
 */
enum { DKV_SCHEDULE_FIXED = 0, DKV_SCHEDULE_PYRAMID = 1 };
int dkv_layer_budgets(const dkv_desc* desc, int32_t schedule, int32_t beta, int32_t* h_budgets_out /* host */);
int dkv_apply_budgets(const dkv_desc* desc, int32_t n_layers, const int32_t* budgets, int32_t* counts, void* stream);

/*
 * Candidates of the recency pattern (the StreamingLLM-style baseline of Section 5.1: attention sinks plus the most
 * recent tokens) for layer index `layer`, in place of dkv_score_window + dkv_select_topk: no scores are involved.
 * For every (sequence, KV head), k = min(layer_max, S'):
 *     idx_out[q][h][0 .. sinks)   the first sinks = min(n_sink, k) prefix positions, in position order,
 *     idx_out[q][h][sinks .. k)   the prefix positions S'-1, S'-2, ... (newest first),
 * so that the first n entries are again "sinks + the n - sinks most recent" and truncation (dkv_apply_budgets)
 * works as for a score-ordered list; entries >= k are -1; counts[q][layer] = k. The window rows themselves are
 * always kept by dkv_gather_kv. idx_out int32 [n_seqs][Hkv][layer_max]; n_sink >= 0. One kernel.
 */
int dkv_select_recent(const dkv_desc* desc, int32_t layer, int32_t n_sink, const int32_t* cu_seqlens, int32_t* idx_out,
                      int32_t* counts, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DKV_H */
