// Observation-window scoring on the bf16 matrix cores (Eq. 1-2; Algorithm 1: softmax(Q_win K^T).mean(-2).pooling(-1)).
// bf16 inputs, head size 128, up to 256 score rows (G * ws) per KV head.
//
// A column of softmax(QK^T) summed over the rows needs every row's normaliser before any column can be
// finished, so the keys are swept twice (the second read is expected to come from the cache hierarchy):
//   stats kernel: S_tile = K_tile . Q^T  (keys as the MFMA M index, rows as N: a lane holds ONE row and 16
//                 keys, so the running row maximum / sum of exponentials is an in-lane reduction); every
//                 workgroup writes one partial (max, sum) per row for its chunk of keys;
//   merge:        the chunk partials of a (sequence, head) become lse2[row] (kernel boundaries are the only
//                 synchronisation between workgroups): in the emit kernel's prologue for a single layer, in a
//                 small kernel of its own when a call covers several layers;
//   emit kernel:  S_tile = Q . K_tile^T (rows as M, keys as N: a lane holds ONE key and 16 rows, so the sum over
//                 the rows is an in-lane reduction), p = exp2(S * c - lse2[row]), window/group sum, max-pool,
//                 write.
// Both use v_mfma_f32_32x32x16_bf16 with the whole Q block of the wavefront resident in registers and K tiles
// staged through LDS (coalesced 16-byte global loads, padded rows, 16-byte LDS reads in MFMA operand layout).
// The MFMAs of one tile are issued in the same step as the exponentials of the tile before it (two accumulator
// sets), while the loads of the tile three steps on are issued and the tile two steps on goes to LDS.
//
// Workgroup = RS x KS wavefronts: RS row slabs of 64 rows (2 MFMA tiles) x KS key tiles of 32 keys.
// Every workgroup owns a contiguous chunk of one (sequence, KV head) and takes it through all layers of the call
// (up to DKV_MAX_SELECT_LAYERS): the key tiles of the layers form one stream of steps, the next layer's Q and
// normalisers arrive while the current layer's last steps run. Pooling across the borders of the output chunks:
// a single-layer call computes (P-1)/2 extra keys on each side of its chunk, so that it never needs another
// workgroup's sums; a multi-layer call computes its own keys only, leaves the column sums next to the borders in the
// workspace, and one small kernel for all layers (score_fix_borders) completes the outputs there. Identical keys
// give bit-identical sums whichever workgroup or lane computes them (fixed summation order per column), and a
// layer gets the same bits whether it is scored alone or as part of a multi-layer call.
#include "dkv_internal.h"

#include <type_traits>

namespace dkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kLdsRow = 272;          // bytes per staged key row: 256 data + 16 pad (conflict-free 16-byte reads)
constexpr int kLdsBudget = 152 * 1024; // dynamic LDS a workgroup may ask for (160 KB per compute unit, less the static part)
constexpr int kMaxHalo = 64;          // >= 2 * half
constexpr float kLog2e = 1.4426950408889634f;

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int RS, int KS>
struct Tile {
  static constexpr int kThreads = RS * KS * 64;
  static constexpr int kKeys = KS * 32;                       // keys per iteration
  static constexpr int kPieces = kKeys * 16 / kThreads;       // 16-byte pieces per thread per tile
  static constexpr int kTileBytes = kKeys * kLdsRow;
};

// The Q block of one (sequence, KV head) - up to RS * 64 rows of 128 - goes through LDS once per workgroup
// (every row is needed by KS wavefronts): load_q_pieces() fetches kQPieces 16-byte pieces per thread (rows past
// `rows` are zero), store_q_pieces() puts them into `qbuf` in the padded row layout of the key tiles, and after a
// barrier read_q_frags() gives each wavefront the fragments of its 64 rows in MFMA operand layout:
// qf[t][j] = 8 consecutive head-dim elements (16 j + 8 (lane / 32) ..) of row rs * 64 + t * 32 + lane % 32.
template <int N> struct PieceVec;
template <> struct PieceVec<2> { typedef uint32_t type __attribute__((ext_vector_type(8))); };
template <> struct PieceVec<4> { typedef uint32_t type __attribute__((ext_vector_type(16))); };
template <> struct PieceVec<8> { typedef uint32_t type __attribute__((ext_vector_type(32))); };

template <int RS, int KS>
struct QStage {
  static constexpr bool kStatsViaLds = true;
  static constexpr bool kEmitViaLds = KS >= 4;                    // else every wavefront loads its own fragments (first layer of a launch)
  static constexpr int kRows = RS * 64;
  static constexpr int kPieces = kRows * 16 / (RS * KS * 64);     // 16 / KS
  static constexpr int kBytes = kRows * kLdsRow;
  static constexpr int kParts = kPieces > 4 ? kPieces / 4 : 1;    // steps over which the next layer's block is fetched
  static constexpr int kPartPieces = kPieces / kParts;
};

template <int RS, int KS>
__device__ inline typename PieceVec<QStage<RS, KS>::kPieces>::type load_q_pieces(const uint16_t* __restrict__ q_head,
                                                                                  int rows) {
  typename PieceVec<QStage<RS, KS>::kPieces>::type reg;
  uint32_t t = threadIdx.x;
  asm volatile("" : "+v"(t));   // the addresses are rebuilt here: kept across the caller's loop they cost registers
#pragma unroll
  for (int i = 0; i < QStage<RS, KS>::kPieces; ++i) {
    const uint32_t pc = t + i * (RS * KS * 64);                // piece pc of the block: row pc / 16, 16 bytes at pc * 16
    uint4 v = make_uint4(0, 0, 0, 0);
    if ((int)(pc >> 4) < rows) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(q_head) + pc * 16u);
    reg[4 * i] = v.x; reg[4 * i + 1] = v.y; reg[4 * i + 2] = v.z; reg[4 * i + 3] = v.w;
  }
  return reg;
}

template <int RS, int KS>
__device__ inline void store_q_pieces(char* __restrict__ qbuf, typename PieceVec<QStage<RS, KS>::kPieces>::type reg) {
#pragma unroll
  for (int i = 0; i < QStage<RS, KS>::kPieces; ++i) {
    const int pc = threadIdx.x + i * (RS * KS * 64);
    *reinterpret_cast<uint4*>(qbuf + (pc >> 4) * kLdsRow + (pc & 15) * 16) =
        make_uint4(reg[4 * i], reg[4 * i + 1], reg[4 * i + 2], reg[4 * i + 3]);
  }
}

// The same for one part of the block: pieces [part * kPartPieces, (part + 1) * kPartPieces) of every thread. The
// kernels fetch the next layer's Q in QStage::kParts steps, at most 4 pieces (16 registers) at a time.
template <int RS, int KS>
__device__ inline typename PieceVec<QStage<RS, KS>::kPartPieces>::type load_q_part(const uint16_t* __restrict__ q_head,
                                                                                    int rows, int part) {
  typename PieceVec<QStage<RS, KS>::kPartPieces>::type reg;
  uint32_t t = threadIdx.x;
  asm volatile("" : "+v"(t));
#pragma unroll
  for (int i = 0; i < QStage<RS, KS>::kPartPieces; ++i) {
    const uint32_t pc = t + (uint32_t)(part * QStage<RS, KS>::kPartPieces + i) * (RS * KS * 64);
    uint4 v = make_uint4(0, 0, 0, 0);
    if ((int)(pc >> 4) < rows) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(q_head) + pc * 16u);
    reg[4 * i] = v.x; reg[4 * i + 1] = v.y; reg[4 * i + 2] = v.z; reg[4 * i + 3] = v.w;
  }
  return reg;
}

template <int RS, int KS>
__device__ inline void store_q_part(char* __restrict__ qbuf, typename PieceVec<QStage<RS, KS>::kPartPieces>::type reg, int part) {
#pragma unroll
  for (int i = 0; i < QStage<RS, KS>::kPartPieces; ++i) {
    const int pc = threadIdx.x + (part * QStage<RS, KS>::kPartPieces + i) * (RS * KS * 64);
    *reinterpret_cast<uint4*>(qbuf + (pc >> 4) * kLdsRow + (pc & 15) * 16) =
        make_uint4(reg[4 * i], reg[4 * i + 1], reg[4 * i + 2], reg[4 * i + 3]);
  }
}

__device__ inline void read_q_frags(const char* __restrict__ qbuf, int rs, bf16x8 (&qf)[2][8]) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const char* row = qbuf + (rs * 64 + t * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
#pragma unroll
    for (int j = 0; j < 8; ++j) qf[t][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(row + j * 32));
  }
}

// The same fragments straight from global memory, every wavefront for itself: used by the emit kernel where only
// two wavefronts share a row slab (KS = 2), for which the detour through LDS measured slower there.
__device__ inline void load_q_frags(const uint16_t* __restrict__ q_head, int rs, int rows, bf16x8 (&qf)[2][8]) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int r = rs * 64 + t * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (r < rows) v = *reinterpret_cast<const uint4*>(q_head + (int64_t)r * 128 + j * 16 + (lane >> 5) * 8);
      qf[t][j] = __builtin_bit_cast(bf16x8, v);
    }
  }
}

// One tile of keys in flight between global memory and LDS: kPieces 16-byte pieces per thread, held as ONE
// vector value (a plain array would be demoted to scratch memory across the loop).

// Fetches one tile of keys [row0, row0 + kKeys) (relative to the chunk start, clamped to its last row, so every
// load stays inside the chunk and clamped rows are cache hits) into registers.
template <int RS, int KS>
__device__ inline typename PieceVec<Tile<RS, KS>::kPieces>::type load_tile(const char* __restrict__ k_chunk,
                                                                            uint32_t stride_token_b, int row0,
                                                                            int last_row) {
  typename PieceVec<Tile<RS, KS>::kPieces>::type reg;
#pragma unroll
  for (int i = 0; i < Tile<RS, KS>::kPieces; ++i) {
    const int p = threadIdx.x + i * Tile<RS, KS>::kThreads;
    int row = row0 + (p >> 4);
    row = row < last_row ? row : last_row;
    const uint32_t off = __umul24((uint32_t)row, stride_token_b) + (uint32_t)(p & 15) * 16u;
    const uint4 v = *reinterpret_cast<const uint4*>(k_chunk + off);
    reg[4 * i] = v.x; reg[4 * i + 1] = v.y; reg[4 * i + 2] = v.z; reg[4 * i + 3] = v.w;
  }
  return reg;
}

template <int RS, int KS>
__device__ inline void store_tile(char* __restrict__ buf, typename PieceVec<Tile<RS, KS>::kPieces>::type reg) {
#pragma unroll
  for (int i = 0; i < Tile<RS, KS>::kPieces; ++i) {
    const int p = threadIdx.x + i * Tile<RS, KS>::kThreads;
    *reinterpret_cast<uint4*>(buf + (p >> 4) * kLdsRow + (p & 15) * 16) =
        make_uint4(reg[4 * i], reg[4 * i + 1], reg[4 * i + 2], reg[4 * i + 3]);
  }
}

// The 8 K fragments (one per 16-wide slice of the head dimension) of the wavefront's 32 keys, read from an LDS
// tile in MFMA operand layout. Issued together so that the LDS latency is paid once per tile.
__device__ inline void read_k_frags(const char* __restrict__ tile, bf16x8 (&kf)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) kf[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + j * 32));
}

// Fragment j of them alone (the emit kernel, short of registers, reads one slice ahead instead of a whole tile
// at once).
__device__ inline bf16x8 read_k_frag(const char* __restrict__ tile, int j) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + j * 32));
}

// Slice j of the two accumulators: acc[t] (+)= (KEYS_AS_M ? K_tile . Q_t^T : Q_t . K_tile^T) over head dims 16j..16j+15.
template <bool KEYS_AS_M>
__device__ inline void mfma_slice(int j, const bf16x8 kfj, const bf16x8 (&qf)[2][8], floatx16 (&acc)[2]) {
  if (j == 0) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
  }
  if (KEYS_AS_M) {
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfj, qf[0][j], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfj, qf[1][j], acc[1], 0, 0, 0);
  } else {
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[0][j], kfj, acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[1][j], kfj, acc[1], 0, 0, 0);
  }
}

template <bool KEYS_AS_M>
__device__ inline void mfma_slice(int j, const bf16x8 (&kf)[8], const bf16x8 (&qf)[2][8], floatx16 (&acc)[2]) {
  if (j == 0) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
  }
  if (KEYS_AS_M) {
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[0][j], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[1][j], acc[1], 0, 0, 0);
  } else {
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[0][j], kf[j], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[1][j], kf[j], acc[1], 0, 0, 0);
  }
}

template <bool KEYS_AS_M>
__device__ inline void mfma_tile(const char* __restrict__ tile, const bf16x8 (&qf)[2][8], floatx16 (&acc)[2]) {
  bf16x8 kf[8];
  read_k_frags(tile, kf);
#pragma unroll
  for (int j = 0; j < 8; ++j) mfma_slice<KEYS_AS_M>(j, kf, qf, acc);
}

// lse2 of the four rows that accumulator registers 4 * (j & 3) .. + 3 of tile j / 4 hold (slice j of the emit
// kernel's exponentials): rows rs * 64 + t * 32 + 8 * (j & 3) + 4 * (lane / 32) + 0..3.
__device__ inline float4 rows_of_slice(const float* __restrict__ row_val, int rs, int j) {
  const int lane = threadIdx.x & 63;
  return *reinterpret_cast<const float4*>(&row_val[rs * 64 + (j >> 2) * 32 + 8 * (j & 3) + 4 * (lane >> 5)]);
}

// Linear chunk index -> (sequence, chunk) for chunks of `chunk` items over (length - window_off) items per
// sequence; also returns the number of chunks of (length) items in the earlier sequences (first_full) and in
// this one (n_full): the statistics kernel cuts all S keys, the emit kernel the S' prefix outputs.
// A single sequence spans [0, total_tokens) (cu_seqlens[0] = 0, cu_seqlens[1] = total_tokens): nothing is read.
// The host sizes the grid of the score kernels for `chunk` keys per workgroup from the token total alone (it does
// not see the lengths, so it allows every sequence a ragged tail): grid_x = total / chunk + n_seqs. With the lengths
// at hand a shorter chunk often fits the same grid, and the longest chunk sets the kernel's time: every kernel of a
// score call starts by finding the shortest multiple of the tile (down to half the host's chunk) whose chunks, over
// all sequences, still fit grid_x - the same value in every workgroup and kernel of the call.
constexpr int kFitMaxSeqs = 32;       // beyond that the search would cost more than it saves
__device__ inline int fitted_chunk(const int32_t* __restrict__ cu, int n_seqs, int chunk, int tile, int grid_x) {
  if (n_seqs == 1 || n_seqs > kFitMaxSeqs) return chunk;
  // lane t of every wavefront tries chunk - t * tile (at most chunk / (2 * tile) <= 32 candidates); fewer keys per
  // chunk mean more chunks, so the feasible candidates are the first ones
  const int c = chunk - (int)(threadIdx.x & 63) * tile;
  bool ok = c >= kMfmaMinChunk && 2 * c >= chunk;
  if (ok) {
    int n = 0, begin = cu[0];
    for (int s = 0; s < n_seqs; ++s) {
      const int end = cu[s + 1];
      n += (end - begin + c - 1) / c;
      begin = end;
    }
    ok = n <= grid_x;
  }
  const unsigned long long feasible = __ballot(ok) | 1ull;           // the host's own chunk always fits
  const int first_bad = ~feasible == 0ull ? 64 : __ffsll((long long)~feasible) - 1;
  return chunk - (first_bad - 1) * tile;
}

__device__ inline bool find_chunk2(const int32_t* __restrict__ cu, int n_seqs, int total_tokens, int chunk,
                                   int window_off, int b, int& seq, int& c, int& nc, int& seq_begin, int& seq_len,
                                   int& first_full, int& n_full) {
  if (n_seqs == 1) {
    int items = total_tokens - window_off;
    items = items > 0 ? items : 0;
    const int n = (items + chunk - 1) / chunk;
    seq = 0; c = b; nc = n; seq_begin = 0; seq_len = total_tokens; first_full = 0;
    n_full = (total_tokens + chunk - 1) / chunk;
    return b < n;
  }
  int begin = cu[0];
  int full = 0;
  for (int s = 0; s < n_seqs; ++s) {
    const int end = cu[s + 1];
    const int len = end - begin;
    const int nf = (len + chunk - 1) / chunk;
    int items = len - window_off;
    items = items > 0 ? items : 0;
    const int n = (items + chunk - 1) / chunk;
    if (b < n) {
      seq = s; c = b; nc = n; seq_begin = begin; seq_len = len; first_full = full; n_full = nf;
      return true;
    }
    b -= n;
    full += nf;
    begin = end;
  }
  return false;
}

// Workgroup barrier that orders LDS traffic only. __syncthreads() also waits for every global load the wavefront
// has in flight (its release fence covers global memory), which would cut the prefetch of the key tiles down to
// what fits between two barriers; the wavefronts of a score kernel talk to each other through LDS alone.
__device__ inline void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Q and K of the layers one launch covers (kernel argument, indexed by the layer's place in the launch).
struct ScoreLayers {
  const uint16_t* q[DKV_MAX_SELECT_LAYERS];
  const char* k[DKV_MAX_SELECT_LAYERS];
};

// The tile `ahead` steps after the start of layer `li` in the stream of n_steps tiles per layer: its layer and
// its step within that layer. Past the end of the call it is the last layer's last step again (loaded, not used).
__device__ inline void stream_tile(int li, int ahead, int n_steps, int n_layers, int& layer, int& step) {
  layer = li;
  step = ahead;
  while (step >= n_steps && layer + 1 < n_layers) {   // at most twice (ahead <= n_steps + 2, n_steps >= 2)
    step -= n_steps;
    ++layer;
  }
  if (step >= n_steps) step = n_steps - 1;
}

// ------------------------------------------------------------------------------------------------------
// Row statistics: one partial (max, sum of exp2) per layer, chunk and row, in the log2 domain:
// y = c * x with c = softmax_scale * log2(e); partial = (max y, sum exp2(y - max y)).
// grid = (chunk upper bound over all S keys, Hkv). A workgroup owns one chunk of one (sequence, KV head) and
// takes it through all n_layers layers of the launch: the geometry is the same for every layer, and while the
// last two steps of a layer run, the first two key tiles and the Q block of the next layer are already being
// fetched, so that only the first layer pays for a cold start.
// ------------------------------------------------------------------------------------------------------
template <int RS, int KS>
__global__ __launch_bounds__(RS * KS * 64) void score_stats_mfma(Params p, int chunk, int n_layers, ScoreLayers src,
                                                                 int64_t stride_token_b, int64_t stride_head_b,
                                                                 const int32_t* __restrict__ cu,
                                                                 float* __restrict__ partials,
                                                                 int64_t partials_stride_layer) {
  using TL = Tile<RS, KS>;
  using QS = QStage<RS, KS>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* tiles = smem;                                                          // 2 x kTileBytes
  char* qbuf = smem + 2 * TL::kTileBytes;                                      // Q staging
  float2* stat = reinterpret_cast<float2*>(smem + 2 * TL::kTileBytes + QS::kBytes);   // [KS][RS * 64]

  chunk = fitted_chunk(cu, p.n_seqs, chunk, TL::kKeys, gridDim.x);
  int seq, c, nc, begin, S, first_full, n_full;
  if (!find_chunk2(cu, p.n_seqs, p.total_tokens, chunk, 0, blockIdx.x, seq, c, nc, begin, S, first_full, n_full)) return;
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rs = wave % RS, ks = wave / RS;
  const int c0 = c * chunk;
  const int len = (c0 + chunk < S ? c0 + chunk : S) - c0;
  const int n_iter = (len + TL::kKeys - 1) / TL::kKeys;
  const int n_steps = n_iter > QS::kParts + 1 ? n_iter : QS::kParts + 1;   // the steps before a layer's last one fetch the next layer's Q
  const int prefix_rel = S - p.w - c0;              // first window key, relative to the chunk (may be <= 0)
  const float cexp = p.scale * kLog2e;
  const int64_t k_off = ((int64_t)begin + c0) * stride_token_b + (int64_t)head * stride_head_b;
  const int64_t q_off = ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w * 128;
  const uint32_t stride_b = (uint32_t)stride_token_b;
  int limit[2];                                     // last key (chunk-relative) visible to this lane's row
#pragma unroll
  for (int t = 0; t < 2; ++t) limit[t] = prefix_rel + (rs * 64 + t * 32 + (lane & 31)) % p.w;
  const int lane_tile = (ks * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
  const int lim_all = prefix_rel < len ? prefix_rel : len;

  // First layer: all first loads are issued together (one memory latency, not three). Tile loads stay in flight
  // for two steps (one step is shorter than the memory latency under load), so there are two register sets:
  // the set of tile u is ld[u & 1].
  typename PieceVec<TL::kPieces>::type ld[2];
  // the K pointer of the layer whose tiles are being fetched stays in scalar registers from step to step (reading it
  // from the kernel argument in every step makes every step begin with a wait)
  int k_layer;
  const char* k_ptr;
  {
    const typename PieceVec<TL::kPieces>::type reg0 = load_tile<RS, KS>(src.k[0] + k_off, stride_b, 0, len - 1);
    const typename PieceVec<QS::kPieces>::type q0 = load_q_pieces<RS, KS>(src.q[0] + q_off, p.rows);
    const typename PieceVec<TL::kPieces>::type reg1 = load_tile<RS, KS>(src.k[0] + k_off, stride_b, TL::kKeys, len - 1);
    int l2, t2;
    stream_tile(0, 2, n_steps, n_layers, l2, t2);
    ld[0] = load_tile<RS, KS>(src.k[l2] + k_off, stride_b, t2 * TL::kKeys, len - 1);   // stored by the first step
    k_layer = l2;
    k_ptr = src.k[l2] + k_off;
    store_tile<RS, KS>(tiles, reg0);
    store_q_pieces<RS, KS>(qbuf, q0);
    store_tile<RS, KS>(tiles + TL::kTileBytes, reg1);
  }
  lds_barrier();                                  // key tiles 0 and 1 and the Q block of the first layer are in LDS
  bf16x8 qf[2][8];
  read_q_frags(qbuf, rs, qf);
  floatx16 acc[2], nxt[2];
  mfma_tile<true>(tiles + lane_tile, qf, acc);
  lds_barrier();                                  // buffer 0 is rewritten by the first step

  // The key tiles of all layers form one stream: n_steps tiles per layer, layer after layer; tile v of the stream
  // lives in LDS buffer v & 1. One step: issue the loads of tile v + 3, MFMAs of tile v + 1 into `b`,
  // exponentials of tile v from `a`, tile v + 2 from registers to LDS. Tiles past the chunk are fully masked (they add exp2(-inf) = 0). The step
  // before a layer's last one fetches the next layer's Q block into LDS; the last step, which has nothing of its
  // own layer left to multiply, takes that Q as its operand for the next layer's tile 0, and is followed by the
  // layer's epilogue - so the matrix pipe, the vector ALU and the loads never pause between layers.
  int li = 0, it = 0;                               // layer of the call and step within it (uniform over the workgroup)
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};
  auto step = [&](auto buffer, floatx16 (&a)[2], floatx16 (&b)[2]) {
    constexpr int kBuf = decltype(buffer)::value;   // buffer of this step's tile
    if (li >= n_layers) return;                     // the padding step of an odd stream
    const bool has_next = li + 1 < n_layers;
    const int q_part = it + 1 + QS::kParts - n_steps;         // part of the next layer's Q block this step fetches
    const bool fetch_q = q_part >= 0 && q_part < QS::kParts && has_next;
    const bool last = it + 1 == n_steps;
    typename PieceVec<QS::kPartPieces>::type qnext;  // local: no value is carried from step to step
    // issued before the tile's loads, which stay in flight past the end of the step (loads return in order)
    if (fetch_q) qnext = load_q_part<RS, KS>(src.q[li + 1] + q_off, p.rows, q_part);
    int la, ta;                                     // tile v + 3: issued in this step, stored to LDS in the next one
    stream_tile(li, it + 3, n_steps, n_layers, la, ta);
    if (la != k_layer) {
      k_layer = la;
      k_ptr = src.k[la] + k_off;
    }
    const int wave_row0 = it * TL::kKeys + ks * 32;
    if (wave_row0 + 32 > lim_all) {                        // touches the window or runs past the chunk
      const int kb = wave_row0 + 4 * (lane >> 5);          // + 8 * (j / 4) + j % 4
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int s = kb + 8 * (j >> 2) + (j & 3);
          if (s > limit[t] || s >= len) a[t][j] = -INFINITY;
        }
    }
    float m_use[2], s0, s1, s2, s3;
    auto exps = [&](int j) {   // one eighth of the exponentials of this step's tile
      const int t = j >> 2, e = (j & 3) * 4;
      if ((j & 3) == 0) {      // row maximum of tile t, new running maximum
        float mx = fmaxf(a[t][0], a[t][1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(a[t][i], a[t][i + 1]));
        const float m_new = fmaxf(m_run[t], mx * cexp);
        m_use[t] = m_new == -INFINITY ? 0.0f : m_new;
        l_run[t] *= fast_exp2(m_run[t] - m_use[t]);
        m_run[t] = m_new;
        s0 = s1 = s2 = s3 = 0.0f;
      }
      s0 += fast_exp2(fmaf(a[t][e], cexp, -m_use[t]));
      s1 += fast_exp2(fmaf(a[t][e + 1], cexp, -m_use[t]));
      s2 += fast_exp2(fmaf(a[t][e + 2], cexp, -m_use[t]));
      s3 += fast_exp2(fmaf(a[t][e + 3], cexp, -m_use[t]));
      if ((j & 3) == 3) l_run[t] += (s0 + s1) + (s2 + s3);
    };
    // 8 slices: two MFMAs of the next tile each, interleaved with one eighth of the exponentials of this tile, so
    // that the matrix pipe and the vector ALU are busy together within one wavefront. After the last layer the
    // product of the last step is of stale operands and unused (cheaper than a second variant of the step).
    if (last) read_q_frags(qbuf, rs, qf);                  // the next layer's Q, stored before the previous barrier
    {
      const char* __restrict__ next_tile = tiles + (kBuf ^ 1) * TL::kTileBytes + lane_tile;
      bf16x8 kf[8];                                        // all eight at once: there are registers to spare here
      read_k_frags(next_tile, kf);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        __builtin_amdgcn_sched_barrier(0);
        // Half-way through the step the tile of step v + 2 goes from registers to LDS: its loads were issued a
        // step and a half ago, and the LDS writes complete under the rest of the step instead of in front of the
        // barrier. (This buffer held this step's tile, whose MFMAs ran before the previous barrier: it is free.)
        // the loads of tile v + 3 go out behind the LDS reads of this step's fragments (measured: 1 % faster than
        // in front of them, where both wavefronts of a SIMD do their address arithmetic before any MFMA can start)
        if (j == 0) ld[kBuf ^ 1] = load_tile<RS, KS>(k_ptr, stride_b, ta * TL::kKeys, len - 1);
        if (j == 4) store_tile<RS, KS>(tiles + kBuf * TL::kTileBytes, ld[kBuf]);
        mfma_slice<true>(j, kf[j], qf, b);
        exps(j);
        // the sums are pinned here: without an anchor the compiler sinks the exponentials of all eight slices past
        // the matrix instructions (the scheduling barrier alone only holds what is already in its region)
        asm volatile("" : "+v"(s0), "+v"(s1), "+v"(s2), "+v"(s3), "+v"(l_run[0]), "+v"(l_run[1]));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (fetch_q) store_q_part<RS, KS>(qbuf, qnext, q_part);   // every wavefront has this layer's Q in registers
    lds_barrier();
    if (!last) {
      ++it;
      return;
    }
    // ---- end of a layer: merge the two half-wavefronts (same row, other keys), then the KS key tiles, publish
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const float m2 = __shfl_xor(m_run[t], 32), l2 = __shfl_xor(l_run[t], 32);
      const float M = fmaxf(m_run[t], m2);
      const float Mu = M == -INFINITY ? 0.0f : M;
      const float Lsum = fmaf(l_run[t], fast_exp2(m_run[t] - Mu), l2 * fast_exp2(m2 - Mu));   // spelled out: both copies of this code round alike
      if (lane < 32) stat[ks * (RS * 64) + rs * 64 + t * 32 + lane] = make_float2(M, Lsum);
      m_run[t] = -INFINITY;
      l_run[t] = 0.0f;
    }
    lds_barrier();
    float2* __restrict__ part = reinterpret_cast<float2*>(partials + li * partials_stride_layer) +
                                (((int64_t)blockIdx.x) * p.Hkv + head) * p.rows_pad;
    if (tid < RS * 64) {                            // no loop around memory instructions: key tiles are in flight
      const int r = tid;
      float M = -INFINITY;
#pragma unroll
      for (int q = 0; q < KS; ++q) M = fmaxf(M, stat[q * (RS * 64) + r].x);
      const float Mu = M == -INFINITY ? 0.0f : M;
      float Lsum = 0.0f;
#pragma unroll
      for (int q = 0; q < KS; ++q) {
        const float2 v = stat[q * (RS * 64) + r];
        Lsum = fmaf(v.y, fast_exp2(v.x - Mu), Lsum);
      }
      part[r] = make_float2(M, Lsum);
    }
    ++li;
    it = 0;
  };
  while (li < n_layers) {                           // the steps alternate between the two accumulator sets
    step(std::integral_constant<int, 0>{}, acc, nxt);
    step(std::integral_constant<int, 1>{}, nxt, acc);
  }
}

// ------------------------------------------------------------------------------------------------------
// Scores: a[s] = row_scale * sum_rows exp2(c * x[row, s] - lse2[row]) over the chunk's outputs plus the pooling
// halo, max-pooled over the prefix. grid = (chunk upper bound over the S' prefix outputs, Hkv).
// ------------------------------------------------------------------------------------------------------
// Column sums of one row slab in the emit kernel: the chunk's outputs, the pooling halo and two tiles of slack
// (the last step computes a tile past the range).
template <int RS, int KS>
__host__ __device__ inline int emit_part_stride(int chunk) { return chunk + kMaxHalo + 2 * Tile<RS, KS>::kKeys; }

// Slabs of that size in LDS: one per row slab, and at least two (the second also holds the pooled outputs).
template <int RS>
__host__ __device__ constexpr int emit_slabs() { return RS > 1 ? RS : 2; }

// Key tile that step `it` of the emit kernel works on (steps past the first tile repeat it: same values again).
__device__ inline int emit_tile(int n_iter, int it) { return it < n_iter ? n_iter - 1 - it : 0; }

// ---- Row normalisers lse2[row] = log2 sum_keys exp2(c * x[row, key]) from the chunk partials of the statistics
// kernel, by the RS * KS * 64 threads of a workgroup: thread (row mrow, group mgrp) merges the chunks mgrp,
// mgrp + KS, ... online in chunk order into `mstage`; after a barrier thread `row` combines the KS groups.
// Written once and used both inside the emit kernel (single-layer launches) and by the merge kernel below, so
// that both give the same bits.
__device__ inline void merge_pair(float& M, float& Lsum, const float2 v) {
  const float Mn = fmaxf(M, v.x);
  const float Mu = Mn == -INFINITY ? 0.0f : Mn;
  Lsum = fmaf(Lsum, fast_exp2(M - Mu), v.y * fast_exp2(v.x - Mu));   // spelled out: every call site rounds alike
  M = Mn;
}

// psrc: partials of chunk 0 of this (layer, sequence, head), float2 [chunk][Hkv][rows_pad]
template <int RS, int KS>
__device__ inline void merge_chunks(const float2* __restrict__ psrc, int n_full, uint32_t chunk_step, float2* __restrict__ mstage) {
  constexpr int kRows = RS * 64;
  const int mrow = threadIdx.x % kRows, mgrp = threadIdx.x / kRows;
  const uint32_t t0 = (uint32_t)mrow + (uint32_t)mgrp * chunk_step;   // 32-bit element offsets from a shared base
  float M = -INFINITY, Lsum = 0.0f;
#pragma unroll 8
  for (int cc = mgrp; cc < n_full; cc += KS, psrc += KS * chunk_step) merge_pair(M, Lsum, psrc[t0]);
  mstage[mgrp * kRows + mrow] = make_float2(M, Lsum);
}

// lse2 of row `row` (< RS * 64) from the KS staged merges; padding rows get +inf: exp2(x - inf) = 0
template <int RS, int KS>
__device__ inline float combine_groups(const float2* __restrict__ mstage, int row, int rows) {
  constexpr int kRows = RS * 64;
  float Mx = -INFINITY;
#pragma unroll
  for (int g = 0; g < KS; ++g) Mx = fmaxf(Mx, mstage[g * kRows + row].x);
  const float Mu = Mx == -INFINITY ? 0.0f : Mx;
  float L = 0.0f;
#pragma unroll
  for (int g = 0; g < KS; ++g) {
    const float2 v = mstage[g * kRows + row];
    L = fmaf(v.y, fast_exp2(v.x - Mu), L);
  }
  return row < rows ? Mx + __log2f(L) : INFINITY;
}

// Merge kernel of multi-layer launches: lse_rows[layer][seq][head][rows_pad] (log2 domain), between the two
// sweeps. grid = (n_seqs, Hkv, n_layers), RS * KS * 64 threads. Inside the emit kernel this merge would sit on
// the critical path of every layer (a chain of dependent loads per thread, 32 deep for 64 chunks).
template <int RS, int KS>
__global__ __launch_bounds__(RS * KS * 64) void score_merge_mfma(Params p, int chunk, int grid_x,
                                                                 const int32_t* __restrict__ cu,
                                                                 const float* __restrict__ partials,
                                                                 int64_t partials_stride_layer,
                                                                 float* __restrict__ lse_rows) {
  constexpr int kRows = RS * 64;
  __shared__ float2 mstage[KS * kRows];
  const int seq = blockIdx.x, head = blockIdx.y, layer = blockIdx.z;
  chunk = fitted_chunk(cu, p.n_seqs, chunk, Tile<RS, KS>::kKeys, grid_x);      // as the statistics kernel cut the keys
  int first_full = 0;
  for (int q = 0; q < seq; ++q) first_full += (cu[q + 1] - cu[q] + chunk - 1) / chunk;
  const int n_full = (cu[seq + 1] - cu[seq] + chunk - 1) / chunk;
  const float2* __restrict__ psrc = reinterpret_cast<const float2*>(partials + layer * partials_stride_layer) +
                                    ((int64_t)first_full * p.Hkv + head) * p.rows_pad;
  merge_chunks<RS, KS>(psrc, n_full, (uint32_t)(p.Hkv * p.rows_pad), mstage);
  __syncthreads();
  if (threadIdx.x < kRows)
    lse_rows[(((int64_t)layer * p.n_seqs + seq) * p.Hkv + head) * p.rows_pad + threadIdx.x] =
        combine_groups<RS, KS>(mstage, threadIdx.x, p.rows);
}

// Row normalisers supplied by the caller for every layer of a multi-layer call (natural log, [n_seqs][Hq][w] per
// layer) into the layout and the log2 domain the emit kernel reads. grid = (n_seqs, Hkv, n_layers), 256 threads.
struct LseLayers {
  const float* lse[DKV_MAX_SELECT_LAYERS];
};

__global__ __launch_bounds__(256) void score_import_lse(Params p, LseLayers src, float* __restrict__ lse_rows) {
  const int seq = blockIdx.x, head = blockIdx.y, layer = blockIdx.z;
  const float* __restrict__ in = src.lse[layer] + ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w;
  float* __restrict__ out = lse_rows + (((int64_t)layer * p.n_seqs + seq) * p.Hkv + head) * p.rows_pad;
  for (int r = threadIdx.x; r < p.rows_pad; r += 256)   // padding rows get +inf: exp2(x - inf) = 0
    out[r] = r < p.rows ? in[r] * kLog2e : INFINITY;
}

// Outputs per thread of the emit kernel's epilogue (the chunk is at most kMaxChunk outputs).
constexpr int kMaxChunk = 4096;

// As in the statistics kernel, a workgroup takes its chunk through all n_layers layers of the launch: the key tiles
// form one stream, the next layer's Q block and row normalisers are fetched while the current layer's last steps
// run. The row normalisers come from lse_rows (multi-layer launches, written by the merge kernel), from lse_in
// (supplied by the caller, natural log, single-layer launches) or are merged here from the chunk partials
// (single-layer launches).
template <int RS, int KS>
__global__ __launch_bounds__(RS * KS * 64) void score_emit_mfma(Params p, int chunk, int n_layers, ScoreLayers src,
                                                                int64_t stride_token_b, int64_t stride_head_b,
                                                                const int32_t* __restrict__ cu,
                                                                const float* __restrict__ partials,
                                                                const float* __restrict__ lse_rows,
                                                                int64_t lse_rows_stride_layer,
                                                                const float* __restrict__ lse_in,
                                                                float* __restrict__ scores, int64_t scores_stride_head,
                                                                int64_t scores_stride_layer, float* __restrict__ edges,
                                                                int64_t edges_stride_layer) {
  using TL = Tile<RS, KS>;
  using QS = QStage<RS, KS>;
  chunk = fitted_chunk(cu, p.n_seqs, chunk, TL::kKeys, gridDim.x);             // not longer than the host's: the LDS fits
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* tiles = smem;                                                          // 2 x kTileBytes
  float* part = reinterpret_cast<float*>(smem + 2 * TL::kTileBytes);           // [emit_slabs][kPartStride]
  const int kPartStride = emit_part_stride<RS, KS>(chunk);
  constexpr int kRows = RS * 64;
  char* qbuf = smem + 2 * TL::kTileBytes + emit_slabs<RS>() * kPartStride * sizeof(float);   // Q staging
  __shared__ float2 mstage[KS * kRows];                                        // partial merges of KS thread groups
  __shared__ __attribute__((aligned(16))) float lse_s[2][kRows];               // lse2 per row, by layer parity

  const int half = p.half;
  int seq, c, nc, begin, S, first_full, n_full;
  if (!find_chunk2(cu, p.n_seqs, p.total_tokens, chunk, p.w, blockIdx.x, seq, c, nc, begin, S, first_full, n_full)) return;
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rs = wave % RS, ks = wave / RS;
  const int prefix = S - p.w;                                // > 0 here
  const int o0 = c * chunk;                                  // outputs [o0, o1)
  const int o1 = o0 + chunk < prefix ? o0 + chunk : prefix;
  // keys [kbeg, kend): the outputs plus the pooling halo, inside the prefix - or, with `edges`, the outputs alone:
  // then the pooled values next to a chunk border lack the neighbour's keys, the column sums of the first and the
  // last `half` keys go to `edges`, and score_fix_borders completes those outputs afterwards
  const int halo = edges != nullptr ? 0 : half;
  const int kbeg = o0 - halo > 0 ? o0 - halo : 0;
  const int kend = o1 + halo < prefix ? o1 + halo : prefix;
  const int len = kend - kbeg;                               // <= chunk + 2 * half
  const int n_iter = (len + TL::kKeys - 1) / TL::kKeys;
  const int n_steps = n_iter > QS::kParts + 1 ? n_iter : QS::kParts + 1;   // the steps before a layer's last one fetch the next layer's Q
  const float cexp = p.scale * kLog2e;
  const int64_t k_off = ((int64_t)begin + kbeg) * stride_token_b + (int64_t)head * stride_head_b;
  const int64_t q_off = ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w * 128;
  const uint32_t stride_b = (uint32_t)stride_token_b;
  const int lane_tile = (ks * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
  // lse2 of row tid of this (sequence, head) in lse_rows, per layer of the launch
  const float* __restrict__ lse_row = lse_rows + ((int64_t)seq * p.Hkv + head) * p.rows_pad + (tid < kRows ? tid : 0);

  // Tiles are taken from the last to the first: the statistics kernel, which ran first to last over the same
  // chunks on the same compute units, left its last tiles as the most recently used lines.
  // First layer: all first loads are issued together (one memory latency, not three). Tile loads stay in flight
  // for two steps (one step is shorter than the memory latency under load), so there are two register sets:
  // the set of the tile of step u is ld[u & 1].
  typename PieceVec<TL::kPieces>::type ld[2];
  bf16x8 qf[2][8];
  int k_layer;                    // layer and K pointer of the tiles being fetched (see the statistics kernel)
  const char* k_ptr;
  {
    const typename PieceVec<TL::kPieces>::type reg0 = load_tile<RS, KS>(src.k[0] + k_off, stride_b, emit_tile(n_iter, 0) * TL::kKeys, len - 1);
    typename PieceVec<QS::kPieces>::type q0;
    if (QS::kEmitViaLds) q0 = load_q_pieces<RS, KS>(src.q[0] + q_off, p.rows);
    else load_q_frags(src.q[0] + q_off, rs, p.rows, qf);
    const typename PieceVec<TL::kPieces>::type reg1 = load_tile<RS, KS>(src.k[0] + k_off, stride_b, emit_tile(n_iter, 1) * TL::kKeys, len - 1);
    int l2, t2;
    stream_tile(0, 2, n_steps, n_layers, l2, t2);
    ld[0] = load_tile<RS, KS>(src.k[l2] + k_off, stride_b, emit_tile(n_iter, t2) * TL::kKeys, len - 1);   // stored by the first step
    k_layer = l2;
    k_ptr = src.k[l2] + k_off;
    store_tile<RS, KS>(tiles, reg0);
    if (QS::kEmitViaLds) store_q_pieces<RS, KS>(qbuf, q0);
    store_tile<RS, KS>(tiles + TL::kTileBytes, reg1);
  }
  // ---- lse2[row] of the first layer
  if (lse_rows != nullptr) {
    if (tid < kRows) lse_s[0][tid] = lse_row[0];
  } else if (lse_in != nullptr) {
    if (tid < kRows)   // padding rows get +inf: exp2(x - inf) = 0
      lse_s[0][tid] = tid < p.rows ? lse_in[((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w + tid] * kLog2e : INFINITY;
  } else {
    merge_chunks<RS, KS>(reinterpret_cast<const float2*>(partials) + ((int64_t)first_full * p.Hkv + head) * p.rows_pad, n_full,
                         (uint32_t)(p.Hkv * p.rows_pad), mstage);
    lds_barrier();
    if (tid < kRows) lse_s[0][tid] = combine_groups<RS, KS>(mstage, tid, p.rows);
  }
  floatx16 acc[2], nxt[2];
  lds_barrier();                                             // lse2 is complete, the first tile and Q are in place
  if (QS::kEmitViaLds) read_q_frags(qbuf, rs, qf);
  mfma_tile<false>(tiles + lane_tile, qf, acc);
  lds_barrier();                                             // buffer 0 is rewritten by the first step

  // The key tiles of all layers form one stream: n_steps tiles per layer, layer after layer; tile v of the stream
  // lives in LDS buffer v & 1. One step: issue the loads of tile v + 3, MFMAs of tile v + 1 into `b`, exponentials
  // and column sums of tile v from `a`, tile v + 2 from registers to LDS. The step before a layer's last one
  // fetches the next layer's Q block into LDS; the last step, which has nothing of its own layer left to multiply,
  // takes that Q as its operand for the next layer's first tile, fetches the next layer's lse2, and is followed
  // by the layer's epilogue. Loads that a step consumes itself are issued before the tile's, which stay in flight
  // past the end of the step (loads return in order). Prefix keys are visible to every window row: no mask;
  // columns past the computed range are discarded in the epilogue. Fixed summation order per column.
  int li = 0, it = 0;                                          // layer of the call and step within it (uniform over the workgroup)
  auto step = [&](auto buffer, floatx16 (&a)[2], floatx16 (&b)[2]) {
    constexpr int kBuf = decltype(buffer)::value;              // buffer of this step's tile
    if (li >= n_layers) return;                                // the padding step of an odd stream
    const bool has_next = li + 1 < n_layers;
    const int q_part = it + 1 + QS::kParts - n_steps;          // part of the next layer's Q block this step fetches
    const bool fetch_q = q_part >= 0 && q_part < QS::kParts && has_next;
    const bool last = it + 1 == n_steps;
    const bool fetch_lse = last && has_next && tid < kRows;    // multi-layer launches come with lse_rows
    typename PieceVec<QS::kPartPieces>::type qnext;            // local: no value is carried from step to step
    float lse_next;
    if (fetch_q) qnext = load_q_part<RS, KS>(src.q[li + 1] + q_off, p.rows, q_part);
    if (fetch_lse) lse_next = lse_row[(li + 1) * lse_rows_stride_layer];
    int la, ta;                                                // tile v + 3: issued in this step, stored to LDS in the next one
    stream_tile(li, it + 3, n_steps, n_layers, la, ta);
    if (la != k_layer) {
      k_layer = la;
      k_ptr = src.k[la] + k_off;
    }
    const float* __restrict__ lse_cur = lse_s[li & 1];
    const int wave_row0 = emit_tile(n_iter, it) * TL::kKeys + ks * 32;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    // one eighth of the exponentials of this step's tile; lz = lse2 of its four rows, read from LDS one slice
    // ahead (the per-row constants of all 32 accumulator registers would not fit beside the rest)
    auto exps = [&](int j, const float4 lz) {
      const int t = j >> 2, e = (j & 3) * 4;
      s0 += fast_exp2(fmaf(a[t][e], cexp, -lz.x));
      s1 += fast_exp2(fmaf(a[t][e + 1], cexp, -lz.y));
      s2 += fast_exp2(fmaf(a[t][e + 2], cexp, -lz.z));
      s3 += fast_exp2(fmaf(a[t][e + 3], cexp, -lz.w));
    };
    float4 lz = rows_of_slice(lse_cur, rs, 0);
    // After the last layer the product of the last step is of stale operands and unused (cheaper than a second
    // variant of the step).
    if (last) read_q_frags(qbuf, rs, qf);                      // the next layer's Q, stored before the previous barrier
    {
      const char* __restrict__ next_tile = tiles + (kBuf ^ 1) * TL::kTileBytes + lane_tile;
      bf16x8 kfj = read_k_frag(next_tile, 0);
      // a wavefront whose 32 keys of this tile all lie past the computed range (the ragged tile of the pooling
      // halo) has no exponentials to take: its column sums are never read
      const bool live = wave_row0 < len;
#pragma unroll
      for (int j = 0; j < 8; ++j) {   // two MFMAs of the next tile, then one eighth of the exponentials of this one
        __builtin_amdgcn_sched_barrier(0);
        const float4 lz_next = rows_of_slice(lse_cur, rs, (j + 1) & 7);
        const bf16x8 kf_ahead = read_k_frag(next_tile, (j + 1) & 7);
        if (j == 0) ld[kBuf ^ 1] = load_tile<RS, KS>(k_ptr, stride_b, emit_tile(n_iter, ta) * TL::kKeys, len - 1);
        if (j == 2) store_tile<RS, KS>(tiles + kBuf * TL::kTileBytes, ld[kBuf]);   // the tile of step v + 2 (see the statistics kernel; measured best here)
        mfma_slice<false>(j, kfj, qf, b);
        if (live) exps(j, lz);
        // pinned here (see the statistics kernel)
        asm volatile("" : "+v"(s0), "+v"(s1), "+v"(s2), "+v"(s3));
        lz = lz_next;
        kfj = kf_ahead;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    float col = (s0 + s1) + (s2 + s3);
    {
      // the other half-wavefront holds the same keys and the other rows: v_permlane32_swap hands every lane the
      // lower half's value ([0]) and the upper half's ([1]) without a trip through the LDS crossbar
      const auto halves = __builtin_amdgcn_permlane32_swap(__float_as_uint(col), __float_as_uint(col), false, false);
      col = __uint_as_float(halves[0]) + __uint_as_float(halves[1]);   // rows 0-3 mod 8 first
    }
    if (lane < 32) part[rs * kPartStride + wave_row0 + lane] = col;
    if (fetch_q) store_q_part<RS, KS>(qbuf, qnext, q_part);    // every wavefront has this layer's Q in registers
    if (fetch_lse) lse_s[(li + 1) & 1][tid] = lse_next;
    lds_barrier();
    if (!last) {
      ++it;
      return;
    }
    // ---- end of a layer (no loops around memory instructions here: the key tiles of the next layer are in
    // flight). Sum the row slabs in a fixed order; positions past the computed range are ignored by the pooling.
    for (int i = tid; i < n_iter * TL::kKeys; i += TL::kThreads) {
      float x = part[i];
#pragma unroll
      for (int q = 1; q < RS; ++q) x += part[q * kPartStride + i];
      part[i] = i < len ? x * p.row_scale : -INFINITY;
    }
    lds_barrier();
    // max-pool into the second slab (its column sums are summed up by now; every thread reads back only what it
    // wrote itself), window [i - half, i + half] cut to [0, len): an index clamped to the range stays inside the
    // window, and taking an element twice does not change a maximum
    float* __restrict__ pooled = part + kPartStride;
    if (edges != nullptr && tid < 2 * half) {                  // [0, half): the first column sums, [half, 2 half): the last
      const int i = tid < half ? tid : len - 2 * half + tid;
      edges[li * edges_stride_layer + ((int64_t)blockIdx.x * p.Hkv + head) * kMaxHalo + tid] =
          i >= 0 && i < len ? part[i] : -INFINITY;
    }
    for (int s = o0 + tid; s < o1; s += TL::kThreads) {
      const int i = s - kbeg;
      float m = part[i];
      for (int o = 1; o <= half; ++o) {
        const float lo = part[i - o > 0 ? i - o : 0], hi = part[i + o < len ? i + o : len - 1];
        m = fmaxf(m, fmaxf(lo, hi));
      }
      pooled[s - o0] = m;
    }
    float* __restrict__ out = scores + li * scores_stride_layer + (int64_t)head * scores_stride_head + begin;
#pragma unroll
    for (int u = 0; u < kMaxChunk / TL::kThreads; ++u) {      // straight-line stores
      const int s = o0 + tid + u * TL::kThreads;
      if (s < o1) out[s] = pooled[s - o0];
    }
    if (c == nc - 1 && tid < p.w) out[prefix + tid] = -INFINITY;   // guard over the window slots (w <= 256 <= threads)
    if (has_next) lds_barrier();                               // `part` is reused by the next layer
    ++li;
    it = 0;
  };
  while (li < n_layers) {                                      // the steps alternate between the two accumulator sets
    step(std::integral_constant<int, 0>{}, acc, nxt);
    step(std::integral_constant<int, 1>{}, nxt, acc);
  }
}

// Completes the outputs next to the chunk borders of an emit launch that left the pooling halo out: output s of
// chunk c within `half` of the border to chunk c + 1 takes the maximum with the neighbour's column sums that its
// pooling window reaches (a maximum is exact, so the result is the one the halo variant computes).
// grid = (chunk upper bound, Hkv, layers), 64 threads: one workgroup per border, thread t < half the output
// half - t before it, thread half + u the output u after it.
__global__ __launch_bounds__(64) void score_fix_borders(Params p, int chunk, int tile, const int32_t* __restrict__ cu,
                                                        const float* __restrict__ edges, int64_t edges_stride_layer,
                                                        float* __restrict__ scores, int64_t scores_stride_head,
                                                        int64_t scores_stride_layer) {
  chunk = fitted_chunk(cu, p.n_seqs, chunk, tile, gridDim.x);  // as the emit kernel cut the outputs
  int seq, c, nc, begin, S, first_full, n_full;
  if (!find_chunk2(cu, p.n_seqs, p.total_tokens, chunk, p.w, blockIdx.x, seq, c, nc, begin, S, first_full, n_full)) return;
  if (c == nc - 1) return;                                     // no chunk behind the last one
  const int head = blockIdx.y, layer = blockIdx.z, half = p.half, t = threadIdx.x;
  if (t >= 2 * half) return;
  const int prefix = S - p.w;
  const int o1 = (c + 1) * chunk;                              // first output of the next chunk (< prefix)
  const int next_len = o1 + chunk < prefix ? chunk : prefix - o1;
  const float* __restrict__ mine = edges + layer * edges_stride_layer + ((int64_t)blockIdx.x * p.Hkv + head) * kMaxHalo + half;
  const float* __restrict__ next = edges + layer * edges_stride_layer + ((int64_t)(blockIdx.x + 1) * p.Hkv + head) * kMaxHalo;
  float* __restrict__ out = scores + layer * scores_stride_layer + (int64_t)head * scores_stride_head + begin;
  float m = -INFINITY;
  int s;
  if (t < half) {            // output o1 - half + t: its window ends at o1 + t, the next chunk's first t + 1 keys
    s = o1 - half + t;
    for (int e = 0; e <= t; ++e) m = fmaxf(m, next[e]);        // -inf past the end of a short last chunk
  } else {                   // output o1 + u: its window starts at o1 + u - half, this chunk's last half - u keys
    const int u = t - half;
    if (u >= next_len) return;
    s = o1 + u;
    for (int e = u; e < half; ++e) m = fmaxf(m, mine[e]);
  }
  out[s] = fmaxf(out[s], m);
}

// Natural-log row normalisers from the chunk partials of the statistics kernel (log2 domain):
// lse_out[(seq * Hq + head * G) * w + r]. grid = (n_seqs, Hkv), 256 threads.
__global__ __launch_bounds__(256) void score_lse_mfma(Params p, int chunk, int tile, int grid_x,
                                                      const int32_t* __restrict__ cu,
                                                      const float* __restrict__ partials, float* __restrict__ lse_out) {
  const int seq = blockIdx.x, head = blockIdx.y;
  chunk = fitted_chunk(cu, p.n_seqs, chunk, tile, grid_x);     // as the statistics kernel cut the keys
  int first_full = 0;
  for (int q = 0; q < seq; ++q) first_full += (cu[q + 1] - cu[q] + chunk - 1) / chunk;
  const int n_full = (cu[seq + 1] - cu[seq] + chunk - 1) / chunk;
  for (int r = threadIdx.x; r < p.rows; r += 256) {
    const float2* __restrict__ src =
        reinterpret_cast<const float2*>(partials) + ((int64_t)first_full * p.Hkv + head) * p.rows_pad + r;
    float M = -INFINITY, Lsum = 0.0f;
    for (int cc = 0; cc < n_full; ++cc) {
      const float2 v = src[(int64_t)cc * p.Hkv * p.rows_pad];
      const float Mn = fmaxf(M, v.x);
      const float Mu = Mn == -INFINITY ? 0.0f : Mn;
      Lsum = Lsum * fast_exp2(M - Mu) + v.y * fast_exp2(v.x - Mu);
      M = Mn;
    }
    lse_out[((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w + r] = (M + __log2f(Lsum)) * (1.0f / kLog2e);
  }
}

// load_tile() forms the byte offset of a key row inside a chunk in 32 bits (a 24-bit multiply): the largest row
// index it can see (the chunk, the pooling halo and two tiles of slack) times the token stride must stay below
// 2^32, and the stride itself below 2^24. Longer strides take the vector-ALU kernels.
bool score_mfma_supported(const Params& p, int dtype, int64_t k_stride_token) {
  const int64_t stride_b = k_stride_token * 2;
  const int64_t max_row = kMaxChunk + kMaxHalo + 2 * 128;
  return dtype == DKV_BF16 && p.d == 128 && p.rows <= 256 && 2 * p.half <= kMaxHalo && stride_b < (1 << 24) &&
         max_row * stride_b < ((int64_t)1 << 32);
}

// Keys per workgroup. Every workgroup pays a fixed cost (locating its chunk, the first loads, the epilogue) and the
// device holds one workgroup per compute unit, so the chunk is the multiple of the tile that minimises
// rounds x (fixed + streaming): as few rounds of workgroups as possible, and within that the shortest chunk.
// The number of chunks is exact for one sequence and an upper bound (one ragged tail per sequence) otherwise.
template <int RS, int KS>
static int pick_chunk(const Params& p, int cus) {
  using TL = Tile<RS, KS>;
  const long long lds_fixed = 2LL * TL::kTileBytes + QStage<RS, KS>::kBytes;
  int max_chunk = (int)((kLdsBudget - lds_fixed) / (emit_slabs<RS>() * (long long)sizeof(float))) - kMaxHalo - 2 * TL::kKeys;
  max_chunk = max_chunk / TL::kKeys * TL::kKeys;
  if (max_chunk > kMaxChunk) max_chunk = kMaxChunk;
  const double fixed_us = 6.0, us_per_key = 0.0102;          // measured: 1.3 us per 128-key step of a full device
  int best = 256;
  double best_cost = 1e30;
  for (int chunk = 256; chunk <= max_chunk; chunk += TL::kKeys) {
    if (chunk % TL::kKeys) continue;
    const long long chunks = p.n_seqs == 1 ? (p.total_tokens + chunk - 1) / chunk : p.total_tokens / chunk + p.n_seqs;
    const long long rounds = (chunks * p.Hkv + cus - 1) / cus;
    const double cost = rounds * (fixed_us + chunk * us_per_key);
    if (cost < best_cost - 1e-9) { best_cost = cost; best = chunk; }
  }
  return best;
}

static int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0)
      cus = 256;
  }
  return cus;
}

template <int RS, int KS>
static hipError_t launch_mfma_t(const Params& p, int phases, int n_layers, const void* const* q_layers,
                                const void* const* k_layers, int64_t k_stride_token, int64_t k_stride_head,
                                const int32_t* cu, float* scores, int64_t scores_stride_head,
                                int64_t scores_stride_layer, char* ws, const WorkspaceLayout& wl, const float* lse_in,
                                const float* const* lse_layers,
                                float* lse_out, hipStream_t st) {
  using TL = Tile<RS, KS>;
  const int chunk = pick_chunk<RS, KS>(p, device_cus());
  float* partials = ws ? reinterpret_cast<float*>(ws + wl.partials) : nullptr;   // no workspace: lse supplied
  const int64_t partials_stride_layer = (int64_t)wl.partials_layer_bytes / (int64_t)sizeof(float);
  const size_t stat_bytes = (size_t)KS * RS * 64 * sizeof(float2);               // the final [KS][RS * 64] partials
  const size_t lds_stats = 2 * TL::kTileBytes + (size_t)QStage<RS, KS>::kBytes + stat_bytes;
  const size_t lds_emit = 2 * TL::kTileBytes + (size_t)emit_slabs<RS>() * emit_part_stride<RS, KS>(chunk) * sizeof(float) +
                          (size_t)QStage<RS, KS>::kBytes;   // the Q staging area serves the next layer in every variant
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_stats_mfma<RS, KS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_stats);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_emit_mfma<RS, KS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  ScoreLayers src{};
  for (int i = 0; i < n_layers && (phases & (kPhaseStats | kPhaseEmit)); ++i) {
    src.q[i] = static_cast<const uint16_t*>(q_layers[i]);
    src.k[i] = static_cast<const char*>(k_layers[i]);
  }
  const int grid_x = p.total_tokens / chunk + p.n_seqs;      // upper bound on chunks over all sequences
  if (phases & kPhaseStats)
    launch(DKV_KERNEL_SCORE_STATS, (score_stats_mfma<RS, KS>), dim3(grid_x, p.Hkv), dim3(TL::kThreads), lds_stats, st, p, chunk,
           n_layers, src, k_stride_token * 2, k_stride_head * 2, cu, partials, partials_stride_layer);
  if (phases & kPhaseEmit) {
    // The emit kernel takes the layers of the call from the last to the first: the statistics kernel has just
    // streamed them first to last, so the last layers are the ones the memory-side cache still holds.
    ScoreLayers rev{};
    for (int i = 0; i < n_layers; ++i) {
      rev.q[i] = src.q[n_layers - 1 - i];
      rev.k[i] = src.k[n_layers - 1 - i];
    }
    const int last = n_layers - 1;
    // several layers: their row normalisers are merged from the chunk partials by a small kernel of its own
    float* lse_rows = nullptr;
    const int64_t lse_rows_stride_layer = (int64_t)p.n_seqs * p.Hkv * p.rows_pad;
    if (n_layers > 1) {
      lse_rows = reinterpret_cast<float*>(ws + wl.lse_rows);
      if (lse_layers != nullptr) {       // single sweep: the caller's normalisers, no statistics
        LseLayers in{};
        for (int i = 0; i < n_layers; ++i) in.lse[i] = lse_layers[i];
        launch(DKV_KERNEL_SCORE_MERGE, score_import_lse, dim3(p.n_seqs, p.Hkv, n_layers), dim3(256), 0, st, p, in, lse_rows);
      } else {
        launch(DKV_KERNEL_SCORE_MERGE, (score_merge_mfma<RS, KS>), dim3(p.n_seqs, p.Hkv, n_layers), dim3(TL::kThreads), 0, st,
               p, chunk, grid_x, cu, static_cast<const float*>(partials), partials_stride_layer, lse_rows);
      }
    } else if (lse_layers != nullptr) {
      lse_in = lse_layers[0];
    }
    // A call over several layers leaves the pooling halo to a small kernel behind the emit kernel (one launch for
    // all layers); a single layer recomputes the halo keys inside the emit kernel, which is cheaper than a launch.
    float* edges = n_layers > 1 && p.half > 0 ? reinterpret_cast<float*>(ws + wl.edges) : nullptr;
    const int64_t edges_stride_layer = (int64_t)wl.edges_layer_bytes / (int64_t)sizeof(float);
    launch(DKV_KERNEL_SCORE_EMIT, (score_emit_mfma<RS, KS>), dim3(grid_x, p.Hkv), dim3(TL::kThreads), lds_emit, st, p, chunk,
           n_layers, rev, k_stride_token * 2, k_stride_head * 2, cu, static_cast<const float*>(partials),
           lse_rows ? static_cast<const float*>(lse_rows) + last * lse_rows_stride_layer : nullptr, -lse_rows_stride_layer,
           lse_in, scores + last * scores_stride_layer, scores_stride_head, -scores_stride_layer, edges, edges_stride_layer);
    if (edges != nullptr)
      launch(DKV_KERNEL_SCORE_BORDERS, score_fix_borders, dim3(grid_x, p.Hkv, n_layers), dim3(64), 0, st, p, chunk,
             (int)TL::kKeys, cu,
             static_cast<const float*>(edges), edges_stride_layer, scores + last * scores_stride_layer, scores_stride_head,
             -scores_stride_layer);
  }
  if (phases & kPhaseLse)
    launch(DKV_KERNEL_SCORE_LSE, score_lse_mfma, dim3(p.n_seqs, p.Hkv), dim3(256), 0, st, p, chunk, (int)TL::kKeys, grid_x, cu,
           partials, lse_out);
  return hipGetLastError();
}

hipError_t launch_score_mfma(const Params& p, int phases, int n_layers, const void* const* q_layers,
                             const void* const* k_layers, int64_t k_stride_token, int64_t k_stride_head,
                             const int32_t* cu, float* scores, int64_t scores_stride_head, int64_t scores_stride_layer,
                             char* ws, const WorkspaceLayout& wl, const float* lse_in, const float* const* lse_layers,
                             float* lse_out, hipStream_t st) {
  if (p.rows <= 64)
    return launch_mfma_t<1, 4>(p, phases, n_layers, q_layers, k_layers, k_stride_token, k_stride_head, cu, scores,
                               scores_stride_head, scores_stride_layer, ws, wl, lse_in, lse_layers, lse_out, st);
  if (p.rows <= 128)
    return launch_mfma_t<2, 4>(p, phases, n_layers, q_layers, k_layers, k_stride_token, k_stride_head, cu, scores,
                               scores_stride_head, scores_stride_layer, ws, wl, lse_in, lse_layers, lse_out, st);
  return launch_mfma_t<4, 2>(p, phases, n_layers, q_layers, k_layers, k_stride_token, k_stride_head, cu, scores,
                             scores_stride_head, scores_stride_layer, ws, wl, lse_in, lse_layers, lse_out, st);
}

}  // namespace dkv
