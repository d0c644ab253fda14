// Observation-window scoring on the bf16 matrix cores (Eq. 1-2; Algorithm 1: softmax(Q_win K^T).mean(-2).pooling(-1)).
// bf16 inputs, head size 128, up to 256 score rows (G * ws) per KV head.
//
// A column of softmax(QK^T) summed over the rows needs every row's normaliser before any column can be
// finished, so the keys are swept twice (the second read is expected to come from the cache hierarchy):
//   stats kernel: S_tile = K_tile . Q^T  (keys as the MFMA M index, rows as N: a lane holds ONE row and 16
//                 keys, so the running row maximum / sum of exponentials is an in-lane reduction);
//   emit kernel:  S_tile = Q . K_tile^T  (rows as M, keys as N: a lane holds ONE key and 16 rows, so the sum
//                 over the rows is an in-lane reduction), p = exp2(S * c - lse2[row]), window/group sum,
//                 max-pool, write.
// Both use v_mfma_f32_32x32x16_bf16 with the whole Q block of the wavefront resident in registers and K tiles
// staged through LDS (coalesced 16-byte global loads, padded rows, 16-byte LDS reads in MFMA operand layout).
//
// Workgroup = RS x KS wavefronts: RS row slabs of 64 rows (2 MFMA tiles) x KS key tiles of 32 keys.
// Every workgroup owns a contiguous chunk of `chunk` keys of one (sequence, KV head).
//
// Pooling across chunk boundaries: a workgroup pools the outputs whose window lies inside its chunk and
// publishes its first/last 2*half raw sums; for every boundary the second of the two neighbours to arrive
// (integer ticket, no waiting) pools the 2*half outputs that straddle it. Maxima are order-independent, so
// the result does not depend on arrival order.
#include "dkv_internal.h"

namespace dkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kLdsRow = 272;          // bytes per staged key row: 256 data + 16 pad (conflict-free 16-byte reads)
constexpr int kMaxChunk = 2048;       // largest `chunk` the launcher picks
constexpr int kEdge = 64;             // floats reserved per boundary side (2 * half <= 62)
constexpr float kLog2e = 1.4426950408889634f;

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Chunking of n items into chunks of `chunk`, the tail merged into the last chunk when shorter than `tail_min`.
__host__ __device__ inline int n_chunks_merged(int n, int chunk, int tail_min) {
  if (n <= 0) return 0;
  const int c = (n - tail_min + chunk) / chunk;
  return c > 1 ? c : 1;
}

__device__ inline bool find_chunk_merged(const int32_t* __restrict__ cu, int n_seqs, int chunk, int tail_min,
                                         int window_off, int b, int& seq, int& c, int& nc, int& seq_begin,
                                         int& seq_len) {
  int begin = cu[0];
  for (int s = 0; s < n_seqs; ++s) {
    const int end = cu[s + 1];
    const int len = end - begin;
    const int n = n_chunks_merged(len - window_off, chunk, tail_min);
    if (b < n) { seq = s; c = b; nc = n; seq_begin = begin; seq_len = len; return true; }
    b -= n;
    begin = end;
  }
  return false;
}

template <int RS, int KS>
struct Tile {
  static constexpr int kThreads = RS * KS * 64;
  static constexpr int kKeys = KS * 32;                       // keys per iteration
  static constexpr int kPieces = kKeys * 16 / kThreads;       // 16-byte pieces per thread per tile
  static constexpr int kTileBytes = kKeys * kLdsRow;
};

// Q fragments of this wavefront's 64 rows: qf[t][j] = 8 consecutive head-dim elements (16 j + 8 (lane / 32) ..)
// of row rs * 64 + t * 32 + lane % 32; rows >= rows are zero.
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

template <int RS, int KS>
__device__ inline void load_tile(const char* __restrict__ k_head, int64_t stride_token_b, int key0, int last_key,
                                 uint4 (&reg)[Tile<RS, KS>::kPieces]) {
#pragma unroll
  for (int i = 0; i < Tile<RS, KS>::kPieces; ++i) {
    const int p = threadIdx.x + i * Tile<RS, KS>::kThreads;
    int key = key0 + (p >> 4);
    key = key < last_key ? key : last_key;   // clamp: loads stay inside the sequence, values are masked later
    reg[i] = *reinterpret_cast<const uint4*>(k_head + (int64_t)key * stride_token_b + (p & 15) * 16);
  }
}

template <int RS, int KS>
__device__ inline void store_tile(char* __restrict__ buf, const uint4 (&reg)[Tile<RS, KS>::kPieces]) {
#pragma unroll
  for (int i = 0; i < Tile<RS, KS>::kPieces; ++i) {
    const int p = threadIdx.x + i * Tile<RS, KS>::kThreads;
    *reinterpret_cast<uint4*>(buf + (p >> 4) * kLdsRow + (p & 15) * 16) = reg[i];
  }
}

// ------------------------------------------------------------------------------------------------------
// Row statistics: partial (max, sum of exp2) per chunk and row, merged by the last workgroup to arrive into
// lse2[row] = log2 sum_s exp2(c * x[row, s]) with c = softmax_scale * log2(e).
// ------------------------------------------------------------------------------------------------------
template <int RS, int KS>
__global__ __launch_bounds__(RS * KS * 64) void score_stats_mfma(Params p, int chunk, const uint16_t* __restrict__ q_win,
                                                                 const char* __restrict__ k, int64_t stride_token_b,
                                                                 int64_t stride_head_b, const int32_t* __restrict__ cu,
                                                                 int32_t* __restrict__ counters, float* __restrict__ lse2,
                                                                 float* __restrict__ partials) {
  using TL = Tile<RS, KS>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* tiles = smem;                                                          // 2 x kTileBytes
  float2* stat = reinterpret_cast<float2*>(smem + 2 * TL::kTileBytes);         // [KS][RS * 64]
  __shared__ int is_last;

  int seq, c, nc, begin, S;
  if (!find_chunk_merged(cu, p.n_seqs, chunk, 1, 0, blockIdx.x, seq, c, nc, begin, S)) return;
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rs = wave / KS, ks = wave % KS;
  const int c0 = c * chunk;
  const int c1 = c == nc - 1 ? S : c0 + chunk;
  const int n_iter = (c1 - c0 + TL::kKeys - 1) / TL::kKeys;
  const int prefix = S - p.w;                       // may be negative for sequences shorter than the window
  const float cexp = p.scale * kLog2e;

  const char* __restrict__ k_head = k + (int64_t)begin * stride_token_b + (int64_t)head * stride_head_b;
  const uint16_t* __restrict__ q_head = q_win + ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w * 128;
  bf16x8 qf[2][8];
  load_q_frags(q_head, rs, p.rows, qf);

  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};
  int limit[2];                                     // last key position visible to this lane's row (causal mask)
#pragma unroll
  for (int t = 0; t < 2; ++t) limit[t] = prefix + (rs * 64 + t * 32 + (lane & 31)) % p.w;

  uint4 reg[TL::kPieces];
  load_tile<RS, KS>(k_head, stride_token_b, c0, S - 1, reg);
  store_tile<RS, KS>(tiles, reg);
  __syncthreads();
  for (int it = 0; it < n_iter; ++it) {
    const int key0 = c0 + it * TL::kKeys;
    if (it + 1 < n_iter) load_tile<RS, KS>(k_head, stride_token_b, key0 + TL::kKeys, S - 1, reg);
    const char* tile = tiles + (it & 1) * TL::kTileBytes + (ks * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
    floatx16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[t][j] = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + j * 32));
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][j], acc[0], 0, 0, 0);   // D[key][row]
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[1][j], acc[1], 0, 0, 0);
    }
    const int wave_key0 = key0 + ks * 32;
    const bool need_mask = wave_key0 + 32 > (prefix < c1 ? prefix : c1);   // touches the window or runs past the chunk
    const int kb = wave_key0 + 4 * (lane >> 5);                            // + 8 * (j / 4) + j % 4
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      if (need_mask) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int s = kb + 8 * (j >> 2) + (j & 3);
          if (s > limit[t] || s >= c1) acc[t][j] = -INFINITY;
        }
      }
      float mx = acc[t][0];
#pragma unroll
      for (int j = 1; j < 16; ++j) mx = fmaxf(mx, acc[t][j]);
      const float m_new = fmaxf(m_run[t], mx * cexp);
      const float m_use = m_new == -INFINITY ? 0.0f : m_new;
      float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
#pragma unroll
      for (int j = 0; j < 16; j += 4) {
        s0 += fast_exp2(fmaf(acc[t][j], cexp, -m_use));
        s1 += fast_exp2(fmaf(acc[t][j + 1], cexp, -m_use));
        s2 += fast_exp2(fmaf(acc[t][j + 2], cexp, -m_use));
        s3 += fast_exp2(fmaf(acc[t][j + 3], cexp, -m_use));
      }
      l_run[t] = l_run[t] * fast_exp2(m_run[t] - m_use) + ((s0 + s1) + (s2 + s3));
      m_run[t] = m_new;
    }
    if (it + 1 < n_iter) store_tile<RS, KS>(tiles + ((it + 1) & 1) * TL::kTileBytes, reg);
    __syncthreads();
  }
  // ---- merge the two half-wavefronts (same row, other keys), then the KS key tiles, then publish
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const float m2 = __shfl_xor(m_run[t], 32), l2 = __shfl_xor(l_run[t], 32);
    const float M = fmaxf(m_run[t], m2);
    const float Mu = M == -INFINITY ? 0.0f : M;
    const float Lsum = l_run[t] * fast_exp2(m_run[t] - Mu) + l2 * fast_exp2(m2 - Mu);
    if (lane < 32) stat[ks * (RS * 64) + rs * 64 + t * 32 + lane] = make_float2(M, Lsum);
  }
  __syncthreads();
  float* __restrict__ part = partials + (((int64_t)blockIdx.x) * p.Hkv + head) * p.rows_pad * 2;
  for (int r = tid; r < RS * 64 && r < p.rows_pad; r += TL::kThreads) {
    float M = -INFINITY;
#pragma unroll
    for (int q = 0; q < KS; ++q) M = fmaxf(M, stat[q * (RS * 64) + r].x);
    const float Mu = M == -INFINITY ? 0.0f : M;
    float Lsum = 0.0f;
#pragma unroll
    for (int q = 0; q < KS; ++q) {
      const float2 v = stat[q * (RS * 64) + r];
      Lsum += v.y * fast_exp2(v.x - Mu);
    }
    part[2 * r] = M;
    part[2 * r + 1] = Lsum;
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const int ticket = atomicAdd(&counters[seq * p.Hkv + head], 1);
    is_last = ticket == nc - 1;
    if (is_last) counters[seq * p.Hkv + head] = 0;       // ready for the next call
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  const int first = blockIdx.x - c;                        // linear index of this sequence's chunk 0
  for (int r = tid; r < p.rows_pad; r += TL::kThreads) {
    float out = INFINITY;                                  // padding rows: exp2(x - inf) = 0 in the emit kernel
    if (r < p.rows) {
      float M = -INFINITY;
      for (int cc = 0; cc < nc; ++cc) {
        const int64_t e = ((((int64_t)(first + cc)) * p.Hkv + head) * p.rows_pad + r) * 2;
        M = fmaxf(M, __hip_atomic_load(partials + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      }
      const float Mu = M == -INFINITY ? 0.0f : M;
      float Lsum = 0.0f;
      for (int cc = 0; cc < nc; ++cc) {
        const int64_t e = ((((int64_t)(first + cc)) * p.Hkv + head) * p.rows_pad + r) * 2;
        const float vm = __hip_atomic_load(partials + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float vl = __hip_atomic_load(partials + e + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        Lsum += vl * fast_exp2(vm - Mu);
      }
      out = M + __log2f(Lsum);
    }
    lse2[((int64_t)seq * p.Hkv + head) * p.rows_pad + r] = out;
  }
}

// ------------------------------------------------------------------------------------------------------
// Scores: a[s] = row_scale * sum_rows exp2(c * x[row, s] - lse2[row]) over the chunk, max-pooled over the prefix.
// ------------------------------------------------------------------------------------------------------
template <int RS, int KS>
__global__ __launch_bounds__(RS * KS * 64) void score_emit_mfma(Params p, int chunk, const uint16_t* __restrict__ q_win,
                                                                const char* __restrict__ k, int64_t stride_token_b,
                                                                int64_t stride_head_b, const int32_t* __restrict__ cu,
                                                                const float* __restrict__ lse2,
                                                                int32_t* __restrict__ edge_counters,
                                                                float* __restrict__ edges, float* __restrict__ scores,
                                                                int64_t scores_stride_head) {
  using TL = Tile<RS, KS>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* tiles = smem;                                                          // 2 x kTileBytes
  float* part = reinterpret_cast<float*>(smem + 2 * TL::kTileBytes);           // [RS][kMaxChunk + 2 * kEdge]
  constexpr int kPartStride = kMaxChunk + 2 * kEdge;
  __shared__ int second[2];

  const int half = p.half;
  int seq, c, nc, begin, S;
  if (!find_chunk_merged(cu, p.n_seqs, chunk, 2 * half + 1, p.w, blockIdx.x, seq, c, nc, begin, S)) return;
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rs = wave / KS, ks = wave % KS;
  const int prefix = S - p.w;                                // > 0 here
  const int c0 = c * chunk;
  const int c1 = c == nc - 1 ? prefix : c0 + chunk;          // the last chunk takes the merged tail
  const int len = c1 - c0;                                   // <= chunk + 2 * half
  const int n_iter = (len + TL::kKeys - 1) / TL::kKeys;
  const float cexp = p.scale * kLog2e;

  const char* __restrict__ k_head = k + (int64_t)begin * stride_token_b + (int64_t)head * stride_head_b;
  const uint16_t* __restrict__ q_head = q_win + ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w * 128;
  bf16x8 qf[2][8];
  load_q_frags(q_head, rs, p.rows, qf);
  // lse2 of the rows this lane accumulates: register j of tile t is row rs*64 + t*32 + 8*(j/4) + 4*(lane/32) + j%4
  float lse_r[2][16];
  {
    const float* __restrict__ src = lse2 + ((int64_t)seq * p.Hkv + head) * p.rows_pad + rs * 64 + 4 * (lane >> 5);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j4 = 0; j4 < 4; ++j4) {
        const float4 v = *reinterpret_cast<const float4*>(src + t * 32 + 8 * j4);
        lse_r[t][4 * j4] = v.x; lse_r[t][4 * j4 + 1] = v.y; lse_r[t][4 * j4 + 2] = v.z; lse_r[t][4 * j4 + 3] = v.w;
      }
  }

  uint4 reg[TL::kPieces];
  load_tile<RS, KS>(k_head, stride_token_b, c0, S - 1, reg);
  store_tile<RS, KS>(tiles, reg);
  __syncthreads();
  for (int it = 0; it < n_iter; ++it) {
    const int key0 = c0 + it * TL::kKeys;
    if (it + 1 < n_iter) load_tile<RS, KS>(k_head, stride_token_b, key0 + TL::kKeys, S - 1, reg);
    const char* tile = tiles + (it & 1) * TL::kTileBytes + (ks * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
    floatx16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[t][j] = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + j * 32));
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[0][j], kf, acc[0], 0, 0, 0);   // D[row][key]
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[1][j], kf, acc[1], 0, 0, 0);
    }
    // prefix keys are visible to every window row: no mask. Fixed summation order per column.
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 16; j += 4) {
        s0 += fast_exp2(fmaf(acc[t][j], cexp, -lse_r[t][j]));
        s1 += fast_exp2(fmaf(acc[t][j + 1], cexp, -lse_r[t][j + 1]));
        s2 += fast_exp2(fmaf(acc[t][j + 2], cexp, -lse_r[t][j + 2]));
        s3 += fast_exp2(fmaf(acc[t][j + 3], cexp, -lse_r[t][j + 3]));
      }
    float col = (s0 + s1) + (s2 + s3);
    const float other = __shfl_xor(col, 32);
    col = lane < 32 ? col + other : other + col;         // rows 0-3 mod 8 first, in both half-wavefronts
    const int local = it * TL::kKeys + ks * 32 + (lane & 31);
    if (lane < 32 && local < kPartStride) part[rs * kPartStride + local] = col;
    if (it + 1 < n_iter) store_tile<RS, KS>(tiles + ((it + 1) & 1) * TL::kTileBytes, reg);
    __syncthreads();
  }
  // ---- sum the row slabs in a fixed order; positions past the chunk are ignored by the pooling
  for (int i = tid; i < n_iter * TL::kKeys && i < kPartStride; i += TL::kThreads) {
    float a = part[i];
#pragma unroll
    for (int q = 1; q < RS; ++q) a += part[q * kPartStride + i];
    part[i] = i < len ? a * p.row_scale : -INFINITY;
  }
  __syncthreads();
  float* __restrict__ out = scores + (int64_t)head * scores_stride_head + begin;
  // ---- outputs whose pooling window lies inside this chunk (sequence ends clip the window)
  const int lo = c == 0 ? 0 : half;
  const int hi = c == nc - 1 ? len : len - half;
  for (int i = lo + tid; i < hi; i += TL::kThreads) {
    float m = part[i];
    for (int o = 1; o <= half; ++o) {
      if (i - o >= 0) m = fmaxf(m, part[i - o]);
      if (i + o < len) m = fmaxf(m, part[i + o]);
    }
    out[c0 + i] = m;
  }
  if (c == nc - 1)
    for (int j = tid; j < p.w; j += TL::kThreads) out[prefix + j] = -INFINITY;   // guard over the window slots
  if (half == 0 || nc == 1) return;
  // ---- boundaries: publish 2*half raw sums per side, the second arrival pools the straddling outputs
  const int g = blockIdx.x;                                 // linear chunk index; boundary g = left edge of chunk g
  const int e2 = 2 * half;
  if (c > 0 && tid < e2) edges[(((int64_t)g) * p.Hkv + head) * (2 * kEdge) + kEdge + tid] = part[tid];
  if (c < nc - 1 && tid >= 64 && tid < 64 + e2)
    edges[(((int64_t)(g + 1)) * p.Hkv + head) * (2 * kEdge) + (tid - 64)] = part[len - e2 + (tid - 64)];
  __threadfence();
  __syncthreads();
  if (tid < 2) {
    const bool has = tid == 0 ? c > 0 : c < nc - 1;
    int sec = 0;
    if (has) {
      int32_t* ctr = &edge_counters[((int64_t)(g + tid)) * p.Hkv + head];
      sec = atomicAdd(ctr, 1) == 1;
      if (sec) *ctr = 0;                                    // ready for the next call
    }
    second[tid] = sec;
  }
  __syncthreads();
  for (int side = 0; side < 2; ++side) {
    if (!second[side]) continue;
    __threadfence();
    const int gb = g + side;                                // boundary index
    const int b = side == 0 ? c0 : c1;                      // boundary position in the sequence
    const float* __restrict__ e = edges + (((int64_t)gb) * p.Hkv + head) * (2 * kEdge);
    // raw[b - 2*half + i] for i in [0, 4*half): left side then right side
    if (tid < e2) {
      // output position b - half + tid needs raw [b - 2*half + tid, b + tid]
      float m = -INFINITY;
      for (int o = 0; o <= e2; ++o) {
        const int i = tid + o;                              // index into the 4*half raw values
        const float v = i < e2 ? __hip_atomic_load(e + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                               : __hip_atomic_load(e + kEdge + (i - e2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        m = fmaxf(m, v);
      }
      out[b - half + tid] = m;
    }
  }
}

bool score_mfma_supported(const Params& p, int dtype) {
  return dtype == DKV_BF16 && p.d == 128 && p.rows <= 256 && p.half <= 31;
}

static int pick_chunk(const Params& p, int keys_per_iter) {
  // aim at one workgroup per compute unit and round: enough keys per workgroup to amortise its Q load
  const long long total = (long long)p.total_tokens * p.Hkv;
  long long per_cu = total / 256;
  long long rounds = (per_cu + 512) / 1024;
  if (rounds < 1) rounds = 1;
  long long chunk = (per_cu + rounds - 1) / rounds;
  chunk = (chunk + keys_per_iter - 1) / keys_per_iter * keys_per_iter;
  if (chunk < 256) chunk = 256;
  if (chunk > kMaxChunk) chunk = kMaxChunk;
  return (int)chunk;
}

template <int RS, int KS>
static hipError_t launch_mfma_t(const Params& p, const void* q_win, const void* k, int64_t k_stride_token,
                                int64_t k_stride_head, const int32_t* cu, float* scores, int64_t scores_stride_head,
                                char* ws, const WorkspaceLayout& wl, hipStream_t st) {
  using TL = Tile<RS, KS>;
  const int chunk = pick_chunk(p, TL::kKeys);
  int32_t* counters = reinterpret_cast<int32_t*>(ws + wl.counters);
  int32_t* edge_counters = reinterpret_cast<int32_t*>(ws + wl.edge_counters);
  float* lse2 = reinterpret_cast<float*>(ws + wl.lse);
  float* partials = reinterpret_cast<float*>(ws + wl.partials);
  float* edges = reinterpret_cast<float*>(ws + wl.edges);
  const size_t lds_stats = 2 * TL::kTileBytes + (size_t)KS * RS * 64 * sizeof(float2);
  const size_t lds_emit = 2 * TL::kTileBytes + (size_t)RS * (kMaxChunk + 2 * kEdge) * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_stats_mfma<RS, KS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_stats);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_emit_mfma<RS, KS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_emit);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid_x = p.total_tokens / chunk + p.n_seqs;      // upper bound on chunks over all sequences
  hipLaunchKernelGGL((score_stats_mfma<RS, KS>), dim3(grid_x, p.Hkv), dim3(TL::kThreads), lds_stats, st, p, chunk,
                     static_cast<const uint16_t*>(q_win), static_cast<const char*>(k), k_stride_token * 2,
                     k_stride_head * 2, cu, counters, lse2, partials);
  hipLaunchKernelGGL((score_emit_mfma<RS, KS>), dim3(grid_x, p.Hkv), dim3(TL::kThreads), lds_emit, st, p, chunk,
                     static_cast<const uint16_t*>(q_win), static_cast<const char*>(k), k_stride_token * 2,
                     k_stride_head * 2, cu, lse2, edge_counters, edges, scores, scores_stride_head);
  return hipGetLastError();
}

hipError_t launch_score_mfma(const Params& p, const void* q_win, const void* k, int64_t k_stride_token,
                             int64_t k_stride_head, const int32_t* cu, float* scores, int64_t scores_stride_head,
                             char* ws, const WorkspaceLayout& wl, hipStream_t st) {
  if (p.rows <= 64) return launch_mfma_t<1, 4>(p, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, st);
  if (p.rows <= 128) return launch_mfma_t<2, 4>(p, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, st);
  return launch_mfma_t<4, 2>(p, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, st);
}

}  // namespace dkv
