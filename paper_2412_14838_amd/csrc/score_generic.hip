// Observation-window scoring, generic VALU path (Eq. 1-2; Algorithm 1: softmax(Q_win K^T).mean(-2).pooling(-1)).
// Handles every element type / head size the library accepts; used for fp32 inputs and for shapes the MFMA
// path is not built for. One thread owns one key: its row lives in registers, the query rows are staged
// through LDS 32 at a time.
//
// Two kernels, because a column of softmax(QK^T) summed over the rows needs every row's normaliser first:
//   stats:  per chunk of keys, per row: maximum m and sum l of exp(x - m), one partial per (chunk, row);
//   emit:   merges the partials of its (sequence, KV head) into lse[row] = m + log(l) (the kernel boundary is
//           the only synchronisation between workgroups), then a[s] = row_scale * sum_rows exp(x[row, s] -
//           lse[row]) for the chunk's keys plus a halo of (P-1)/2 on each side, max-pooled over the prefix.
#include "dkv_internal.h"

namespace dkv {

constexpr int kQRows = 32;   // query rows staged per pass

template <typename T> struct Elt;
template <> struct Elt<float> {
  static __device__ inline float load(const float* p) { return *p; }
};
template <> struct Elt<uint16_t> {   // bf16 bit patterns
  static __device__ inline float load(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
};

template <typename T, int D>
__device__ inline void load_key_row(const T* __restrict__ src, float (&kreg)[D]) {
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int j = 0; j < D; j += 4) {
      const float4 f = *reinterpret_cast<const float4*>(src + j);
      kreg[j] = f.x; kreg[j + 1] = f.y; kreg[j + 2] = f.z; kreg[j + 3] = f.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < D; j += 8) {
      const uint4 u = *reinterpret_cast<const uint4*>(src + j);
      const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        kreg[j + 2 * t] = __uint_as_float(wds[t] << 16);
        kreg[j + 2 * t + 1] = __uint_as_float(wds[t] & 0xffff0000u);
      }
    }
  }
}

// Stages query rows [r0, r0 + kQRows) of one (sequence, KV head) into LDS as fp32; rows >= rows are zero.
template <typename T, int D>
__device__ inline void stage_q(const T* __restrict__ q_head, int r0, int rows, float* __restrict__ qs) {
  for (int e = threadIdx.x; e < kQRows * D; e += blockDim.x) {
    const int r = r0 + e / D;
    qs[e] = r < rows ? Elt<T>::load(q_head + (int64_t)r * D + e % D) : 0.0f;
  }
}

// grid = (chunk upper bound, Hkv); block = kGenericKeys threads.
template <typename T, int D>
__global__ __launch_bounds__(kGenericKeys) void score_stats_generic(Params p, const T* __restrict__ q_win,
                                                                    const T* __restrict__ k, int64_t k_stride_token,
                                                                    int64_t k_stride_head, const int32_t* __restrict__ cu,
                                                                    float2* __restrict__ partials) {
  __shared__ float qs[kQRows * D];
  __shared__ float xs[kQRows][kGenericKeys + 1];
  int seq, c, begin, S;
  if (!find_chunk(cu, p.n_seqs, kGenericKeys, 0, blockIdx.x, seq, c, begin, S)) return;
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int s = c * kGenericKeys + tid;          // this thread's key position
  const int s_ld = s < S ? s : S - 1;            // clamp the load, mask the value
  float kreg[D];
  load_key_row<T, D>(k + (int64_t)(begin + s_ld) * k_stride_token + (int64_t)head * k_stride_head, kreg);
  const T* __restrict__ q_head = q_win + ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w * D;
  float2* __restrict__ part = partials + (((int64_t)blockIdx.x) * p.Hkv + head) * p.rows_pad;
  for (int r0 = 0; r0 < p.rows; r0 += kQRows) {
    __syncthreads();
    stage_q<T, D>(q_head, r0, p.rows, qs);
    __syncthreads();
    for (int rr = 0; rr < kQRows; ++rr) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < D; ++j) acc = fmaf(qs[rr * D + j], kreg[j], acc);
      const int i = (r0 + rr) % p.w;                       // window row of this query row
      const bool visible = s < S && s <= S - p.w + i;      // causal mask inside the window
      xs[rr][tid] = visible ? acc * p.scale : -INFINITY;
    }
    __syncthreads();
    // each wavefront reduces kQRows / 4 rows over the chunk's keys
    for (int rr = wv * (kQRows / 4); rr < (wv + 1) * (kQRows / 4); ++rr) {
      float m = -INFINITY;
      for (int j = lane; j < kGenericKeys; j += 64) m = fmaxf(m, xs[rr][j]);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      float l = 0.0f;
      if (m > -INFINITY)
        for (int j = lane; j < kGenericKeys; j += 64) l += __expf(xs[rr][j] - m);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
      if (lane == 0 && r0 + rr < p.rows_pad) part[r0 + rr] = make_float2(m, l);
    }
  }
}

// grid = (chunk upper bound over prefix outputs, Hkv); block = kGenericKeys threads. Thread t owns key
// c * CO - half + t; CO = kGenericKeys - 2 * half outputs per workgroup.
template <typename T, int D>
__global__ __launch_bounds__(kGenericKeys) void score_emit_generic(Params p, const T* __restrict__ q_win,
                                                                   const T* __restrict__ k, int64_t k_stride_token,
                                                                   int64_t k_stride_head, const int32_t* __restrict__ cu,
                                                                   const float2* __restrict__ partials,
                                                                   const float* __restrict__ lse_in,
                                                                   float* __restrict__ scores,
                                                                   int64_t scores_stride_head) {
  __shared__ float qs[kQRows * D];
  __shared__ float lse_s[DKV_MAX_ROWS];
  __shared__ float araw[kGenericKeys];
  const int CO = kGenericKeys - 2 * p.half;
  int seq, c, begin, S;
  if (!find_chunk(cu, p.n_seqs, CO, p.w, blockIdx.x, seq, c, begin, S)) return;
  const int head = blockIdx.y, tid = threadIdx.x;
  const int prefix = S - p.w;                          // > 0 here
  const int s = c * CO - p.half + tid;
  const bool in_prefix = s >= 0 && s < prefix;
  const int s_ld = s < 0 ? 0 : (s < S ? s : S - 1);
  float kreg[D];
  load_key_row<T, D>(k + (int64_t)(begin + s_ld) * k_stride_token + (int64_t)head * k_stride_head, kreg);
  const T* __restrict__ q_head = q_win + ((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w * D;
  if (lse_in != nullptr) {   // row normalisers supplied by the caller (natural log, one per window row)
    for (int r = tid; r < p.rows; r += kGenericKeys)
      lse_s[r] = lse_in[((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w + r];
  } else {
    // chunks of the statistics kernel that belong to this sequence: [first, first + n_full), in linear order
    int first = 0;
    for (int q = 0; q < seq; ++q) first += chunks_of(cu[q + 1] - cu[q], 0, kGenericKeys);
    const int n_full = chunks_of(S, 0, kGenericKeys);
    for (int r = tid; r < p.rows; r += kGenericKeys) {
      float m = -INFINITY;
      for (int cc = 0; cc < n_full; ++cc) m = fmaxf(m, partials[(((int64_t)(first + cc)) * p.Hkv + head) * p.rows_pad + r].x);
      float l = 0.0f;
      for (int cc = 0; cc < n_full; ++cc) {
        const float2 v = partials[(((int64_t)(first + cc)) * p.Hkv + head) * p.rows_pad + r];
        if (v.x > -INFINITY) l += v.y * __expf(v.x - m);
      }
      lse_s[r] = m + __logf(l);
    }
  }
  float a = 0.0f;
  for (int r0 = 0; r0 < p.rows; r0 += kQRows) {
    __syncthreads();
    stage_q<T, D>(q_head, r0, p.rows, qs);
    __syncthreads();
    const int rn = p.rows - r0 < kQRows ? p.rows - r0 : kQRows;
    for (int rr = 0; rr < rn; ++rr) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < D; ++j) acc = fmaf(qs[rr * D + j], kreg[j], acc);
      a += __expf(acc * p.scale - lse_s[r0 + rr]);     // prefix keys are visible to every window row
    }
  }
  araw[tid] = in_prefix ? a * p.row_scale : -INFINITY;  // outside the prefix: ignored by the pooling
  __syncthreads();
  float* __restrict__ out = scores + (int64_t)head * scores_stride_head + begin;
  if (tid >= p.half && tid < p.half + CO && s < prefix) {
    float m = araw[tid];
    for (int o = 1; o <= p.half; ++o) m = fmaxf(m, fmaxf(araw[tid - o], araw[tid + o]));
    out[s] = m;
  }
  // the workgroup that owns the last prefix outputs also writes the -inf guard over the window slots
  if (c == chunks_of(S, p.w, CO) - 1)
    for (int j = tid; j < p.w; j += kGenericKeys) out[prefix + j] = -INFINITY;
}

// Natural-log row normalisers from the chunk partials: lse_out[(seq * Hq + head * G) * w + r]. grid = (n_seqs, Hkv).
__global__ __launch_bounds__(256) void score_lse_generic(Params p, const int32_t* __restrict__ cu,
                                                         const float2* __restrict__ partials,
                                                         float* __restrict__ lse_out) {
  const int seq = blockIdx.x, head = blockIdx.y;
  int first = 0;
  for (int q = 0; q < seq; ++q) first += chunks_of(cu[q + 1] - cu[q], 0, kGenericKeys);
  const int n_full = chunks_of(cu[seq + 1] - cu[seq], 0, kGenericKeys);
  for (int r = threadIdx.x; r < p.rows; r += 256) {
    float m = -INFINITY;
    for (int cc = 0; cc < n_full; ++cc) m = fmaxf(m, partials[(((int64_t)(first + cc)) * p.Hkv + head) * p.rows_pad + r].x);
    float l = 0.0f;
    for (int cc = 0; cc < n_full; ++cc) {
      const float2 v = partials[(((int64_t)(first + cc)) * p.Hkv + head) * p.rows_pad + r];
      if (v.x > -INFINITY) l += v.y * __expf(v.x - m);
    }
    lse_out[((int64_t)seq * p.Hq + (int64_t)head * p.G) * p.w + r] = m + __logf(l);
  }
}

template <typename T, int D>
static hipError_t launch_generic_t(const Params& p, int phases, const void* q_win, const void* k, int64_t k_stride_token,
                                   int64_t k_stride_head, const int32_t* cu, float* scores, int64_t scores_stride_head,
                                   char* ws, const WorkspaceLayout& wl, const float* lse_in, float* lse_out,
                                   hipStream_t st) {
  float2* partials = ws ? reinterpret_cast<float2*>(ws + wl.partials) : nullptr;   // no workspace: lse supplied
  const int chunks_stats = p.total_tokens / kGenericKeys + p.n_seqs;
  if (phases & kPhaseStats)
    launch(DKV_KERNEL_SCORE_STATS, (score_stats_generic<T, D>), dim3(chunks_stats, p.Hkv), dim3(kGenericKeys), 0, st, p,
                       static_cast<const T*>(q_win), static_cast<const T*>(k), k_stride_token, k_stride_head, cu,
                       partials);
  const int CO = kGenericKeys - 2 * p.half;
  const int chunks_emit = p.total_tokens / CO + p.n_seqs;
  if (phases & kPhaseEmit)
    launch(DKV_KERNEL_SCORE_EMIT, (score_emit_generic<T, D>), dim3(chunks_emit, p.Hkv), dim3(kGenericKeys), 0, st, p,
                       static_cast<const T*>(q_win), static_cast<const T*>(k), k_stride_token, k_stride_head, cu,
                       partials, lse_in, scores, scores_stride_head);
  if (phases & kPhaseLse)
    launch(DKV_KERNEL_SCORE_LSE, score_lse_generic, dim3(p.n_seqs, p.Hkv), dim3(256), 0, st, p, cu, partials, lse_out);
  return hipGetLastError();
}

hipError_t launch_score_generic(const Params& p, int phases, int dtype, const void* q_win, const void* k, int64_t k_stride_token,
                                int64_t k_stride_head, const int32_t* cu, float* scores, int64_t scores_stride_head,
                                char* ws, const WorkspaceLayout& wl, const float* lse_in, float* lse_out, hipStream_t st) {
  if (dtype == DKV_F32) {
    if (p.d == 64) return launch_generic_t<float, 64>(p, phases, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, lse_in, lse_out, st);
    return launch_generic_t<float, 128>(p, phases, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, lse_in, lse_out, st);
  }
  if (p.d == 64) return launch_generic_t<uint16_t, 64>(p, phases, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, lse_in, lse_out, st);
  return launch_generic_t<uint16_t, 128>(p, phases, q_win, k, k_stride_token, k_stride_head, cu, scores, scores_stride_head, ws, wl, lse_in, lse_out, st);
}

}  // namespace dkv
