// Decode-phase attention of one new token per sequence over the compressed cache of one layer (Section 4.3:
// decoding is unchanged - ordinary softmax attention over the keys and values the prefill retained).
//
// The cache block of (sequence, KV head) holds at most ws + B^l rows (a few thousand at most), so one layer's
// work is small and latency-bound: it is cut into slabs of 64 (bf16) or 32 (fp32) cache rows, one workgroup per (slab, KV head,
// sequence), so that a layer fills the GPU (split along the keys, merged by a second kernel):
//   partial kernel: K and V rows of the slab go to LDS with coalesced 16-byte loads; one thread per (row, query
//                   head of the group) takes the dot product; per query head the slab's maximum m, the sum of
//                   exponentials l and the unnormalised output acc[d] = sum_r exp(x_r - m) V_r are written;
//   merge kernel:   out = sum_s acc_s exp(m_s - M) / sum_s l_s exp(m_s - M), lse = M + log(sum ...).
// All arithmetic in fp32 on the vector ALU (a single query row per head leaves nothing for the matrix cores).
#include "dkv_internal.h"

namespace dkv {

constexpr int kDecThreads = 256;

__device__ inline float elem_to_float(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ inline float elem_to_float(float x) { return x; }

// Valid row r (0 <= r < w_q + n) of a cache block -> slot of the block: the w_q window rows sit in the last w_q of
// the first w slots, the n retained rows follow from slot w.
__device__ inline int cache_slot(int r, int w, int wq) { return r < wq ? w - wq + r : w + (r - wq); }

// Strides (in elements) from one layer of a call to the next: queries, cache blocks, partial results, outputs.
struct DecodeLayerStrides {
  int64_t q, cache, partial, out, lse;
};

// grid = (slabs x layers of the call, Hkv, n_seqs), 256 threads. partial layout per layer: [seq][Hq][slab][D + 2]
// floats: m, l, acc[D]. Layer i of the call is layer `layer` + i; its tensors lie i layer strides behind the pointers.
template <typename T, int D>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(int w, int layer_max, int L, int layer, int Hq,
                                                                     int G, float scale, int n_slabs,
                                                                     DecodeLayerStrides ls_, const T* __restrict__ q_new,
                                                                     const T* __restrict__ kb, const T* __restrict__ vb,
                                                                     int64_t stride_seq, int64_t stride_head,
                                                                     const int32_t* __restrict__ cu,
                                                                     const int32_t* __restrict__ counts,
                                                                     float* __restrict__ partial) {
  constexpr int ROWS = decode_slab_rows(sizeof(T));   // 64 two-byte rows or 32 four-byte rows: 32 KB of LDS for K and V
  constexpr int VEC = 16 / sizeof(T);                  // elements per 16-byte piece
  constexpr int PIECES = D / VEC;                      // pieces per row
  __shared__ __attribute__((aligned(16))) T ks[ROWS * D];
  __shared__ __attribute__((aligned(16))) T vs[ROWS * D];
  __shared__ float qs[kDecodeMaxGroup * D];
  __shared__ float xs[kDecodeMaxGroup * ROWS];          // logits, then exp(x - m)
  __shared__ float ms[kDecodeMaxGroup], ls[kDecodeMaxGroup];
  const int slab = blockIdx.x % n_slabs, lz = blockIdx.x / n_slabs, head = blockIdx.y, seq = blockIdx.z, tid = threadIdx.x;
  layer += lz;
  q_new += lz * ls_.q;
  kb += lz * ls_.cache;
  vb += lz * ls_.cache;
  partial += lz * ls_.partial;
  const int S = cu[seq + 1] - cu[seq];
  const int wq = S < w ? S : w;
  int n = counts[seq * L + layer];
  n = n < 0 ? 0 : (n < layer_max ? n : layer_max);
  const int R = wq + n;
  const int r0 = slab * ROWS;
  const int rows = R - r0 < ROWS ? R - r0 : ROWS;       // <= 0: an empty slab
  float* __restrict__ part = partial + (((int64_t)seq * Hq + (int64_t)head * G) * n_slabs + slab) * (D + 2);
  if (rows <= 0) return;                                // the merge kernel only reads the slabs that hold rows
  const T* __restrict__ kblock = kb + (int64_t)seq * stride_seq + (int64_t)head * stride_head;
  const T* __restrict__ vblock = vb + (int64_t)seq * stride_seq + (int64_t)head * stride_head;
  for (int pc = tid; pc < rows * PIECES; pc += kDecThreads) {
    const int r = pc / PIECES, c = pc % PIECES;
    const int64_t off = (int64_t)cache_slot(r0 + r, w, wq) * D + c * VEC;
    *reinterpret_cast<uint4*>(&ks[r * D + c * VEC]) = *reinterpret_cast<const uint4*>(kblock + off);
    *reinterpret_cast<uint4*>(&vs[r * D + c * VEC]) = *reinterpret_cast<const uint4*>(vblock + off);
  }
  const T* __restrict__ q_head = q_new + ((int64_t)seq * Hq + (int64_t)head * G) * D;
  for (int i = tid; i < G * D; i += kDecThreads) qs[i] = elem_to_float(q_head[i]);
  __syncthreads();
  // logits: one (row, query head) pair per thread, the row read as 16-byte pieces. The lanes of a wavefront read
  // different rows of the LDS tile; each starts at a row-dependent piece, so that they fall on different banks.
  for (int pair = tid; pair < G * ROWS; pair += kDecThreads) {
    const int g = pair / ROWS, r = pair % ROWS;
    float x = -INFINITY;
    if (r < rows) {
      float acc = 0.0f;
#pragma unroll 4
      for (int c = 0; c < PIECES; ++c) {
        const int cc = (c + r) & (PIECES - 1);
        T kv[VEC];
        *reinterpret_cast<uint4*>(kv) = *reinterpret_cast<const uint4*>(&ks[r * D + cc * VEC]);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc = fmaf(qs[g * D + cc * VEC + e], elem_to_float(kv[e]), acc);
      }
      x = acc * scale;
    }
    xs[pair] = x;
  }
  __syncthreads();
  // per query head: maximum and sum of exponentials over the slab's rows (one wavefront per head, a lane per row)
  {
    const int wave = tid >> 6, lane = tid & 63;
    for (int g = wave; g < G; g += kDecThreads / 64) {
      const float x = lane < ROWS ? xs[g * ROWS + lane] : -INFINITY;
      float m = x;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      const float e = lane < rows ? __expf(x - m) : 0.0f;
      float l = e;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
      if (lane < ROWS) xs[g * ROWS + lane] = e;
      if (lane == 0) { ms[g] = m; ls[g] = l; }
    }
  }
  __syncthreads();
  // unnormalised output: one (query head, head-dim element) per thread
  for (int i = tid; i < G * D; i += kDecThreads) {
    const int g = i / D, j = i % D;
    float acc = 0.0f;
    for (int r = 0; r < rows; ++r) acc = fmaf(xs[g * ROWS + r], elem_to_float(vs[r * D + j]), acc);
    part[(int64_t)g * n_slabs * (D + 2) + 2 + j] = acc;
  }
  if (tid < G) {
    part[(int64_t)tid * n_slabs * (D + 2)] = ms[tid];
    part[(int64_t)tid * n_slabs * (D + 2) + 1] = ls[tid];
  }
}

// grid = (Hq x layers of the call, n_seqs), D threads: thread j merges element j of the slabs that hold rows (the first
// ceil(R / rows_per_slab) of them; the others were never written).
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(int w, int layer_max, int L, int layer, int Hq, int n_slabs,
                                                         int rows_per_slab, DecodeLayerStrides ls_,
                                                         const int32_t* __restrict__ cu,
                                                         const int32_t* __restrict__ counts,
                                                         const float* __restrict__ partial, float* __restrict__ out,
                                                         float* __restrict__ lse_out) {
  __shared__ float factor[kDecodeMaxSlabs];
  __shared__ float red[2];
  const int g = blockIdx.x % Hq, lz = blockIdx.x / Hq, seq = blockIdx.y, j = threadIdx.x;
  layer += lz;
  partial += lz * ls_.partial;
  out += lz * ls_.out;
  if (lse_out) lse_out += lz * ls_.lse;
  const int S = cu[seq + 1] - cu[seq];
  int n = counts[seq * L + layer];
  n = n < 0 ? 0 : (n < layer_max ? n : layer_max);
  const int R = (S < w ? S : w) + n;
  const int used = (R + rows_per_slab - 1) / rows_per_slab;            // <= n_slabs <= kDecodeMaxSlabs
  const float* __restrict__ part = partial + ((int64_t)seq * Hq + g) * n_slabs * (D + 2);
  // the first wavefront: maximum over the slabs, then every slab's weight exp(m_s - M) and the total sum
  if (j < 64) {
    float M = -INFINITY;
    for (int s = j; s < used; s += 64) M = fmaxf(M, part[(int64_t)s * (D + 2)]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    float Lsum = 0.0f;
    for (int s = j; s < used; s += 64) {
      const float f = __expf(part[(int64_t)s * (D + 2)] - M);
      factor[s] = f;
      Lsum += part[(int64_t)s * (D + 2) + 1] * f;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) Lsum += __shfl_xor(Lsum, o);
    if (j == 0) { red[0] = M; red[1] = Lsum; }
  }
  __syncthreads();
  float acc = 0.0f;
#pragma unroll 8
  for (int s = 0; s < used; ++s) acc = fmaf(part[(int64_t)s * (D + 2) + 2 + j], factor[s], acc);
  const float M = red[0], Lsum = red[1];
  // a sequence without any cached row (S = 0) has nothing to attend to: zeros, lse = -inf
  out[((int64_t)seq * Hq + g) * D + j] = used > 0 && Lsum > 0.0f ? acc / Lsum : 0.0f;
  if (lse_out && j == 0) lse_out[(int64_t)seq * Hq + g] = used > 0 && Lsum > 0.0f ? M + __logf(Lsum) : -INFINITY;
}

template <typename T, int D>
static hipError_t launch_decode_t(const Params& p, int layer, int n_layers, const void* q_new, const void* kb,
                                  const void* vb, int64_t stride_layer, int64_t stride_seq, int64_t stride_head,
                                  const int32_t* cu, const int32_t* counts, float* out, float* lse_out, float* partial,
                                  int64_t partial_stride_layer, hipStream_t st) {
  constexpr int kRows = decode_slab_rows(sizeof(T));
  const int n_slabs = (p.w + p.layer_max + kRows - 1) / kRows;
  DecodeLayerStrides ls{};
  ls.q = (int64_t)p.n_seqs * p.Hq * D;
  ls.cache = stride_layer;
  ls.partial = partial_stride_layer;
  ls.out = (int64_t)p.n_seqs * p.Hq * D;
  ls.lse = (int64_t)p.n_seqs * p.Hq;
  launch(DKV_KERNEL_DECODE, (decode_partial_kernel<T, D>), dim3(n_slabs * n_layers, p.Hkv, p.n_seqs), dim3(kDecThreads), 0,
         st, p.w, p.layer_max, p.L, layer, p.Hq, p.G, p.scale, n_slabs, ls, static_cast<const T*>(q_new),
         static_cast<const T*>(kb), static_cast<const T*>(vb), stride_seq, stride_head, cu, counts, partial);
  launch(DKV_KERNEL_DECODE, (decode_merge_kernel<D>), dim3(p.Hq * n_layers, p.n_seqs), dim3(D), 0, st, p.w, p.layer_max,
         p.L, layer, p.Hq, n_slabs, kRows, ls, cu, counts, static_cast<const float*>(partial), out, lse_out);
  return hipGetLastError();
}

// n_layers consecutive layers from `layer` on: queries and outputs [n_layers][n_seqs][Hq][d] contiguous, cache blocks
// stride_layer elements apart.
hipError_t launch_decode(const Params& p, int dtype, int layer, int n_layers, const void* q_new, const void* kb,
                         const void* vb, int64_t stride_layer, int64_t stride_seq, int64_t stride_head, const int32_t* cu,
                         const int32_t* counts, float* out, float* lse_out, char* ws, const WorkspaceLayout& wl,
                         hipStream_t st) {
  float* partial = reinterpret_cast<float*>(ws + wl.decode_partials);
  const int64_t psl = (int64_t)(wl.decode_partials_layer_bytes / sizeof(float));
  if (dtype == DKV_F32) {
    if (p.d == 64) return launch_decode_t<float, 64>(p, layer, n_layers, q_new, kb, vb, stride_layer, stride_seq, stride_head, cu, counts, out, lse_out, partial, psl, st);
    return launch_decode_t<float, 128>(p, layer, n_layers, q_new, kb, vb, stride_layer, stride_seq, stride_head, cu, counts, out, lse_out, partial, psl, st);
  }
  if (p.d == 64) return launch_decode_t<uint16_t, 64>(p, layer, n_layers, q_new, kb, vb, stride_layer, stride_seq, stride_head, cu, counts, out, lse_out, partial, psl, st);
  return launch_decode_t<uint16_t, 128>(p, layer, n_layers, q_new, kb, vb, stride_layer, stride_seq, stride_head, cu, counts, out, lse_out, partial, psl, st);
}

}  // namespace dkv
