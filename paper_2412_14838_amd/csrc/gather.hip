// Compaction of retained K/V rows (Algorithm 1, the two cat(K[:, :-ws].gather(indices), K[:, -ws:]) lines).
// Pure streaming copy: every row slot is moved as 16-byte lane transfers, K and V in the same pass.
#include "dkv_internal.h"

namespace dkv {

// Source tensors of the layers one call covers (kernel argument, indexed by the layer's place in the call).
struct GatherSources {
  const char* k[DKV_MAX_SELECT_LAYERS];
  const char* v[DKV_MAX_SELECT_LAYERS];
};

// One workgroup copies ROWS = 256 / LANES row slots of one (layer, sequence, KV head); LANES lanes x 16 bytes = one
// row. grid = (slot_blocks * n_seqs * layers of the call, Hkv), slot_blocks = ceil((w + layer_max) / ROWS): the
// (sequence, layer) pair rides in x, whose range is 2^31, not in z, whose range is 65535.
template <int LANES>
__global__ __launch_bounds__(256) void gather_kernel(int w, int layer_max, int L, int layer0, int n_seqs, int row_bytes,
                                                     int slot_blocks,
                                                     GatherSources src_layers,
                                                     int64_t stride_token_b, int64_t stride_head_b,
                                                     const int32_t* __restrict__ cu, const int32_t* __restrict__ idx0,
                                                     int64_t idx_stride_layer,
                                                     const int32_t* __restrict__ counts, char* __restrict__ k_out0,
                                                     char* __restrict__ v_out0, int64_t out_stride_layer_b,
                                                     int64_t out_stride_seq_b, int64_t out_stride_head_b) {
  constexpr int ROWS = 256 / LANES;
  const int pair = blockIdx.x / slot_blocks, slot_block = blockIdx.x % slot_blocks;
  const int seq = pair % n_seqs, lz = pair / n_seqs, head = blockIdx.y;
  const int layer = layer0 + lz;
  const char* __restrict__ k = src_layers.k[lz];
  const char* __restrict__ v = src_layers.v[lz];
  const int32_t* __restrict__ idx = idx0 + (int64_t)lz * idx_stride_layer;
  char* __restrict__ k_out = k_out0 + (int64_t)lz * out_stride_layer_b;
  char* __restrict__ v_out = v_out0 + (int64_t)lz * out_stride_layer_b;
  const int slot = slot_block * ROWS + threadIdx.x / LANES;
  const int lane = threadIdx.x % LANES;
  if (slot >= w + layer_max || lane * 16 >= row_bytes) return;
  const int begin = cu[seq];
  const int S = cu[seq + 1] - begin;
  const int prefix = S > w ? S - w : 0;
  int src;
  if (slot < w) {
    src = S - w + slot;                 // window row; absent when the sequence is shorter than the window
    if (src < 0) return;
  } else {
    const int j = slot - w;
    int count = counts[seq * L + layer];
    count = count < layer_max ? count : layer_max;
    if (j >= count) return;
    src = idx[((int64_t)seq * gridDim.y + head) * layer_max + j];   // gridDim.y = Hkv
    if (src < 0 || src >= prefix) return;
  }
  const int64_t in_off = (int64_t)(begin + src) * stride_token_b + (int64_t)head * stride_head_b + lane * 16;
  const int64_t out_off = (int64_t)seq * out_stride_seq_b + (int64_t)head * out_stride_head_b +
                          (int64_t)slot * row_bytes + lane * 16;
  const uint4 kk = *reinterpret_cast<const uint4*>(k + in_off);
  const uint4 vv = *reinterpret_cast<const uint4*>(v + in_off);
  *reinterpret_cast<uint4*>(k_out + out_off) = kk;
  *reinterpret_cast<uint4*>(v_out + out_off) = vv;
}

hipError_t launch_gather(const Params& p, int elt_bytes, int layer, int n_layers, const void* const* k_layers,
                         const void* const* v_layers, int64_t stride_token, int64_t stride_head, const int32_t* cu,
                         const int32_t* idx, int64_t idx_stride_layer, const int32_t* counts, void* k_out, void* v_out,
                         int64_t out_stride_layer, int64_t out_stride_seq, int64_t out_stride_head, hipStream_t st) {
  const int row_bytes = p.d * elt_bytes;          // 128, 256 or 512
  const int lanes = row_bytes / 16;               // 8, 16 or 32
  const int slots = p.w + p.layer_max;
  GatherSources src{};
  for (int i = 0; i < n_layers; ++i) {
    src.k[i] = static_cast<const char*>(k_layers[i]);
    src.v[i] = static_cast<const char*>(v_layers[i]);
  }
  auto go = [&](auto kernel, int LANES) {
    const int rows = 256 / LANES;
    const int slot_blocks = (slots + rows - 1) / rows;
    dim3 grid(slot_blocks * p.n_seqs * n_layers, p.Hkv);
    launch(DKV_KERNEL_GATHER, kernel, grid, dim3(256), 0, st, p.w, p.layer_max, p.L, layer, p.n_seqs, row_bytes,
           slot_blocks, src,
           stride_token * elt_bytes, stride_head * elt_bytes, cu, idx, idx_stride_layer, counts,
           static_cast<char*>(k_out), static_cast<char*>(v_out), out_stride_layer * elt_bytes,
           out_stride_seq * elt_bytes, out_stride_head * elt_bytes);
  };
  if (lanes <= 8) go(gather_kernel<8>, 8);
  else if (lanes <= 16) go(gather_kernel<16>, 16);
  else go(gather_kernel<32>, 32);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// Tight packing of the final cache (Algorithm 1, last line: K^c, V^c <- K^b, V^b after the truncations).
// ------------------------------------------------------------------------------------------------------

// row_offsets[i] = first packed row of block i = (sequence q, layer l), i = q * L + l; a block holds
// Hkv * (w_q + n) rows, n = min(counts[q][l], layer_max), w_q = window rows the sequence has. One workgroup.
__global__ __launch_bounds__(1024) void pack_offsets_kernel(int n_seqs, int L, int Hkv, int w, int layer_max,
                                                            const int32_t* __restrict__ cu,
                                                            const int32_t* __restrict__ counts,
                                                            int64_t* __restrict__ row_offsets) {
  __shared__ long long wave_sum[16];
  __shared__ long long carry;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  const int total = n_seqs * L;
  for (int base = 0; base < total; base += 1024) {
    const int i = base + tid;
    long long rows = 0;
    if (i < total) {
      const int q = i / L;
      const int S = cu[q + 1] - cu[q];
      int n = counts[i];
      n = n < 0 ? 0 : (n < layer_max ? n : layer_max);
      rows = (long long)Hkv * ((S < w ? S : w) + n);
    }
    long long incl = rows;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const long long t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    if (lane == 63) wave_sum[wv] = incl;
    __syncthreads();
    long long before = carry;
    for (int j = 0; j < wv; ++j) before += wave_sum[j];
    if (i < total) row_offsets[i] = before + incl - rows;
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) row_offsets[total] = carry;
}

// grid = (slot_blocks * n_seqs * L, Hkv), slot_blocks = ceil((w + layer_max) / ROWS) (the (sequence, layer) pair rides
// in x: z ends at 65535), 256 threads: LANES lanes x 16 bytes = one row.
// Packed block of (q, l), head h: rows [off + h * (w_q + n), + w_q + n): the n retained rows in selection order,
// then the window rows in position order (the order of Algorithm 1's cat). Blocks that would pass `capacity_rows`
// are not written.
template <int LANES>
__global__ __launch_bounds__(256) void pack_cache_kernel(int w, int layer_max, int L, int n_seqs, int row_bytes,
                                                         int slot_blocks, const int32_t* __restrict__ cu,
                                                         const int32_t* __restrict__ counts,
                                                         const int64_t* __restrict__ row_offsets,
                                                         const char* __restrict__ kb, const char* __restrict__ vb,
                                                         int64_t stride_layer_b, int64_t stride_seq_b,
                                                         int64_t stride_head_b, char* __restrict__ k_packed,
                                                         char* __restrict__ v_packed, int64_t capacity_rows) {
  constexpr int ROWS = 256 / LANES;
  const int pair = blockIdx.x / slot_blocks;
  const int q = pair % n_seqs, l = pair / n_seqs, h = blockIdx.y;
  const int slot = (blockIdx.x % slot_blocks) * ROWS + threadIdx.x / LANES;      // packed slot inside the head's rows
  const int lane = threadIdx.x % LANES;
  if (lane * 16 >= row_bytes) return;
  const int S = cu[q + 1] - cu[q];
  const int wq = S < w ? S : w;
  int n = counts[q * L + l];
  n = n < 0 ? 0 : (n < layer_max ? n : layer_max);
  if (slot >= wq + n) return;
  const int64_t off = row_offsets[q * L + l];
  if (row_offsets[q * L + l + 1] > capacity_rows) return;
  // buffer layout: window rows first (the last wq of the w window slots), then the retained rows
  const int src_slot = slot < n ? w + slot : (w - wq) + (slot - n);
  const int64_t in_off = (int64_t)l * stride_layer_b + (int64_t)q * stride_seq_b + (int64_t)h * stride_head_b +
                         (int64_t)src_slot * row_bytes + lane * 16;
  const int64_t out_off = (off + (int64_t)h * (wq + n) + slot) * row_bytes + lane * 16;
  *reinterpret_cast<uint4*>(k_packed + out_off) = *reinterpret_cast<const uint4*>(kb + in_off);
  *reinterpret_cast<uint4*>(v_packed + out_off) = *reinterpret_cast<const uint4*>(vb + in_off);
}

hipError_t launch_pack_cache(const Params& p, int elt_bytes, const int32_t* cu, const int32_t* counts, const void* kb,
                             const void* vb, int64_t stride_layer, int64_t stride_seq, int64_t stride_head,
                             void* k_packed, void* v_packed, int64_t capacity_rows, int64_t* row_offsets,
                             hipStream_t st) {
  const int row_bytes = p.d * elt_bytes;
  const int lanes = row_bytes / 16;
  launch(DKV_KERNEL_PACK, pack_offsets_kernel, dim3(1), dim3(1024), 0, st, p.n_seqs, p.L, p.Hkv, p.w, p.layer_max, cu,
         counts, row_offsets);
  const int slots = p.w + p.layer_max;
  auto go = [&](auto kernel, int LANES) {
    const int rows = 256 / LANES;
    const int slot_blocks = (slots + rows - 1) / rows;
    dim3 grid(slot_blocks * p.n_seqs * p.L, p.Hkv);
    launch(DKV_KERNEL_PACK, kernel, grid, dim3(256), 0, st, p.w, p.layer_max, p.L, p.n_seqs, row_bytes, slot_blocks, cu, counts,
           static_cast<const int64_t*>(row_offsets), static_cast<const char*>(kb), static_cast<const char*>(vb),
           stride_layer * elt_bytes, stride_seq * elt_bytes, stride_head * elt_bytes, static_cast<char*>(k_packed),
           static_cast<char*>(v_packed), capacity_rows);
  };
  if (lanes <= 8) go(pack_cache_kernel<8>, 8);
  else if (lanes <= 16) go(pack_cache_kernel<16>, 16);
  else go(pack_cache_kernel<32>, 32);
  return hipGetLastError();
}

}  // namespace dkv
