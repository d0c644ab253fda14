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
// row. grid = (ceil((w + layer_max) / ROWS), Hkv, n_seqs * layers of the call).
template <int LANES>
__global__ __launch_bounds__(256) void gather_kernel(int w, int layer_max, int L, int layer0, int n_seqs, int row_bytes,
                                                     GatherSources src_layers,
                                                     int64_t stride_token_b, int64_t stride_head_b,
                                                     const int32_t* __restrict__ cu, const int32_t* __restrict__ idx0,
                                                     int64_t idx_stride_layer,
                                                     const int32_t* __restrict__ counts, char* __restrict__ k_out0,
                                                     char* __restrict__ v_out0, int64_t out_stride_layer_b,
                                                     int64_t out_stride_seq_b, int64_t out_stride_head_b) {
  constexpr int ROWS = 256 / LANES;
  const int seq = blockIdx.z % n_seqs, lz = blockIdx.z / n_seqs, head = blockIdx.y;
  const int layer = layer0 + lz;
  const char* __restrict__ k = src_layers.k[lz];
  const char* __restrict__ v = src_layers.v[lz];
  const int32_t* __restrict__ idx = idx0 + (int64_t)lz * idx_stride_layer;
  char* __restrict__ k_out = k_out0 + (int64_t)lz * out_stride_layer_b;
  char* __restrict__ v_out = v_out0 + (int64_t)lz * out_stride_layer_b;
  const int slot = blockIdx.x * ROWS + threadIdx.x / LANES;
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
    dim3 grid((slots + rows - 1) / rows, p.Hkv, p.n_seqs * n_layers);
    launch(DKV_KERNEL_GATHER, kernel, grid, dim3(256), 0, st, p.w, p.layer_max, p.L, layer, p.n_seqs, row_bytes, src,
           stride_token * elt_bytes, stride_head * elt_bytes, cu, idx, idx_stride_layer, counts,
           static_cast<char*>(k_out), static_cast<char*>(v_out), out_stride_layer * elt_bytes,
           out_stride_seq * elt_bytes, out_stride_head * elt_bytes);
  };
  if (lanes <= 8) go(gather_kernel<8>, 8);
  else if (lanes <= 16) go(gather_kernel<16>, 16);
  else go(gather_kernel<32>, 32);
  return hipGetLastError();
}

}  // namespace dkv
