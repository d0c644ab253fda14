// Decode-phase attention of one new token per sequence over the compressed cache of one layer (Section 4.3:
// decoding is unchanged - ordinary softmax attention over the keys and values the prefill retained).
//
// The cache block of (sequence, KV head) holds at most ws + B^l rows (a few thousand at most), so one layer's
// work is small: it is cut into slabs of 128 (bf16) or 64 (fp32) cache rows, one workgroup per (slab, KV head,
// sequence, layer of the call), so that the call fills the GPU (split along the keys, merged by a second kernel):
//   partial kernel: per query head the slab's maximum m, the sum of exponentials l and the unnormalised output
//                   acc[d] = sum_r exp(x_r - m) V_r.
//                   bf16 caches: on the matrix cores, see decode_partial_mfma_kernel below.
//                   fp32 caches: on the vector ALU, nothing staged: the lanes of a wavefront that share a cache row
//                   each hold one 16-byte piece of its K and of its V in registers (a wavefront-wide load covers
//                   whole rows, all loads of the slab are in flight together); the dot products are summed over
//                   those lanes by DPP, the softmax weights stay in registers, and each group of lanes leaves
//                   (m, l, acc) of its own rows in LDS, where the workgroup merges them;
//   merge kernel:   out = sum_s acc_s exp(m_s - M) / sum_s l_s exp(m_s - M), lse = M + log(sum ...).
// All sums in fp32.
#include "dkv_internal.h"

namespace dkv {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecHeadsPerPass = 4;     // query heads of the group taken through the slab together

// Valid row r (0 <= r < w_q + n) of a cache block -> slot of the block: the w_q window rows sit in the last w_q of
// the first w slots, the n retained rows follow from slot w.
__device__ inline int cache_slot(int r, int w, int wq) { return r < wq ? w - wq + r : w + (r - wq); }

// Strides (in elements) from one layer of a call to the next: queries, cache blocks, partial results, outputs.
struct DecodeLayerStrides {
  int64_t q, cache, partial, out, lse;
};

// A 16-byte piece as fp32 values.
__device__ inline void unpack_piece(const uint4& r, float (&f)[4], float) {
  f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
}

// Dot product of the pieces a and b, added to c.
__device__ inline float dot_piece(const uint4& a, const uint4& b, float c, float) {
  c = fmaf(__uint_as_float(a.x), __uint_as_float(b.x), c);
  c = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), c);
  c = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), c);
  c = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), c);
  return c;
}

// The value of another lane of the same row of 16 lanes (a DPP move; every lane is active where this is used).
template <int CTRL>
__device__ inline float dpp_lane(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the LANES (8, 16 or 32) consecutive lanes that share a cache row; every one of them gets the sum.
template <int LANES>
__device__ inline float sum_over_row_lanes(float v) {
  v += dpp_lane<0xB1>(v);                     // quad_perm [1,0,3,2]
  v += dpp_lane<0x4E>(v);                     // quad_perm [2,3,0,1]
  v += dpp_lane<0x141>(v);                    // row_half_mirror: the other quad of the 8
  if (LANES >= 16) v += dpp_lane<0x140>(v);   // row_mirror: the other 8 of the 16
  if (LANES >= 32) v += __shfl_xor(v, 16);
  return v;
}

// grid = (KV heads x sequences x layers of the call, slabs), 256 threads; the slab is the slow index, so that the
// slabs past the rows a block holds (the grid is sized without knowing the counts) come last and leave at once.
// partial layout per layer: [seq][Hq][slab][D + 2] floats: m, l, acc[D]. Layer i of the call is layer `layer` + i;
// its tensors lie i layer strides behind the pointers.
// ONE_PASS: the group has at most kDecHeadsPerPass query heads, so K is dead once the logits are there (fewer
// registers, one more wavefront per SIMD).
template <typename T, int D, bool ONE_PASS>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(int w, int layer_max, int L, int layer, int Hq,
                                                                     int Hkv, int n_seqs, int G, float scale,
                                                                     DecodeLayerStrides ls_, const T* __restrict__ q_new,
                                                                     const T* __restrict__ kb, const T* __restrict__ vb,
                                                                     int64_t stride_seq, int64_t stride_head,
                                                                     const int32_t* __restrict__ cu,
                                                                     const int32_t* __restrict__ counts,
                                                                     float* __restrict__ partial) {
  constexpr int ROWS = decode_slab_rows(sizeof(T));   // rows of a slab
  constexpr int VEC = 16 / sizeof(T);                  // elements per 16-byte piece
  constexpr int LPR = D / VEC;                         // lanes that share a row: 8, 16 or 32
  constexpr int RPL = 64 / LPR;                        // rows a wavefront-wide load covers
  constexpr int WROWS = ROWS / kDecWaves;              // rows per wavefront
  constexpr int ITER = WROWS / RPL;                    // loads of K (and of V) per lane
  constexpr int UNITS = kDecWaves * RPL;               // groups of lanes, each with rows of its own
  constexpr int GB = kDecHeadsPerPass;
  constexpr int USTRIDE = GB * D + 8;                  // floats per unit in LDS (padded: the units' pieces fall on different banks)
  static_assert(ITER >= 1 && ITER * RPL * kDecWaves == ROWS, "a slab is a whole number of wavefront-wide loads");
  __shared__ __attribute__((aligned(16))) float acc_s[UNITS * USTRIDE];
  __shared__ float m_s[UNITS * GB], l_s[UNITS * GB];
  const int n_slabs = gridDim.y, slab = blockIdx.y, tid = threadIdx.x;
  const int head = blockIdx.x % Hkv, seq = (blockIdx.x / Hkv) % n_seqs, lz = blockIdx.x / (Hkv * n_seqs);
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
  if (r0 >= R) return;                                  // an empty slab: the merge kernel only reads the slabs that hold rows
  float* __restrict__ part = partial + (((int64_t)seq * Hq + (int64_t)head * G) * n_slabs + slab) * (D + 2);
  const T* __restrict__ kblock = kb + (int64_t)seq * stride_seq + (int64_t)head * stride_head;
  const T* __restrict__ vblock = vb + (int64_t)seq * stride_seq + (int64_t)head * stride_head;
  const int wave = tid >> 6, lane = tid & 63, piece = lane % LPR, lg = lane / LPR;
  const int unit = wave * RPL + lg;
  const float scale2 = scale * 1.4426950408889634f;
  // this lane's pieces of K and V, all requested before the first is used; rows past the block's last read as zeros
  uint4 kreg[ITER], vreg[ITER];
  unsigned ok = 0u;
#pragma unroll
  for (int it = 0; it < ITER; ++it) {
    const int r = r0 + wave * WROWS + it * RPL + lg;
    kreg[it] = make_uint4(0, 0, 0, 0);
    vreg[it] = make_uint4(0, 0, 0, 0);
    if (r < R) {
      const int64_t off = (int64_t)cache_slot(r, w, wq) * D + piece * VEC;
      kreg[it] = *reinterpret_cast<const uint4*>(kblock + off);
      vreg[it] = *reinterpret_cast<const uint4*>(vblock + off);
      ok |= 1u << it;
    }
  }
  const T* __restrict__ q_head = q_new + ((int64_t)seq * Hq + (int64_t)head * G) * D + piece * VEC;
  for (int g0 = 0; g0 < (ONE_PASS ? 1 : G); g0 += GB) {
    uint4 qr[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      qr[g] = make_uint4(0, 0, 0, 0);
      if (g0 + g < G) qr[g] = *reinterpret_cast<const uint4*>(q_head + (int64_t)(g0 + g) * D);
    }
    // logits of this unit's rows in units of log 2 (exponentials are 2^x): x[g][it], the same in all lanes of the unit
    float x[GB][ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        const float a = sum_over_row_lanes<LPR>(dot_piece(qr[g], kreg[it], 0.0f, T()));
        x[g][it] = (ok >> it & 1u) ? a * scale2 : -INFINITY;
      }
    }
    // softmax weights relative to the unit's own maximum, and the unit's share of the output
    float m[GB], l[GB], acc[GB][VEC];
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      m[g] = x[g][0];
#pragma unroll
      for (int it = 1; it < ITER; ++it) m[g] = fmaxf(m[g], x[g][it]);
      l[g] = 0.0f;
      const float m_finite = fmaxf(m[g], -3.0e38f);      // a unit without rows: 2^(-inf - m_finite) = 0, not NaN
#pragma unroll
      for (int it = 0; it < ITER; ++it) {
        x[g][it] = __builtin_amdgcn_exp2f(x[g][it] - m_finite);
        l[g] += x[g][it];
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[g][e] = 0.0f;
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      float vf[VEC];
      unpack_piece(vreg[it], vf, T());
#pragma unroll
      for (int g = 0; g < GB; ++g)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[g][e] = fmaf(x[g][it], vf[e], acc[g][e]);
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      float* __restrict__ dst = &acc_s[unit * USTRIDE + g * D + piece * VEC];
#pragma unroll
      for (int e = 0; e < VEC; e += 4) *reinterpret_cast<float4*>(dst + e) = make_float4(acc[g][e], acc[g][e + 1], acc[g][e + 2], acc[g][e + 3]);
      if (piece == 0) { m_s[unit * GB + g] = m[g]; l_s[unit * GB + g] = l[g]; }
    }
    __syncthreads();
    // the slab's result per query head: the units merged (a unit without rows has m = -inf, l = 0, acc = 0)
    for (int i = tid; i < GB * D; i += kDecThreads) {
      const int g = i / D, j = i % D;
      if (g0 + g >= G) break;
      float M = -INFINITY;
#pragma unroll
      for (int u = 0; u < UNITS; ++u) M = fmaxf(M, m_s[u * GB + g]);      // finite: the slab's first row is valid
      float a = 0.0f, lsum = 0.0f;
#pragma unroll
      for (int u = 0; u < UNITS; ++u) {
        const float f = __builtin_amdgcn_exp2f(m_s[u * GB + g] - M);       // 0 for a unit without rows
        a = fmaf(acc_s[u * USTRIDE + g * D + j], f, a);
        lsum = fmaf(l_s[u * GB + g], f, lsum);
      }
      float* __restrict__ dst = part + (int64_t)(g0 + g) * n_slabs * (D + 2);
      dst[2 + j] = a;
      if (j == 0) { dst[0] = M * 0.6931471805599453f; dst[1] = lsum; }
    }
    __syncthreads();                                    // the LDS blocks are reused by the next heads of the group
  }
}

// ------------------------------------------------------------------------------------------------------
// The same partial results for bf16 caches on the matrix cores (v_mfma_f32_32x32x16_bf16). A wavefront owns 32 rows
// of the slab; all G <= 16 query heads of the group go through together as the N side of the tiles.
//   logits   S[row][head] = sum_d K[row][d] Q[head][d]: A = K with a lane per row (lane % 32) holding 8 consecutive
//            head-dim elements per 16-wide step (16-byte loads straight from the cache block: the two lanes of a row
//            fetch adjacent pieces, the eight steps complete the row's cache lines), B = Q likewise (heads past G are
//            zero). The result tile has a lane per head and, in its 16 registers, the rows
//            8 (i / 4) + 4 (lane / 32) + i % 4: the softmax over rows is in-lane plus one exchange between the halves.
//   output   O[head][d] = sum_row P[head][row] V[row][d]: A = P, which each lane already holds for its head - the
//            contraction index may visit the rows in any order, and the order (step s, half h, e) -> row
//            8 (2 s + e / 4) + 4 h + e % 4 is the one the registers are in. P goes in as two bf16 terms, hi + lo
//            (the residue is below 2^-17 of P), V exactly. B = V needs a lane per head-dim column with 8 rows in its
//            registers, i.e. V transposed: every wavefront stages its 32 rows of V in LDS (coalesced 16-byte loads,
//            rows padded by 16 bytes) and reads columns as 2-byte words.
// The per-wavefront results (max, sum, unnormalised output per head) meet in LDS as in the vector-ALU kernel.
// ------------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline uint32_t pack_bf16_pair(float a, float b) {
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}

template <int D>
__global__ __launch_bounds__(kDecThreads) void decode_partial_mfma_kernel(int w, int layer_max, int L, int layer, int Hq,
                                                                          int Hkv, int n_seqs, int G, float scale,
                                                                          DecodeLayerStrides ls_,
                                                                          const uint16_t* __restrict__ q_new,
                                                                          const uint16_t* __restrict__ kb,
                                                                          const uint16_t* __restrict__ vb,
                                                                          int64_t stride_seq, int64_t stride_head,
                                                                          const int32_t* __restrict__ cu,
                                                                          const int32_t* __restrict__ counts,
                                                                          float* __restrict__ partial) {
  constexpr int ROWS = decode_slab_rows(2);            // 128 rows per slab
  constexpr int WROWS = ROWS / kDecWaves;              // 32 rows per wavefront: one tile
  constexpr int DS = D / 16;                           // 16-wide steps over the head dimension
  constexpr int DT = D / 32;                           // 32-wide tiles of the output's head dimension
  constexpr int PIECES = D / 8;                        // 16-byte pieces per row
  constexpr int RPL = 64 / PIECES;                     // rows a wavefront-wide coalesced load covers
  constexpr int ITER = WROWS / RPL;                    // such loads per wavefront for its rows of V
  constexpr int VSTRIDE = D * 2 + 16;                  // bytes per staged row of V (the halves of a wavefront read rows 4 apart: other banks)
  constexpr int GMAX = kDecodeMaxGroup;
  static_assert(WROWS == 32 && GMAX <= 32, "one 32x32 tile of rows x heads per wavefront");
  static_assert(GMAX * D * 4 <= WROWS * VSTRIDE, "a wavefront's unnormalised outputs reuse its staging area");
  __shared__ __attribute__((aligned(16))) char stage[kDecWaves][WROWS * VSTRIDE];
  __shared__ float m_s[kDecWaves][GMAX], l_s[kDecWaves][GMAX];
  const int n_slabs = gridDim.y, slab = blockIdx.y, tid = threadIdx.x;
  const int head = blockIdx.x % Hkv, seq = (blockIdx.x / Hkv) % n_seqs, lz = blockIdx.x / (Hkv * n_seqs);
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
  if (r0 >= R) return;                                  // an empty slab
  float* __restrict__ part = partial + (((int64_t)seq * Hq + (int64_t)head * G) * n_slabs + slab) * (D + 2);
  const uint16_t* __restrict__ kblock = kb + (int64_t)seq * stride_seq + (int64_t)head * stride_head;
  const uint16_t* __restrict__ vblock = vb + (int64_t)seq * stride_seq + (int64_t)head * stride_head;
  const int wave = tid >> 6, lane = tid & 63, col = lane & 31, half = lane >> 5;
  const int wr0 = r0 + wave * WROWS;                    // first row of this wavefront
  const int rows_left = R - wr0;                        // rows of the wavefront that exist (may be <= 0)
  char* __restrict__ my_stage = stage[wave];

  // ---- loads: K in operand layout (lane = row), Q likewise (lane = head), V coalesced for the staging
  uint4 ka[DS], qb[DS], vreg[ITER];
  {
    const bool ok = col < rows_left;
    const int64_t off = ok ? (int64_t)cache_slot(wr0 + col, w, wq) * D + half * 8 : 0;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
      ka[ds] = make_uint4(0, 0, 0, 0);
      if (ok) ka[ds] = *reinterpret_cast<const uint4*>(kblock + off + ds * 16);
    }
    const uint16_t* __restrict__ q_head = q_new + ((int64_t)seq * Hq + (int64_t)head * G) * D;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
      qb[ds] = make_uint4(0, 0, 0, 0);
      if (col < G) qb[ds] = *reinterpret_cast<const uint4*>(q_head + (int64_t)col * D + ds * 16 + half * 8);
    }
    const int piece = lane % PIECES, lg = lane / PIECES;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int r = it * RPL + lg;
      vreg[it] = make_uint4(0, 0, 0, 0);                // rows past the block's last: zeros (their weights are zero too)
      if (r < rows_left) vreg[it] = *reinterpret_cast<const uint4*>(vblock + (int64_t)cache_slot(wr0 + r, w, wq) * D + piece * 8);
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it)
      *reinterpret_cast<uint4*>(my_stage + (it * RPL + lg) * VSTRIDE + piece * 16) = vreg[it];
  }

  // ---- logits: rows x heads
  floatx16 sc;
#pragma unroll
  for (int i = 0; i < 16; ++i) sc[i] = 0.0f;
#pragma unroll
  for (int ds = 0; ds < DS; ++ds)
    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[ds]), __builtin_bit_cast(bf16x8, qb[ds]), sc, 0, 0, 0);
  // this lane: head `col`, rows 8 (i / 4) + 4 half + i % 4 of the wavefront; in units of log 2
  const float scale2 = scale * 1.4426950408889634f;
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = 8 * (i >> 2) + 4 * half + (i & 3);
    sc[i] = row < rows_left ? sc[i] * scale2 : -INFINITY;
    mx = fmaxf(mx, sc[i]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_finite = fmaxf(mx, -3.0e38f);           // a wavefront without rows: 2^(-inf - m_finite) = 0, not NaN
  float lsum = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    sc[i] = __builtin_amdgcn_exp2f(sc[i] - m_finite);
    lsum += sc[i];
  }
  lsum += __shfl_xor(lsum, 32);
  if (half == 0 && col < GMAX) { m_s[wave][col] = mx; l_s[wave][col] = lsum; }

  // ---- P as two bf16 operands per step of 16 rows
  uint4 p_hi[2], p_lo[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = sc[8 * s + 2 * e], b = sc[8 * s + 2 * e + 1];
      hi[e] = pack_bf16_pair(a, b);
      lo[e] = pack_bf16_pair(a - __uint_as_float(hi[e] << 16), b - __uint_as_float(hi[e] & 0xffff0000u));
    }
    p_hi[s] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    p_lo[s] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
  }

  // ---- output: heads x head-dim columns; B = V read column-wise from the staged rows (this wavefront's own stores)
  floatx16 oc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) oc[dt][i] = 0.0f;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      uint32_t vv[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {                     // rows of the contraction slots 2 e and 2 e + 1 of step s
        const int row_a = 8 * (2 * s + (2 * e) / 4) + 4 * half + (2 * e) % 4;
        const uint32_t a = *reinterpret_cast<const uint16_t*>(my_stage + row_a * VSTRIDE + (dt * 32 + col) * 2);
        const uint32_t b = *reinterpret_cast<const uint16_t*>(my_stage + (row_a + 1) * VSTRIDE + (dt * 32 + col) * 2);
        vv[e] = a | (b << 16);
      }
      const bf16x8 vop = __builtin_bit_cast(bf16x8, make_uint4(vv[0], vv[1], vv[2], vv[3]));
      oc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, p_hi[s]), vop, oc[dt], 0, 0, 0);
      oc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, p_lo[s]), vop, oc[dt], 0, 0, 0);
    }
  }
  // this lane: column dt * 32 + col, heads 8 (i / 4) + 4 half + i % 4. The staged V is spent (the wavefront's LDS
  // accesses complete in order): its place takes the wavefront's outputs [head][D]
  float* __restrict__ my_out = reinterpret_cast<float*>(my_stage);
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int hd = 8 * (i >> 2) + 4 * half + (i & 3);
      if (hd < GMAX) my_out[hd * D + dt * 32 + col] = oc[dt][i];
    }
  __syncthreads();
  // ---- the slab's result per query head: the wavefronts merged
  for (int i = tid; i < G * D; i += kDecThreads) {
    const int g = i / D, j = i % D;
    float M = -INFINITY;
#pragma unroll
    for (int u = 0; u < kDecWaves; ++u) M = fmaxf(M, m_s[u][g]);          // finite: the slab's first row is valid
    float a = 0.0f, lt = 0.0f;
#pragma unroll
    for (int u = 0; u < kDecWaves; ++u) {
      const float f = __builtin_amdgcn_exp2f(m_s[u][g] - M);              // 0 for a wavefront without rows
      a = fmaf(reinterpret_cast<const float*>(stage[u])[g * D + j], f, a);
      lt = fmaf(l_s[u][g], f, lt);
    }
    float* __restrict__ dst = part + (int64_t)g * n_slabs * (D + 2);
    dst[2 + j] = a;
    if (j == 0) { dst[0] = M * 0.6931471805599453f; dst[1] = lt; }
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
  const dim3 grid_partial(p.Hkv * p.n_seqs * n_layers, n_slabs);
  if constexpr (sizeof(T) == 2) {
    launch(DKV_KERNEL_DECODE, (decode_partial_mfma_kernel<D>), grid_partial, dim3(kDecThreads), 0,
           st, p.w, p.layer_max, p.L, layer, p.Hq, p.Hkv, p.n_seqs, p.G, p.scale, ls, static_cast<const uint16_t*>(q_new),
           static_cast<const uint16_t*>(kb), static_cast<const uint16_t*>(vb), stride_seq, stride_head, cu, counts, partial);
  } else if (p.G <= kDecHeadsPerPass) {
    launch(DKV_KERNEL_DECODE, (decode_partial_kernel<T, D, true>), grid_partial, dim3(kDecThreads), 0,
           st, p.w, p.layer_max, p.L, layer, p.Hq, p.Hkv, p.n_seqs, p.G, p.scale, ls, static_cast<const T*>(q_new),
           static_cast<const T*>(kb), static_cast<const T*>(vb), stride_seq, stride_head, cu, counts, partial);
  } else {
    launch(DKV_KERNEL_DECODE, (decode_partial_kernel<T, D, false>), grid_partial, dim3(kDecThreads), 0,
           st, p.w, p.layer_max, p.L, layer, p.Hq, p.Hkv, p.n_seqs, p.G, p.scale, ls, static_cast<const T*>(q_new),
           static_cast<const T*>(kb), static_cast<const T*>(vb), stride_seq, stride_head, cu, counts, partial);
  }
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
