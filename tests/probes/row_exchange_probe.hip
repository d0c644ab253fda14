// Measurement aid (not part of the library): what does it cost to exchange per-row softmax statistics between the
// workgroups of one (sequence, KV head) row INSIDE a kernel, which is what a scoring kernel that keeps its chunk of K
// on chip between the two sweeps of Eq. 1 would have to do once per layer?
//
// 256 workgroups of 512 threads, one per compute unit (forced by the LDS request), rows of `per_row` workgroups.
// Per iteration every workgroup publishes 128 (max, sum) pairs (1 KB), signals a per-(iteration, row) counter, waits
// - a bounded number of polls - until the whole row has signalled, and reads the row's records (per_row KB).
//   mode 0: agent-scope atomics for records, counter and reads (coherent across the eight XCCs of the device);
//   mode 1: rows built from workgroups that report the same XCC_ID; records written with plain stores and read with
//           plain loads from slots that are used once per launch (no stale line can sit in a first-level cache),
//           counter incremented and polled with atomics that execute in that XCC's L2.
// Prints microseconds per iteration (event time of the whole launch / iterations) and the mean time workgroups
// spend in the phases, from the 100 MHz wall clock. Every wait is bounded; a timeout is reported, not waited out.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

constexpr int kThreads = 512;
constexpr int kRows = 128;          // (max, sum) pairs per record
constexpr int kMaxSpin = 1 << 18;

__device__ inline unsigned xcc_id() { return __builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20) & 0xf; }   // HW_REG_XCC_ID

__device__ inline unsigned l2_atomic_read(unsigned* p) {   // returning atomic add of 0: executes in the XCC's L2
  unsigned v, zero = 0;
  asm volatile("global_atomic_add %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p), "v"(zero) : "memory");
  return v;
}
__device__ inline void l2_atomic_inc(unsigned* p) {
  unsigned one = 1;
  asm volatile("global_atomic_add %0, %1, off" :: "v"(p), "v"(one) : "memory");
}

__global__ __launch_bounds__(kThreads) void probe(float2* rec, unsigned* counters, unsigned* xcc_ticket, unsigned* xcc_of,
                                                  int iters, int per_row, int mode, int* errors, int* timeouts,
                                                  long long* stamps) {
  extern __shared__ char lds[];
  __shared__ int ok_s, row_s, member_s;
  const int tid = threadIdx.x;
  const int n_rows = gridDim.x / per_row;
  if (tid == 0) {
    const unsigned x = xcc_id();
    xcc_of[blockIdx.x] = x;
    if (mode == 0) { row_s = blockIdx.x / per_row; member_s = blockIdx.x % per_row; }
    else {   // rows inside one XCC, members in order of arrival (32 workgroups per XCC when every compute unit has one)
      const unsigned t = atomicAdd(&xcc_ticket[x], 1u);
      const int rows_per_xcc = (gridDim.x / 8) / per_row;
      row_s = x * rows_per_xcc + (t / per_row) % rows_per_xcc; member_s = t % per_row;
    }
  }
  __syncthreads();
  const int row = row_s, member = member_s;
  long long t_sig = 0, t_read = 0;
  int bad = 0;
  for (int it = 0; it < iters; ++it) {
    const long long t0 = wall_clock64();
    float2* my = rec + (((size_t)it * n_rows + row) * per_row + member) * kRows;
    if (tid < kRows) {
      const float2 v = make_float2((float)(it * 131 + row * 7 + member), (float)tid);
      if (mode == 0) __hip_atomic_store(reinterpret_cast<unsigned long long*>(&my[tid]), *reinterpret_cast<const unsigned long long*>(&v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else my[tid] = v;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    unsigned* ctr = counters + (size_t)it * n_rows + row;
    if (tid == 0) {
      int ok = 1;
      if (mode == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else l2_atomic_inc(ctr);
      int spins = 0;
      while (true) {
        const unsigned c = mode == 0 ? __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : l2_atomic_read(ctr);
        if (c >= (unsigned)per_row) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > kMaxSpin) { ok = 0; break; }
      }
      ok_s = ok;
    }
    __syncthreads();
    const long long t1 = wall_clock64();
    if (!ok_s) { if (tid == 0) atomicAdd(timeouts, 1); break; }
    const float2* rowrec = rec + ((size_t)it * n_rows + row) * per_row * kRows;
    float2 vv[8];                     // per_row * kRows <= 8 * kThreads; all loads in flight together
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = tid + j * kThreads;
      vv[j] = make_float2(0.f, 0.f);
      if (i < per_row * kRows) {
        if (mode == 0) {
          const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(&rowrec[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          vv[j] = *reinterpret_cast<const float2*>(&u);
        } else vv[j] = rowrec[i];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = tid + j * kThreads;
      if (i < per_row * kRows) bad += vv[j].x != (float)(it * 131 + row * 7 + i / kRows) || vv[j].y != (float)(i % kRows);
    }
    __syncthreads();
    const long long t2 = wall_clock64();
    t_sig += t1 - t0; t_read += t2 - t1;
  }
  if (bad) atomicAdd(errors, bad);
  if (tid == 0) { stamps[2 * blockIdx.x] = t_sig; stamps[2 * blockIdx.x + 1] = t_read; }
}

int main() {
  hipDeviceProp_t prop; CHECK(hipGetDeviceProperties(&prop, 0));
  const int grid = 256, iters = 64;
  printf("device: %s, %d compute units\n", prop.name, prop.multiProcessorCount); fflush(stdout);
  float2* rec; unsigned *counters, *ticket, *xcc_of; int *errors, *timeouts; long long* stamps;
  CHECK(hipMalloc(&rec, (size_t)iters * grid * kRows * sizeof(float2)));
  CHECK(hipMalloc(&counters, (size_t)iters * grid * 4)); CHECK(hipMalloc(&ticket, 64)); CHECK(hipMalloc(&xcc_of, grid * 4));
  CHECK(hipMalloc(&errors, 4)); CHECK(hipMalloc(&timeouts, 4)); CHECK(hipMalloc(&stamps, grid * 16));
  CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&probe), hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
  hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  for (int mode = 0; mode < 2; ++mode)
    for (int per_row : {32, 8}) {
      float best = 1e9f; int err = 0, to = 0;
      std::vector<long long> st(grid * 2);
      for (int rep = 0; rep < 5; ++rep) {
        CHECK(hipMemset(counters, 0, (size_t)iters * grid * 4)); CHECK(hipMemset(ticket, 0, 64));
        CHECK(hipMemset(errors, 0, 4)); CHECK(hipMemset(timeouts, 0, 4)); CHECK(hipMemset(rec, 0, (size_t)iters * grid * kRows * sizeof(float2)));
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(probe, dim3(grid), dim3(kThreads), 100 * 1024, 0, rec, counters, ticket, xcc_of, iters, per_row, mode, errors, timeouts, stamps);
        CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
        float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
        best = ms < best ? ms : best;
        CHECK(hipMemcpy(&err, errors, 4, hipMemcpyDeviceToHost)); CHECK(hipMemcpy(&to, timeouts, 4, hipMemcpyDeviceToHost));
        CHECK(hipMemcpy(st.data(), stamps, grid * 16, hipMemcpyDeviceToHost));
        if (to || err) break;
      }
      double sig = 0, rd = 0;
      for (int b = 0; b < grid; ++b) { sig += st[2 * b]; rd += st[2 * b + 1]; }
      printf("%-44s rows of %2d workgroups: %5.2f us per exchange (best of 5 launches of %d); publish + signal + wait %.2f us, read %.2f us; errors %d, timeouts %d\n",
             mode == 0 ? "agent scope (any placement):" : "inside one XCC (L2 atomics, fresh slots):", per_row, best * 1e3 / iters, iters,
             sig / grid / iters / 100.0, rd / grid / iters / 100.0, err, to);
      fflush(stdout);
    }
  std::vector<unsigned> x(grid);
  CHECK(hipMemcpy(x.data(), xcc_of, grid * 4, hipMemcpyDeviceToHost));
  int per_xcc[16] = {0};
  for (int b = 0; b < grid; ++b) per_xcc[x[b] & 15]++;
  printf("workgroup -> XCC of the first 16 workgroups:"); for (int b = 0; b < 16; ++b) printf(" %u", x[b]);
  printf("; workgroups per XCC:"); for (int i = 0; i < 8; ++i) printf(" %d", per_xcc[i]); printf("\n");
  return 0;
}
