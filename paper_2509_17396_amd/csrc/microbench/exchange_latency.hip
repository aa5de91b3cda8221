// Microbenchmark, not part of libepicache: what one exchange of row statistics between the workgroups that share
// a KV head would cost if scoring kept its logits (or its keys) on chip and read K once.  Persistent grid of one
// workgroup per CU; per round every workgroup publishes 1.5 KB, bumps its cluster's counter (release), waits until
// all members have (acquire), and reads every member's 1.5 KB.  Every wait is bounded, so every wave exits.
// Build and run:  hipcc --offload-arch=gfx950 -O3 -std=c++17 -w -Xclang -target-feature -Xclang -packed-fp32-ops
//                 exchange_latency.hip -o exchange_latency && ./exchange_latency
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s failed: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)

constexpr int kSlotFloats = 384;  // 1.5 KB per workgroup and round

template <int CS, bool SAMEXCD>
__global__ __launch_bounds__(512) void exchange(float* slots, unsigned* counters, unsigned* fails, float* out,
                                                int rounds, int work_iters) {
  const int wg = blockIdx.x, tid = threadIdx.x;
  // cluster membership
  int cluster, member;
  if (SAMEXCD) {  // ids equal modulo 8 share an XCD
    const int xcd = wg & 7, within = wg >> 3;   // within: 0..gridDim/8-1
    cluster = xcd + 8 * (within / CS);
    member = within % CS;
  } else {
    cluster = wg / CS;
    member = wg % CS;
  }
  float acc = 0.f;
  for (int r = 0; r < rounds; r++) {
    // some register-only work between exchanges
    float x = (float)(tid + r);
    for (int i = 0; i < work_iters; i++) x = fmaf(x, 1.0001f, 0.5f);
    // publish this workgroup's slot (double buffered by round parity)
    float* mine = slots + (((size_t)(r & 1) * gridDim.x) + (size_t)cluster * CS + member) * kSlotFloats;
    if (tid < kSlotFloats) mine[tid] = x + (float)member;
    __syncthreads();
    if (tid == 0) {
      __atomic_fetch_add(&counters[cluster], 1u, __ATOMIC_RELEASE);  // agent scope by default in HIP
      const unsigned want = (unsigned)CS * (unsigned)(r + 1);
      int spins = 0;
      while (__atomic_load_n(&counters[cluster], __ATOMIC_ACQUIRE) < want) {
        if (++spins > 2000000) { atomicAdd(fails, 1u); break; }
        __builtin_amdgcn_s_sleep(2);
      }
    }
    __syncthreads();
    // read all members' slots
    const float* base = slots + (((size_t)(r & 1) * gridDim.x) + (size_t)cluster * CS) * kSlotFloats;
    float s = 0.f;
    for (int i = tid; i < CS * kSlotFloats; i += 512) s += __builtin_nontemporal_load(base + i);
    acc += s;
    __syncthreads();
  }
  if (acc == 123.456f) out[wg * 512 + tid] = acc;  // keep the work alive
}

template <int CS, bool SAMEXCD>
int run(int grid, int rounds, int work_iters, const char* tag) {
  float *slots, *out;
  unsigned *counters, *fails;
  CHECK(hipMalloc(&slots, (size_t)2 * grid * kSlotFloats * 4));
  CHECK(hipMalloc(&out, (size_t)grid * 512 * 4));
  CHECK(hipMalloc(&counters, 4096));
  CHECK(hipMalloc(&fails, 4));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  float best = 1e30f;
  unsigned hf = 0;
  for (int rep = 0; rep < 3; rep++) {
    CHECK(hipMemset(counters, 0, 4096));
    CHECK(hipMemset(fails, 0, 4));
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL((exchange<CS, SAMEXCD>), dim3(grid), dim3(512), 0, 0, slots, counters, fails, out, rounds, work_iters);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    if (ms < best) best = ms;
    CHECK(hipMemcpy(&hf, fails, 4, hipMemcpyDeviceToHost));
  }
  printf("%-28s grid %d cluster %d rounds %d work %d: %.3f ms total, %.2f us per round, wait failures %u\n", tag, grid, CS,
         rounds, work_iters, best, best * 1e3f / rounds, hf);
  fflush(stdout);
  hipFree(slots); hipFree(out); hipFree(counters); hipFree(fails);
  return 0;
}

int main() {
  int dev_cus = 0;
  CHECK(hipDeviceGetAttribute(&dev_cus, hipDeviceAttributeMultiprocessorCount, 0));
  printf("CUs %d\n", dev_cus);
  const int grid = 256;
  // baseline: no exchange cost visible when work dominates
  if (run<8, true>(grid, 200, 0, "same-xcd cs8 nowork")) return 1;
  if (run<8, true>(grid, 200, 2000, "same-xcd cs8 work2000")) return 1;
  if (run<8, false>(grid, 200, 0, "cross-xcd cs8 nowork")) return 1;
  if (run<32, true>(grid, 200, 0, "same-xcd cs32 nowork")) return 1;
  if (run<32, false>(grid, 200, 0, "cross-xcd cs32 nowork")) return 1;
  if (run<1, true>(grid, 200, 0, "cs1 nowork (floor)")) return 1;
  if (run<1, true>(grid, 200, 2000, "cs1 work2000 (floor)")) return 1;
  return 0;
}
