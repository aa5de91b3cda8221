// Microbenchmark, not part of libepicache: how the matrix cores and the vector ALU of one SIMD share issue, and
// what the clock does when the whole chip runs such code.  Hand-written instruction streams (inline assembly, all
// operands in registers): MFMAs alone, (multiply-add, exp2, add) triples alone, the two interleaved with the
// accumulators in VGPRs or AccVGPRs, the 16x16x32 form, the MFMAs bunched in front of the triples, and the
// interleaved stream with idle cycles (s_sleep) behind every iteration.  Run with
// 32 workgroups (an eighth of the CUs, one wave per SIMD: nothing throttles), 256 (every CU, one wave per SIMD)
// and 512 (two waves per SIMD).
// Build and run:  hipcc --offload-arch=gfx950 -O3 -std=c++17 -w -Xclang -target-feature -Xclang -packed-fp32-ops
//                 mfma_valu_issue.hip -o mfma_valu_issue && ./mfma_valu_issue
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
constexpr int ITERS = 20000;

#define TRIPLE(x, y) "v_fma_f32 " x ", " x ", %[c2], %[nm]\n\tv_exp_f32 " x ", " x "\n\tv_add_f32 " y ", " y ", " x "\n\t"
#define T2A TRIPLE("%[x0]", "%[s0]") TRIPLE("%[x1]", "%[s1]")
#define T2B TRIPLE("%[x2]", "%[s0]") TRIPLE("%[x3]", "%[s1]")

template <int MODE>
__global__ __launch_bounds__(256) void k(const uint4* in, float* out, unsigned long long* cyc) {
  bf16x8 a = __builtin_bit_cast(bf16x8, in[threadIdx.x & 63]), b = __builtin_bit_cast(bf16x8, in[64 + (threadIdx.x & 63)]);
  f32x16 c0 = {0}, c1 = {0}, c2v = {0}, c3 = {0};
  f32x4 d0 = {0}, d1 = {0}, d2 = {0}, d3 = {0};
  float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, s0 = 0, s1 = 0;
  const float c2 = 0.999f, nm = -0.001f;
  unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < ITERS; it++) {
    if (MODE == 0)  // 4 MFMAs (VGPR accumulators), 2 triples behind each
      asm volatile("v_mfma_f32_32x32x16_bf16 %[c0], %[a], %[b], %[c0]\n\t" T2A "v_mfma_f32_32x32x16_bf16 %[c1], %[a], %[b], %[c1]\n\t" T2B
                   "v_mfma_f32_32x32x16_bf16 %[c2v], %[a], %[b], %[c2v]\n\t" T2A "v_mfma_f32_32x32x16_bf16 %[c3], %[a], %[b], %[c3]\n\t" T2B
                   : [c0] "+v"(c0), [c1] "+v"(c1), [c2v] "+v"(c2v), [c3] "+v"(c3), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [s0] "+v"(s0), [s1] "+v"(s1)
                   : [a] "v"(a), [b] "v"(b), [c2] "v"(c2), [nm] "v"(nm));
    if (MODE == 6 || MODE == 7)  // MODE 0 with idle cycles behind it: s_sleep 1 (about 64 clocks) or s_sleep 3 (about 192)
      asm volatile("v_mfma_f32_32x32x16_bf16 %[c0], %[a], %[b], %[c0]\n\t" T2A "v_mfma_f32_32x32x16_bf16 %[c1], %[a], %[b], %[c1]\n\t" T2B
                   "v_mfma_f32_32x32x16_bf16 %[c2v], %[a], %[b], %[c2v]\n\t" T2A "v_mfma_f32_32x32x16_bf16 %[c3], %[a], %[b], %[c3]\n\t" T2B
                   "s_sleep %[nap]\n\t"
                   : [c0] "+v"(c0), [c1] "+v"(c1), [c2v] "+v"(c2v), [c3] "+v"(c3), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [s0] "+v"(s0), [s1] "+v"(s1)
                   : [a] "v"(a), [b] "v"(b), [c2] "v"(c2), [nm] "v"(nm), [nap] "n"(MODE == 6 ? 1 : 3));
    if (MODE == 1)  // the same with the accumulators in AccVGPRs
      asm volatile("v_mfma_f32_32x32x16_bf16 %[c0], %[a], %[b], %[c0]\n\t" T2A "v_mfma_f32_32x32x16_bf16 %[c1], %[a], %[b], %[c1]\n\t" T2B
                   "v_mfma_f32_32x32x16_bf16 %[c2v], %[a], %[b], %[c2v]\n\t" T2A "v_mfma_f32_32x32x16_bf16 %[c3], %[a], %[b], %[c3]\n\t" T2B
                   : [c0] "+a"(c0), [c1] "+a"(c1), [c2v] "+a"(c2v), [c3] "+a"(c3), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [s0] "+v"(s0), [s1] "+v"(s1)
                   : [a] "v"(a), [b] "v"(b), [c2] "v"(c2), [nm] "v"(nm));
    if (MODE == 2)  // 8 x 16x16x32 MFMAs (same flops as 4 x 32x32x16), 1 triple behind each
      asm volatile("v_mfma_f32_16x16x32_bf16 %[d0], %[a], %[b], %[d0]\n\t" TRIPLE("%[x0]", "%[s0]") "v_mfma_f32_16x16x32_bf16 %[d1], %[a], %[b], %[d1]\n\t" TRIPLE("%[x1]", "%[s1]")
                   "v_mfma_f32_16x16x32_bf16 %[d2], %[a], %[b], %[d2]\n\t" TRIPLE("%[x2]", "%[s0]") "v_mfma_f32_16x16x32_bf16 %[d3], %[a], %[b], %[d3]\n\t" TRIPLE("%[x3]", "%[s1]")
                   "v_mfma_f32_16x16x32_bf16 %[d0], %[a], %[b], %[d0]\n\t" TRIPLE("%[x0]", "%[s0]") "v_mfma_f32_16x16x32_bf16 %[d1], %[a], %[b], %[d1]\n\t" TRIPLE("%[x1]", "%[s1]")
                   "v_mfma_f32_16x16x32_bf16 %[d2], %[a], %[b], %[d2]\n\t" TRIPLE("%[x2]", "%[s0]") "v_mfma_f32_16x16x32_bf16 %[d3], %[a], %[b], %[d3]\n\t" TRIPLE("%[x3]", "%[s1]")
                   : [d0] "+v"(d0), [d1] "+v"(d1), [d2] "+v"(d2), [d3] "+v"(d3), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [s0] "+v"(s0), [s1] "+v"(s1)
                   : [a] "v"(a), [b] "v"(b), [c2] "v"(c2), [nm] "v"(nm));
    if (MODE == 3)  // 4 MFMAs alone
      asm volatile("v_mfma_f32_32x32x16_bf16 %[c0], %[a], %[b], %[c0]\n\tv_mfma_f32_32x32x16_bf16 %[c1], %[a], %[b], %[c1]\n\t"
                   "v_mfma_f32_32x32x16_bf16 %[c2v], %[a], %[b], %[c2v]\n\tv_mfma_f32_32x32x16_bf16 %[c3], %[a], %[b], %[c3]\n\t"
                   : [c0] "+v"(c0), [c1] "+v"(c1), [c2v] "+v"(c2v), [c3] "+v"(c3) : [a] "v"(a), [b] "v"(b));
    if (MODE == 4)  // 8 triples alone
      asm volatile(T2A T2B T2A T2B : [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [s0] "+v"(s0), [s1] "+v"(s1) : [c2] "v"(c2), [nm] "v"(nm));
    if (MODE == 5)  // 4 MFMAs, the 8 triples bunched behind the last
      asm volatile("v_mfma_f32_32x32x16_bf16 %[c0], %[a], %[b], %[c0]\n\tv_mfma_f32_32x32x16_bf16 %[c1], %[a], %[b], %[c1]\n\t"
                   "v_mfma_f32_32x32x16_bf16 %[c2v], %[a], %[b], %[c2v]\n\tv_mfma_f32_32x32x16_bf16 %[c3], %[a], %[b], %[c3]\n\t" T2A T2B T2A T2B
                   : [c0] "+v"(c0), [c1] "+v"(c1), [c2v] "+v"(c2v), [c3] "+v"(c3), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [s0] "+v"(s0), [s1] "+v"(s1)
                   : [a] "v"(a), [b] "v"(b), [c2] "v"(c2), [nm] "v"(nm));
  }
  unsigned long long t1 = __builtin_readcyclecounter();
  float s = x0 + x1 + x2 + x3 + s0 + s1;
  for (int v = 0; v < 16; v++) s += c0[v] + c1[v] + c2v[v] + c3[v];
  for (int v = 0; v < 4; v++) s += d0[v] + d1[v] + d2[v] + d3[v];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) cyc[0] = t1 - t0;
}

template <int MODE>
void run(const char* tag, int blocks, const uint4* in, float* out, unsigned long long* cyc) {
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(256), 0, 0, in, out, cyc);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(256), 0, 0, in, out, cyc);
  (void)hipEventRecord(e1);
  (void)hipEventSynchronize(e1);
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  unsigned long long c; (void)hipMemcpy(&c, cyc, 8, hipMemcpyDeviceToHost);
  printf("%-64s blocks %4d: %.3f ms, %.1f ns per iteration, timer ticks per iteration %.1f\n", tag, blocks, ms, ms * 1e6 / ITERS, (double)c / ITERS);
  fflush(stdout);
}

int main() {
  uint4* in; float* out; unsigned long long* cyc;
  (void)hipMalloc(&in, 16 * 128); (void)hipMalloc(&out, 4 * 256 * 2048); (void)hipMalloc(&cyc, 8);
  uint32_t h[512]; uint32_t s = 12345;
  for (int i = 0; i < 512; i++) { s = s * 1664525u + 1013904223u; h[i] = (s & 0x807F807Fu) | 0x3F003F00u; }
  (void)hipMemcpy(in, h, sizeof(h), hipMemcpyHostToDevice);
  for (int blocks : {32, 256, 512}) {
    run<3>("4 MFMA 32x32x16 alone", blocks, in, out, cyc);
    run<4>("8 (fma, exp2, add) alone", blocks, in, out, cyc);
    run<0>("4 x (MFMA 32x32x16 + 2 triples), VGPR accumulators", blocks, in, out, cyc);
    run<1>("4 x (MFMA 32x32x16 + 2 triples), AccVGPR accumulators", blocks, in, out, cyc);
    run<2>("8 x (MFMA 16x16x32 + 1 triple)", blocks, in, out, cyc);
    run<5>("4 MFMA 32x32x16, then 8 triples", blocks, in, out, cyc);
    run<6>("4 x (MFMA 32x32x16 + 2 triples), then s_sleep 1", blocks, in, out, cyc);
    run<7>("4 x (MFMA 32x32x16 + 2 triples), then s_sleep 3", blocks, in, out, cyc);
  }
  return 0;
}
