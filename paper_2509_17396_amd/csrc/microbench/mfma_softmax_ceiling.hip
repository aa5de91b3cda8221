// Microbenchmark, not part of libepicache: what this chip sustains for the instruction mix of the scoring passes.
// Every SIMD runs v_mfma_f32_32x32x16_bf16 into independent accumulators with 0-3 (multiply-add, exp2, add)
// triples of plain vector work behind each MFMA; operands live in registers, there is no memory or LDS traffic,
// nothing waits on anything.  The scoring passes (Sec. 2.3, Eq. 1) issue 8 MFMAs and 16 such triples per 32x32
// tile of logits at head_dim 128, i.e. the "+ 2" line.  Operands are random bf16 values (all-zero operands draw
// less power and run faster; last line).  One more variant takes the row sums through the matrix core instead of
// the vector adds: the weights are packed to bf16 and every fourth MFMA is followed by one product with a
// constant operand (2 extra MFMAs per 8), which is slower than the adds it replaces; another drops the multiply-add in
// front of the exp2 and pays one extra MFMA per 8 (scale and reference folded into the contraction): no faster.
// Build and run:  hipcc --offload-arch=gfx950 -O3 -std=c++17 -w -Xclang -target-feature -Xclang -packed-fp32-ops
//                 mfma_softmax_ceiling.hip -o mfma_softmax_ceiling && ./mfma_softmax_ceiling
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
constexpr int ITERS = 20000;

template <int NACC, int VALU>
__global__ __launch_bounds__(256) void k(const uint4* in, float* out, unsigned long long* cyc) {
  bf16x8 a = __builtin_bit_cast(bf16x8, in[threadIdx.x & 63]), b = __builtin_bit_cast(bf16x8, in[64 + (threadIdx.x & 63)]);
  f32x16 c[NACC];
  for (int i = 0; i < NACC; i++) for (int v = 0; v < 16; v++) c[i][v] = 0.f;
  float x[16];
  unsigned pk[4] = {0, 0, 0, 0};
  f32x16 ones_acc = {0};
  for (int v = 0; v < 16; v++) x[v] = threadIdx.x * 1e-3f + v;
  unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < ITERS; it++) {
#pragma unroll
    for (int i = 0; i < NACC; i++) {
      c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i], 0, 0, 0);
      if (VALU == 21) {   // same without the multiply at all
#pragma unroll
        for (int v = 0; v < 2; v++) {
          const int j = (i * 2 + v) & 15;
          x[j] = __builtin_amdgcn_exp2f(x[j]);
          x[(j + 5) & 15] = x[(j + 5) & 15] * 0.5f + x[j];
        }
        if ((i & 7) == 7) ones_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, ones_acc, 0, 0, 0);
      } else if (VALU == 12) {
#pragma unroll
        for (int v = 0; v < 2; v++) {
          const int j = (i * 2 + v) & 15;
          x[j] = __builtin_amdgcn_exp2f(fmaf(x[j], 0.999f, -0.001f));
        }
        typedef __attribute__((ext_vector_type(2))) float f2;
        typedef __attribute__((ext_vector_type(2))) __bf16 b2;
        const f2 pr = {x[(i * 2) & 15], x[(i * 2 + 1) & 15]};
        pk[i & 3] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, b2));
        if ((i & 3) == 3) {
          typedef __attribute__((ext_vector_type(4))) unsigned u4;
          const u4 w = {pk[0], pk[1], pk[2], pk[3]};
          ones_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, w), ones_acc, 0, 0, 0);
        }
      } else
#pragma unroll
      for (int v = 0; v < VALU; v++) {
        const int j = (i * VALU + v) & 15;
        x[j] = __builtin_amdgcn_exp2f(fmaf(x[j], 0.999f, -0.001f)) + x[(j + 5) & 15];
      }
    }
  }
  unsigned long long t1 = __builtin_readcyclecounter();
  float s = 0.f;
  for (int i = 0; i < NACC; i++) for (int v = 0; v < 16; v++) s += c[i][v];
  for (int v = 0; v < 16; v++) s += x[v] + ones_acc[v];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) cyc[0] = t1 - t0;
}

template <int NACC, int VALU>
void run(const char* tag, int wps, const uint4* in, float* out, unsigned long long* cyc) {
  dim3 g(256 * wps), b(256);
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  hipLaunchKernelGGL((k<NACC, VALU>), g, b, 0, 0, in, out, cyc);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL((k<NACC, VALU>), g, b, 0, 0, in, out, cyc);
  (void)hipEventRecord(e1);
  (void)hipEventSynchronize(e1);
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  unsigned long long c; (void)hipMemcpy(&c, cyc, 8, hipMemcpyDeviceToHost);
  const double flops = 2.0 * 32 * 32 * 16 * NACC * (double)ITERS * 4 * 256 * wps;
  printf("%-40s %d wave(s)/SIMD: %.3f ms, %.0f TFLOP/s, counter ticks per MFMA (one wave) %.1f, ticks/us %.0f\n", tag, wps, ms,
         flops / ms / 1e9, (double)c / ITERS / NACC, (double)c / (ms * 1e3));
  fflush(stdout);
}

int main() {
  uint4* in; float* out; unsigned long long* cyc;
  (void)hipMalloc(&in, 16 * 128); (void)hipMalloc(&out, 4 * 256 * 1024); (void)hipMalloc(&cyc, 8);
  uint32_t h[512];
  uint32_t s = 12345;
  for (int i = 0; i < 512; i++) { s = s * 1664525u + 1013904223u; h[i] = (s & 0x807F807Fu) | 0x3F003F00u; }  // random bf16 pairs around 1
  (void)hipMemcpy(in, h, sizeof(h), hipMemcpyHostToDevice);
  for (int wps : {1, 2, 3, 4}) {
    run<8, 0>("MFMA only, 8 accumulators", wps, in, out, cyc);
    run<8, 1>("MFMA + 1 (fma, exp2, add) each", wps, in, out, cyc);
    run<8, 2>("MFMA + 2 (fma, exp2, add) each", wps, in, out, cyc);
    run<8, 3>("MFMA + 3 (fma, exp2, add) each", wps, in, out, cyc);
    run<8, 12>("MFMA + 2 (fma, exp2) + cvt_pk, +1 MFMA per 4", wps, in, out, cyc);
    run<8, 21>("MFMA + 2 (exp2, fma-accumulate), +1 MFMA per 8", wps, in, out, cyc);
  }
  (void)hipMemset(in, 0, 16 * 128);
  run<8, 0>("MFMA only, 8 accumulators, zero operands", 2, in, out, cyc);
  return 0;
}
