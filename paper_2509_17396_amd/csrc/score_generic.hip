// Generic scoring kernels (fp32 inputs, or bf16 with a head_dim the MFMA path
// does not cover).  Plain fp32 FMA dot products, one exponential per logit and
// pass; same two-pass structure as the MFMA path:
//   pass 1: per query row, base-2 log-sum-exp statistics over the N context keys
//   pass 2: per context key, reduce exp2(logit - lse_row) over the G*p rows (Eq. 1)
#include <hip/hip_bf16.h>

#include "epicache_internal.h"

namespace epicache {
namespace {

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__hip_bfloat16 x) { return __bfloat162float(x); }

constexpr int kMaxD = 256;

// One wave per query row; lanes stride over the keys.
template <typename T>
__global__ __launch_bounds__(256) void score_generic_stats(const T* __restrict__ q,
                                                          const T* __restrict__ k,
                                                          float2* __restrict__ stats, Plan pl) {
  __shared__ float qs[4][kMaxD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int r = blockIdx.x * 4 + wave;
  const bool active = r < pl.R;
  if (active) {
    const int g = r / pl.p, t = r % pl.p;
    const T* qrow = q + b * pl.qsb + (int64_t)(h * pl.G + g) * pl.qsh + (int64_t)t * pl.qst;
    for (int c = lane; c < pl.d; c += 64) qs[wave][c] = to_f32(qrow[c]);
  }
  __syncthreads();
  if (!active) return;
  const T* kbase = k + b * pl.ksb + (int64_t)h * pl.ksh;
  const int N = ctx_rows(pl, bh);
  float m = -INFINITY, D = 0.f;
  for (int i = lane; i < N; i += 64) {
    const T* krow = kbase + (int64_t)i * pl.kst;
    float dot = 0.f;
    for (int c = 0; c < pl.d; c++) dot = fmaf(qs[wave][c], to_f32(krow[c]), dot);
    const float z = dot * pl.c2;
    const float mn = fmaxf(m, z);
    D = D * exp2f(m - mn) + exp2f(z - mn);  // first term: exp2(-inf) * 0 = 0
    m = mn;
  }
  if (pl.causal_patch && N > 0) {
    // the patch's own keys follow the context; token t = r % p sees patch keys 0..t
    const int t = r % pl.p;
    for (int j = lane; j <= t; j += 64) {
      const T* krow = kbase + (int64_t)(N + j) * pl.kst;
      float dot = 0.f;
      for (int c = 0; c < pl.d; c++) dot = fmaf(qs[wave][c], to_f32(krow[c]), dot);
      const float z = dot * pl.c2;
      const float mn = fmaxf(m, z);
      D = D * exp2f(m - mn) + exp2f(z - mn);
      m = mn;
    }
  }
  for (int off = 32; off >= 1; off >>= 1) {
    const float mo = __shfl_xor(m, off), Do = __shfl_xor(D, off);
    const float mn = fmaxf(m, mo);
    const float a = (m == -INFINITY) ? 0.f : D * exp2f(m - mn);
    const float c = (mo == -INFINITY) ? 0.f : Do * exp2f(mo - mn);
    D = a + c;
    m = mn;
  }
  if (lane == 0) stats[(size_t)bh * pl.Rpad + r] = make_float2(m, D);
}

// 32 keys per workgroup, 8 row lanes per key.
template <typename T, int REDUCE>
__global__ __launch_bounds__(256) void score_generic_reduce(const T* __restrict__ q,
                                                           const T* __restrict__ k,
                                                           const float2* __restrict__ stats,
                                                           float* __restrict__ scores, Plan pl) {
  extern __shared__ float smem[];
  const int ldk = pl.d + 1;
  float* ks = smem;                // [32][d+1]
  float* red = smem + 32 * ldk;    // [8][32]
  const int bh = blockIdx.y, b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int key0 = blockIdx.x * 32;
  const int N = ctx_rows(pl, bh);
  if (key0 >= N) return;  // a shorter head of a ragged batch: no keys here
  const T* kbase = k + b * pl.ksb + (int64_t)h * pl.ksh;
  for (int e = threadIdx.x; e < 32 * pl.d; e += 256) {
    const int kk = e / pl.d, c = e % pl.d;
    const int i = key0 + kk;
    ks[kk * ldk + c] = i < N ? to_f32(kbase[(int64_t)i * pl.kst + c]) : 0.f;
  }
  __syncthreads();
  const int key = threadIdx.x & 31, rl = threadIdx.x >> 5;
  float acc = 0.f;  // weights are >= 0, so 0 is neutral for max and for sum
  for (int r = rl; r < pl.R; r += 8) {
    const int g = r / pl.p, t = r % pl.p;
    const T* qrow = q + b * pl.qsb + (int64_t)(h * pl.G + g) * pl.qsh + (int64_t)t * pl.qst;
    float dot = 0.f;
    for (int c = 0; c < pl.d; c++) dot = fmaf(to_f32(qrow[c]), ks[key * ldk + c], dot);
    const float2 st = stats[(size_t)bh * pl.Rpad + r];
    const float w = exp2f(dot * pl.c2 - st.x) / st.y;
    acc = REDUCE == EPICACHE_REDUCE_MAX ? fmaxf(acc, w) : acc + w;
  }
  red[rl * 32 + key] = acc;
  __syncthreads();
  if (rl == 0 && key0 + key < N) {
    for (int j = 1; j < 8; j++) {
      const float o = red[j * 32 + key];
      acc = REDUCE == EPICACHE_REDUCE_MAX ? fmaxf(acc, o) : acc + o;
    }
    scores[(size_t)bh * pl.N + key0 + key] = acc;
  }
}

// Caller-supplied natural-log normalisers -> the (base-2 max, sum) pairs the reduction pass reads.
// Rows of one KV head are contiguous in row_lse: (b*Hq + h*G + g)*p + t = (b*Hkv + h)*R + g*p + t.
__global__ void lse_to_stats(const float* __restrict__ row_lse, float2* __restrict__ stats, int R, int Rpad,
                             size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const size_t bh = i / R;
  const int r = (int)(i % R);
  stats[bh * Rpad + r] = make_float2(row_lse[i] * 1.44269504088896340736f, 1.0f);
}

template <typename T>
hipError_t launch_t(const Plan& pl, const T* q, const T* k, float* scores, float2* stats, bool stats_ready,
                    hipStream_t stream) {
  const int nbh = pl.nb * pl.Hkv;
  dim3 g1((pl.R + 3) / 4, nbh), g2((pl.N + 31) / 32, nbh);
  const size_t smem = (size_t)(32 * (pl.d + 1) + 8 * 32) * sizeof(float);
  if (!stats_ready) hipLaunchKernelGGL(score_generic_stats<T>, g1, dim3(256), 0, stream, q, k, stats, pl);
  if (pl.reduce == EPICACHE_REDUCE_MAX)
    hipLaunchKernelGGL((score_generic_reduce<T, EPICACHE_REDUCE_MAX>), g2, dim3(256), smem, stream,
                       q, k, stats, scores, pl);
  else
    hipLaunchKernelGGL((score_generic_reduce<T, EPICACHE_REDUCE_SUM>), g2, dim3(256), smem, stream,
                       q, k, stats, scores, pl);
  return hipGetLastError();
}

// dst[i] = reduce(dst[i], src[i]): the scores of two disjoint sets of scoring rows become those of their union
// (every scoring row is normalised on its own, so a long patch can be scored in chunks of its tokens).
template <int REDUCE>
__global__ void combine_scores(float* __restrict__ dst, const float* __restrict__ src, size_t total) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = REDUCE == EPICACHE_REDUCE_MAX ? fmaxf(dst[i], src[i]) : dst[i] + src[i];
}

}  // namespace

hipError_t launch_combine_scores(const Plan& pl, float* dst, const float* src, hipStream_t stream) {
  const size_t total = (size_t)pl.nb * pl.Hkv * pl.N;
  const size_t blocks = (total + 255) / 256;
  const dim3 grid((unsigned)(blocks < (1u << 20) ? blocks : (1u << 20)));
  if (pl.reduce == EPICACHE_REDUCE_MAX)
    hipLaunchKernelGGL(combine_scores<EPICACHE_REDUCE_MAX>, grid, dim3(256), 0, stream, dst, src, total);
  else
    hipLaunchKernelGGL(combine_scores<EPICACHE_REDUCE_SUM>, grid, dim3(256), 0, stream, dst, src, total);
  return hipGetLastError();
}

hipError_t launch_score_generic(const Plan& pl, const void* q, const void* k, float* scores,
                                float2* stats, bool stats_ready, hipStream_t stream) {
  if (pl.dtype == EPICACHE_DTYPE_F32)
    return launch_t<float>(pl, static_cast<const float*>(q), static_cast<const float*>(k), scores,
                           stats, stats_ready, stream);
  return launch_t<__hip_bfloat16>(pl, static_cast<const __hip_bfloat16*>(q),
                                  static_cast<const __hip_bfloat16*>(k), scores, stats, stats_ready, stream);
}

hipError_t launch_lse_to_stats(const Plan& pl, const float* row_lse, float2* stats, hipStream_t stream) {
  const size_t total = (size_t)pl.nb * pl.Hkv * pl.R;
  hipLaunchKernelGGL(lse_to_stats, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, row_lse,
                     stats, pl.R, pl.Rpad, total);
  return hipGetLastError();
}

}  // namespace epicache
