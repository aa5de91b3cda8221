// Episode geometry on segment embeddings (paper Sec. 3.1): centroid and centroid-closest member of
// every cluster (Stage 1, Eq. 3) and query-to-episode matching (Stage 3a; Stage 3b's rule that a
// query below the similarity threshold opens a new episode).  Small, latency-bound kernels: the
// inputs are a few thousand embedding vectors at most.
//
// One workgroup per cluster (medoids) or per query (matching); a wave owns one vector at a time and
// reduces dot products with lane shuffles, so all sums have a fixed order and results repeat exactly.
#include "epicache_internal.h"

namespace epicache {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ float wave_sum(float x) {
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// (cosine, index) candidates: larger cosine wins, equal cosines go to the lower index.
__device__ __forceinline__ bool better(float c, int i, float best_c, int best_i) {
  return c > best_c || (c == best_c && i < best_i);
}

__device__ __forceinline__ float cosine_from(float dot, float sq_u, float sq_v) {
  const float den = sqrtf(sq_u) * sqrtf(sq_v);
  return den > 0.f ? dot / den : 0.f;
}

// Block-wide argmax over the per-wave candidates; the result lands in out_c / out_i (thread 0).
__device__ __forceinline__ void block_best(float c, int i, float* sc, int* si, float& out_c, int& out_i) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) sc[wave] = c, si[wave] = i;
  __syncthreads();
  out_c = sc[0], out_i = si[0];
  for (int w = 1; w < kWaves; w++)
    if (better(sc[w], si[w], out_c, out_i)) out_c = sc[w], out_i = si[w];
}

constexpr int kNoIndex = 0x7fffffff;

constexpr int kMedoidThreads = 1024;
constexpr int kMedoidWaves = kMedoidThreads / 64;
constexpr int kMaxDim = 8192;  // the centroid of a cluster is kept in LDS while its members are compared
constexpr int kRowsInFlight = 32;

// Centroids: workgroup (e, j) owns dims [256 j, 256 j + 256) of cluster e and sweeps the segments in index
// order, 32 rows at a time.  Rows of other clusters are read too and multiplied by 0: no branch in the loop
// and 32 independent loads in flight per thread (the sweep is latency-bound; splitting the dims over
// workgroups multiplies the bytes in flight).
__global__ __launch_bounds__(kThreads) void episode_centroids(const float* __restrict__ emb,
                                                              const int32_t* __restrict__ assign, int K, int D,
                                                              float* __restrict__ centroids) {
  const int e = blockIdx.x, d = blockIdx.y * kThreads + threadIdx.x;
  const bool own = d < D;
  const float* col = emb + (own ? d : 0);
  float acc = 0.f;
  int count = 0;
  for (int k0 = 0; k0 < K; k0 += kRowsInFlight) {
    float x[kRowsInFlight];
    bool m[kRowsInFlight];
#pragma unroll
    for (int u = 0; u < kRowsInFlight; u++) {
      const int k = k0 + u < K ? k0 + u : K - 1;
      x[u] = col[(size_t)k * D];
      const bool mine = k0 + u < K && assign[k] == e;
      m[u] = mine;
      count += mine;
    }
#pragma unroll
    for (int u = 0; u < kRowsInFlight; u++) acc += m[u] ? x[u] : 0.f;  // a select: a non-finite row of another cluster cannot leak in
  }
  if (own) centroids[(size_t)e * D + d] = count ? acc / (float)count : 0.f;
}

// Centroid-closest member of cluster e: the centroid (written by the kernel above) goes to LDS, the members
// are dealt to the 16 waves round-robin, each wave keeps its best (cosine, index).
__global__ __launch_bounds__(kMedoidThreads) void episode_medoids(const float* __restrict__ emb,
                                                                  const int32_t* __restrict__ assign, int K,
                                                                  int D, const float* __restrict__ centroids,
                                                                  int32_t* __restrict__ medoid) {
  extern __shared__ float cent[];  // [D]
  __shared__ float sc[kMedoidWaves];
  __shared__ int si[kMedoidWaves];
  const int e = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  for (int d = tid; d < D; d += kMedoidThreads) cent[d] = centroids[(size_t)e * D + d];
  __syncthreads();
  float csq = 0.f;
  for (int d = lane; d < D; d += 64) csq = fmaf(cent[d], cent[d], csq);
  csq = wave_sum(csq);
  float best_c = -INFINITY;
  int best_i = kNoIndex, seen = 0;
  for (int k0 = 0; k0 < K; k0 += 64) {
    // membership of 64 segments at a time: one coalesced load and a ballot instead of a dependent load per segment
    const int kk = k0 + lane;
    uint64_t members = __ballot(kk < K && assign[kk] == e);
    while (members) {
      const int k = k0 + __ffsll((unsigned long long)members) - 1;
      members &= members - 1;
      if ((seen++ % kMedoidWaves) != wave) continue;
      float dot = 0.f, sq = 0.f;
      for (int d = lane; d < D; d += 64) {
        const float x = emb[(size_t)k * D + d];
        dot = fmaf(x, cent[d], dot);
        sq = fmaf(x, x, sq);
      }
      const float c = cosine_from(wave_sum(dot), wave_sum(sq), csq);
      if (better(c, k, best_c, best_i)) best_c = c, best_i = k;
    }
  }
  if (lane == 0) sc[wave] = best_c, si[wave] = best_i;
  __syncthreads();
  if (tid == 0) {
    float c = sc[0];
    int i = si[0];
    for (int w = 1; w < kMedoidWaves; w++)
      if (better(sc[w], si[w], c, i)) c = sc[w], i = si[w];
    medoid[e] = i == kNoIndex ? -1 : i;  // an empty cluster has no member
  }
}

__global__ __launch_bounds__(kThreads) void match_queries(const float* __restrict__ queries,
                                                          const float* __restrict__ centroids, int E, int D,
                                                          float tau, int32_t* __restrict__ episode,
                                                          float* __restrict__ cosine_opt) {
  __shared__ float sc[kWaves];
  __shared__ int si[kWaves];
  const int qi = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* q = queries + (size_t)qi * D;
  float qsq = 0.f;
  for (int d = lane; d < D; d += 64) qsq = fmaf(q[d], q[d], qsq);
  qsq = wave_sum(qsq);
  float best_c = -INFINITY;
  int best_i = kNoIndex;
  for (int e = wave; e < E; e += kWaves) {
    const float* c = centroids + (size_t)e * D;
    float dot = 0.f, sq = 0.f;
    for (int d = lane; d < D; d += 64) {
      const float x = c[d];
      dot = fmaf(x, q[d], dot);
      sq = fmaf(x, x, sq);
    }
    const float cs = cosine_from(wave_sum(dot), qsq, wave_sum(sq));
    if (better(cs, e, best_c, best_i)) best_c = cs, best_i = e;
  }
  float c;
  int i;
  block_best(best_c, best_i, sc, si, c, i);
  if (tid == 0) {
    episode[qi] = c >= tau ? i : -1;
    if (cosine_opt) cosine_opt[qi] = c;
  }
}

}  // namespace

hipError_t launch_episode_medoids(const float* emb, const int32_t* assign, int K, int E, int D,
                                  float* centroids, int32_t* medoid, hipStream_t stream) {
  if (D > kMaxDim) return hipErrorInvalidValue;
  hipLaunchKernelGGL(episode_centroids, dim3(E, (D + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, emb,
                     assign, K, D, centroids);
  hipLaunchKernelGGL(episode_medoids, dim3(E), dim3(kMedoidThreads), (size_t)D * sizeof(float), stream, emb,
                     assign, K, D, centroids, medoid);
  return hipGetLastError();
}

hipError_t launch_match_queries(const float* queries, const float* centroids, int nq, int E, int D, float tau,
                                int32_t* episode, float* cosine_opt, hipStream_t stream) {
  hipLaunchKernelGGL(match_queries, dim3(nq), dim3(kThreads), 0, stream, queries, centroids, E, D, tau,
                     episode, cosine_opt);
  return hipGetLastError();
}

}  // namespace epicache
