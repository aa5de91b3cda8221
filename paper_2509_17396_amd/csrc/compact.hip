// In-place, order-preserving compaction of the K and V caches (the cache returns
// to M entries after each block, paper Sec. 2.2 and App. A.3): row j of every
// (batch item, KV head) becomes row keep[j], keep strictly ascending.
//
// Hazard of doing this in place: keep[j] >= j, so the destination rows of one
// part of the job are the source rows of another.  The job is therefore cut
// only along axes that never alias - (batch item, head), K vs V, and 16-byte
// column slices of the head_dim row - and each workgroup walks its rows in
// ascending chunks: all loads of a chunk, a barrier, then its stores.  A later
// chunk only reads rows at or beyond its own first destination row, which no
// earlier chunk writes, so chunks need no further ordering.
#include "epicache_internal.h"

namespace epicache {
namespace {

constexpr int kUnroll = 8;  // row rounds in flight per thread: 8 x 16 B
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Every byte is touched exactly once, so loads and stores are marked non-temporal: among the cache-policy
// combinations tried (nt, sc0, sc1 on loads and stores) nt on both is the fastest, 4 % ahead of the default.
__device__ __forceinline__ u32x4 load_row16(const unsigned char* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ void store_row16(unsigned char* p, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}

__global__ __launch_bounds__(256) void compact_rows(unsigned char* __restrict__ kbuf,
                                                    unsigned char* __restrict__ vbuf,
                                                    const int32_t* __restrict__ keep, Plan pl,
                                                    int slices, int tpr) {
  // blockIdx.x = slice + slices * (tensor + 2 * bh)
  const int slice = blockIdx.x % slices;
  const int rest = blockIdx.x / slices;
  const int tensor = rest & 1, bh = rest >> 1;
  const int b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int rpr = 256 / tpr;                 // rows per round
  const int rr = threadIdx.x / tpr, col = threadIdx.x % tpr;
  const bool lane_on = rr < rpr;
  const size_t pitch = (size_t)pl.kst * pl.elem;
  unsigned char* base = (tensor ? vbuf : kbuf) + ((size_t)b * pl.ksb + (size_t)h * pl.ksh) * pl.elem +
                        ((size_t)slice * tpr + col) * 16;
  const int32_t* idx = keep + (size_t)bh * pl.keep_stride;
  int n = pl.n_keep;
  if (pl.n_kept) {  // ragged batch: this head's own count, never beyond the pitch of its index row
    n = pl.n_kept[bh];
    n = n < 0 ? 0 : (n > pl.keep_stride ? pl.keep_stride : n);
  }
  const int chunk = kUnroll * rpr;

  int src[kUnroll];
  auto load_idx = [&](int c0) {
#pragma unroll
    for (int u = 0; u < kUnroll; u++) {
      const int j = c0 + u * rpr + rr;
      src[u] = (lane_on && j < n) ? idx[j] : -1;
    }
  };
  load_idx(0);
  for (int c0 = 0; c0 < n; c0 += chunk) {
    u32x4 data[kUnroll];
    int cur[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; u++) {
      cur[u] = src[u];
      // Rows already in place (a kept prefix) are neither read nor written.  An index outside [0, N) (not one
      // epicache_topk writes) is skipped like the -1 of an idle lane, so no access leaves the rows the strides
      // were validated for.
      if ((unsigned)cur[u] >= (unsigned)pl.N) cur[u] = -1;
      if (cur[u] >= 0 && cur[u] != c0 + u * rpr + rr)
        data[u] = load_row16(base + (size_t)cur[u] * pitch);
    }
    if (c0 + chunk < n) load_idx(c0 + chunk);
    __syncthreads();  // every load of this chunk has landed before any of its stores
#pragma unroll
    for (int u = 0; u < kUnroll; u++) {
      const int j = c0 + u * rpr + rr;
      if (cur[u] >= 0 && cur[u] != j) store_row16(base + (size_t)j * pitch, data[u]);
    }
  }
}

}  // namespace

hipError_t launch_compact(const Plan& pl, const int32_t* keep, void* k, void* v,
                          hipStream_t stream) {
  if (!pl.n_kept && pl.N <= pl.M) return hipSuccess;  // nothing is evicted, rows stay where they are
  const int row_chunks = pl.d * pl.elem / 16;  // 16-byte chunks per row (head_dim % 8 == 0)
  const int64_t problems = (int64_t)pl.nb * pl.Hkv * 2;
  int slices = 1;
  while (problems * slices < 1024 && row_chunks % (slices * 2) == 0 && row_chunks / (slices * 2) >= 8)
    slices *= 2;
  const int tpr = row_chunks / slices;
  hipLaunchKernelGGL(compact_rows, dim3((unsigned)(problems * slices)), dim3(256), 0, stream,
                     static_cast<unsigned char*>(k), static_cast<unsigned char*>(v), keep, pl, slices,
                     tpr);
  return hipGetLastError();
}

}  // namespace epicache
