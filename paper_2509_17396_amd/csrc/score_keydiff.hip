// KeyDiff scoring (paper App. A.2, "KeyDiff"): an attention-free scorer for the same select /
// compact back end.  Per (batch item, KV head): anchor = mean of the N context keys, score of row i
// = -cos(k_i, anchor).  A zero key or a zero anchor has cosine 0.
//
// Two streaming passes over K, both HBM-bound:
//   keydiff_partial: column sums of 512-row chunks, one workgroup per chunk, written to the workspace
//                    (no atomics: the chunk sums are added in a fixed order, so results repeat exactly);
//   keydiff_scores:  every workgroup rebuilds the anchor from the chunk sums (a few KB from L2), then
//                    computes dot(k_i, anchor) and |k_i|^2 for its rows.
// A row is read by d*elem/16 threads with one 16-byte load each.  When those are 8 or 16 lanes (bf16
// d = 64/128, fp32 d = 32/64) the per-row sums are reduced with in-register lane permutations and the
// scores of a chunk leave through LDS as one contiguous run; other head dims meet in LDS.
#include <hip/hip_bf16.h>

#include <type_traits>

#include "epicache_internal.h"

namespace epicache {
namespace {

constexpr int kThreads = 256;
constexpr int kChunkRows = 512;  // rows per workgroup in both passes
constexpr int kUnroll = 8;       // row rounds in flight per thread in the scoring pass

template <typename T>
struct Vec;
template <>
struct Vec<float> {
  static constexpr int kLen = 4;
  __device__ static void unpack(const uint4& v, float (&x)[4]) {
    x[0] = __uint_as_float(v.x), x[1] = __uint_as_float(v.y);
    x[2] = __uint_as_float(v.z), x[3] = __uint_as_float(v.w);
  }
  __device__ static void load(const void* p, float (&x)[4]) { unpack(*reinterpret_cast<const uint4*>(p), x); }
};
template <>
struct Vec<__hip_bfloat16> {
  static constexpr int kLen = 8;
  __device__ static void unpack(const uint4& v, float (&x)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      x[2 * i] = __uint_as_float(w[i] << 16);          // bf16 -> fp32: the bits, shifted up
      x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static void load(const void* p, float (&x)[8]) { unpack(*reinterpret_cast<const uint4*>(p), x); }
};

template <typename T>
__global__ __launch_bounds__(kThreads) void keydiff_partial(const T* __restrict__ k,
                                                            float* __restrict__ partial, Plan pl, int chunks) {
  constexpr int VL = Vec<T>::kLen;
  __shared__ float sm[kThreads * VL];
  const int bh = blockIdx.y, b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int N = ctx_rows(pl, bh);
  const int tpr = pl.d / VL, rpr = kThreads / tpr;
  const int rr = threadIdx.x / tpr, col = threadIdx.x % tpr;
  const int row0 = blockIdx.x * kChunkRows;
  const int row_end = min(N, row0 + kChunkRows);
  const unsigned char* base = reinterpret_cast<const unsigned char*>(k + b * pl.ksb + (int64_t)h * pl.ksh) +
                              (size_t)col * 16;
  const size_t pitch = (size_t)pl.kst * sizeof(T);
  float acc[VL];
#pragma unroll
  for (int e = 0; e < VL; e++) acc[e] = 0.f;
  if (rr < rpr) {
    int row = row0 + rr;
    for (; row + 7 * rpr < row_end; row += 8 * rpr) {  // eight loads in flight per thread
      float x[8][VL];
#pragma unroll
      for (int u = 0; u < 8; u++) Vec<T>::load(base + (size_t)(row + u * rpr) * pitch, x[u]);
#pragma unroll
      for (int u = 0; u < 8; u++)
#pragma unroll
        for (int e = 0; e < VL; e++) acc[e] += x[u][e];
    }
    for (; row < row_end; row += rpr) {
      float x[VL];
      Vec<T>::load(base + (size_t)row * pitch, x);
#pragma unroll
      for (int e = 0; e < VL; e++) acc[e] += x[e];
    }
#pragma unroll
    for (int e = 0; e < VL; e++) sm[rr * pl.d + col * VL + e] = acc[e];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < pl.d; c += kThreads) {
    float s = 0.f;
    for (int g = 0; g < rpr; g++) s += sm[g * pl.d + c];
    partial[((size_t)bh * chunks + blockIdx.x) * pl.d + c] = s;
  }
}

// Sum over the 8 or 16 consecutive lanes that share a row, with data-parallel-primitive lane
// permutations inside a 16-lane row (no LDS traffic): lane pairs (i, i^1), (i, i^2), then i <-> 7-i
// within each half row and i <-> 15-i within the row.  Every lane of the group ends with the total.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
  auto perm = [](float v, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, false));
  };
  x += perm(x, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
  x += perm(x, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
  x += perm(x, std::integral_constant<int, 0x141>{});  // row_half_mirror
  if (LANES == 16) x += perm(x, std::integral_constant<int, 0x140>{});  // row_mirror
  return x;
}

// IN_WAVE: d*elem/16 is 8 or 16, so the lanes of a row sit inside one 16-lane row of a wave.
template <typename T, bool IN_WAVE>
__global__ __launch_bounds__(kThreads) void keydiff_scores(const T* __restrict__ k,
                                                           const float* __restrict__ partial,
                                                           float* __restrict__ scores, Plan pl, int chunks) {
  constexpr int VL = Vec<T>::kLen;
  __shared__ float anchor[256];
  __shared__ float anchor_norm;
  __shared__ float red_dot[kUnroll][kThreads], red_sq[kUnroll][kThreads];
  __shared__ float out[kChunkRows];
  const int bh = blockIdx.y, b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int N = ctx_rows(pl, bh);
  const int row0 = blockIdx.x * kChunkRows;
  if (row0 >= N) return;
  const int tid = threadIdx.x;
  const int tpr = pl.d / VL, rpr = kThreads / tpr;
  const int rr = tid / tpr, col = tid % tpr;

  const unsigned char* base = reinterpret_cast<const unsigned char*>(k + b * pl.ksb + (int64_t)h * pl.ksh) +
                              (size_t)col * 16;
  const size_t pitch = (size_t)pl.kst * sizeof(T);
  const int row_end = min(N, row0 + kChunkRows);
  const int rows_per_iter = kUnroll * rpr;

  // raw 16-byte loads; they are widened to fp32 only when used, which keeps many loads in flight
  // at 4 registers each
  auto load_rows = [&](int it0, uint4 (&x)[kUnroll]) {
#pragma unroll
    for (int u = 0; u < kUnroll; u++) {
      const int row = it0 + u * rpr + rr;
      x[u] = make_uint4(0, 0, 0, 0);
      if (rr < rpr && row < row_end) x[u] = *reinterpret_cast<const uint4*>(base + (size_t)row * pitch);
    }
  };
  uint4 xr[kUnroll];
  if constexpr (IN_WAVE) load_rows(row0, xr);  // in flight while the anchor is rebuilt

  // anchor = (sum of the chunk sums) / N, in chunk order
  for (int c = tid; c < pl.d; c += kThreads) {
    float s = 0.f;
    for (int g = 0; g < chunks; g++) s += partial[((size_t)bh * chunks + g) * pl.d + c];
    anchor[c] = s / (float)N;
  }
  __syncthreads();
  if (tid < 64) {
    float s = 0.f;
    for (int c = tid; c < pl.d; c += 64) s = fmaf(anchor[c], anchor[c], s);
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (tid == 0) anchor_norm = sqrtf(s);
  }
  __syncthreads();
  const float an = anchor_norm;
  float a[VL];
#pragma unroll
  for (int e = 0; e < VL; e++) a[e] = rr < rpr ? anchor[col * VL + e] : 0.f;

  if constexpr (IN_WAVE) {
    // reduce in registers, no barrier; scores are collected in LDS and written as one contiguous run
    for (int it0 = row0; it0 < row_end; it0 += rows_per_iter) {
#pragma unroll
      for (int u = 0; u < kUnroll; u++) {
        float x[VL];
        Vec<T>::unpack(xr[u], x);
        float dot = 0.f, sq = 0.f;
#pragma unroll
        for (int e = 0; e < VL; e++) {
          dot = fmaf(x[e], a[e], dot);
          sq = fmaf(x[e], x[e], sq);
        }
        if (tpr == 16) dot = group_sum<16>(dot), sq = group_sum<16>(sq);
        else dot = group_sum<8>(dot), sq = group_sum<8>(sq);
        const int row = it0 + u * rpr + rr;
        if (col == 0 && row < row_end) {
          const float den = sqrtf(sq) * an;
          out[row - row0] = den > 0.f ? -dot / den : 0.f;
        }
        // refill this slot for the next iteration as soon as it has been consumed
        const int nrow = row + rows_per_iter;
        xr[u] = make_uint4(0, 0, 0, 0);
        if (nrow < row_end) xr[u] = *reinterpret_cast<const uint4*>(base + (size_t)nrow * pitch);
      }
    }
    __syncthreads();
    for (int j = tid; j < row_end - row0; j += kThreads) scores[(size_t)bh * pl.N + row0 + j] = out[j];
  } else {
    for (int it0 = row0; it0 < row_end; it0 += rows_per_iter) {
      float x[kUnroll][VL];  // all loads of the iteration are issued before the first use
#pragma unroll
      for (int u = 0; u < kUnroll; u++) {
        const int row = it0 + u * rpr + rr;
        if (rr < rpr && row < row_end) {
          Vec<T>::load(base + (size_t)row * pitch, x[u]);
        } else {
#pragma unroll
          for (int e = 0; e < VL; e++) x[u][e] = 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < kUnroll; u++) {
        float dot = 0.f, sq = 0.f;
#pragma unroll
        for (int e = 0; e < VL; e++) {
          dot = fmaf(x[u][e], a[e], dot);
          sq = fmaf(x[u][e], x[u][e], sq);
        }
        red_dot[u][tid] = dot;
        red_sq[u][tid] = sq;
      }
      __syncthreads();
      for (int j = tid; j < rows_per_iter; j += kThreads) {  // j-th row of this iteration
        const int u = j / rpr, g = j % rpr;
        const int row = it0 + j;
        if (row < row_end) {
          float dot = 0.f, sq = 0.f;
          for (int c = 0; c < tpr; c++) {
            dot += red_dot[u][g * tpr + c];
            sq += red_sq[u][g * tpr + c];
          }
          const float den = sqrtf(sq) * an;
          scores[(size_t)bh * pl.N + row] = den > 0.f ? -dot / den : 0.f;
        }
      }
      __syncthreads();  // the exchange buffers are rewritten by the next iteration
    }
  }
}

template <typename T>
hipError_t launch_t(const Plan& pl, const T* k, float* scores, float* partial, hipStream_t stream) {
  const int chunks = (pl.N + kChunkRows - 1) / kChunkRows;
  dim3 grid(chunks, pl.nb * pl.Hkv);
  hipLaunchKernelGGL(keydiff_partial<T>, grid, dim3(kThreads), 0, stream, k, partial, pl, chunks);
  const int tpr = pl.d / Vec<T>::kLen;
  if (tpr == 16 || tpr == 8)
    hipLaunchKernelGGL((keydiff_scores<T, true>), grid, dim3(kThreads), 0, stream, k, partial, scores, pl, chunks);
  else
    hipLaunchKernelGGL((keydiff_scores<T, false>), grid, dim3(kThreads), 0, stream, k, partial, scores, pl, chunks);
  return hipGetLastError();
}

}  // namespace

size_t keydiff_workspace_bytes(const Plan& pl) {
  const size_t chunks = (pl.N + kChunkRows - 1) / kChunkRows;
  return (size_t)pl.nb * pl.Hkv * chunks * pl.d * sizeof(float);
}

hipError_t launch_score_keydiff(const Plan& pl, const void* k, float* scores, void* workspace,
                                hipStream_t stream) {
  float* partial = static_cast<float*>(workspace);
  if (pl.dtype == EPICACHE_DTYPE_F32) return launch_t<float>(pl, static_cast<const float*>(k), scores, partial, stream);
  return launch_t<__hip_bfloat16>(pl, static_cast<const __hip_bfloat16*>(k), scores, partial, stream);
}

}  // namespace epicache
