// Per-(batch item, KV head) top-M selection (the retention rule of paper Sec. 3.1
// Stage 2 / Alg. 1 phase A3) as an exact radix select.
//
// One workgroup owns one score row.  Scores are mapped to unsigned keys whose
// integer order is the float order, the n_keep-th largest key is found with
// four 8-bit histogram passes (most significant byte first), then every wave
// walks its contiguous segment of the row in index order and emits the kept
// indices with ballot + popcount prefix sums: all keys above the threshold,
// plus the first `need_eq` keys equal to it (lower index wins a tie), which
// makes the count exactly n_keep and keeps the output ascending.
#include "epicache_internal.h"
#include "select_util.h"

namespace epicache {
namespace {

// VPT > 0: each thread keeps VPT keys in registers (N <= blockDim.x * VPT).
// VPT == 0: keys are re-read from global memory in every pass (any N).
template <int VPT>
__global__ __launch_bounds__(1024) void topk_select(const float* __restrict__ scores,
                                                    int32_t* __restrict__ keep, int N, int n_keep,
                                                    int pitch) {
  __shared__ uint32_t hist_rep[256 * kHistCopies];  // one digit's histogram, every bin once per LDS bank
  __shared__ uint32_t hist[256];
  __shared__ uint32_t wave_gt[16], wave_eq[16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nwaves = blockDim.x >> 6;
  const float* row = scores + (size_t)blockIdx.x * N;
  int32_t* out = keep + (size_t)blockIdx.x * pitch;  // rows of kept indices are `pitch` apart

  const int groups = VPT > 0 ? VPT : (N + nwaves * 64 - 1) / (nwaves * 64);  // 64-wide groups per wave
  const int base = wave * groups * 64 + lane;

  uint32_t regs[VPT > 0 ? VPT : 1];
  if constexpr (VPT > 0) {
#pragma unroll
    for (int j = 0; j < VPT; j++) {
      const int i = base + j * 64;
      regs[j] = i < N ? order_key(row[i]) : 0u;
    }
  }
  auto key_at = [&](int j) -> uint32_t {
    if constexpr (VPT > 0) return regs[j];
    const int i = base + j * 64;
    return i < N ? order_key(row[i]) : 0u;
  };

  for (int i = tid; i < 256 * kHistCopies; i += blockDim.x) hist_rep[i] = 0;
  __syncthreads();

  uint32_t prefix = 0, mask = 0;
  uint32_t kth = (uint32_t)n_keep;  // rank (1 = largest) still to be located inside the current prefix class
#pragma unroll 1
  for (int pass = 0; pass < 4; pass++) {
    const int shift = 24 - 8 * pass;
    if constexpr (VPT > 0) {
#pragma unroll
      for (int j = 0; j < VPT; j++) {
        const uint32_t key = key_at(j);
        if (base + j * 64 < N && (key & mask) == prefix) hist_count(hist_rep, (key >> shift) & 255u, lane);
      }
    } else {
      for (int j = 0; j < groups; j++) {
        const uint32_t key = key_at(j);
        if (base + j * 64 < N && (key & mask) == prefix) hist_count(hist_rep, (key >> shift) & 255u, lane);
      }
    }
    __syncthreads();
    hist_fold(hist_rep, hist, tid);
    __syncthreads();
    uint32_t bin, above;
    locate_digit(hist, kth, lane, bin, above);  // every wave scans the 256 bins itself
    prefix |= bin << shift;
    mask |= 255u << shift;
    kth -= above;
  }
  const uint32_t thr = prefix;    // key of the n_keep-th largest score
  const uint32_t need_eq = kth;   // how many keys equal to thr are kept (>= 1)

  // per-wave counts, then an exclusive prefix over the waves
  uint32_t cgt = 0, ceq = 0;
  auto count_group = [&](int j) {
    const uint32_t key = key_at(j);
    const bool valid = base + j * 64 < N;
    cgt += __popcll(__ballot(valid && key > thr));
    ceq += __popcll(__ballot(valid && key == thr));
  };
  if constexpr (VPT > 0) {
#pragma unroll
    for (int j = 0; j < VPT; j++) count_group(j);
  } else {
    for (int j = 0; j < groups; j++) count_group(j);
  }
  if (lane == 0) wave_gt[wave] = cgt, wave_eq[wave] = ceq;
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; w++) gt_before += wave_gt[w], eq_before += wave_eq[w];

  auto emit_group = [&](int j) {
    const uint32_t key = key_at(j);
    const int i = base + j * 64;
    const bool valid = i < N;
    const bool is_gt = valid && key > thr, is_eq = valid && key == thr;
    const uint64_t bgt = __ballot(is_gt), beq = __ballot(is_eq);
    const uint32_t my_gt = gt_before + lanes_below(bgt);
    const uint32_t my_eq = eq_before + lanes_below(beq);
    if (is_gt || (is_eq && my_eq < need_eq)) out[my_gt + min(my_eq, need_eq)] = i;
    gt_before += __popcll(bgt);
    eq_before += __popcll(beq);
  };
  if constexpr (VPT > 0) {
#pragma unroll
    for (int j = 0; j < VPT; j++) emit_group(j);
  } else {
    for (int j = 0; j < groups; j++) emit_group(j);
  }
}

__global__ void iota_keep(int32_t* keep, int n_keep, size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) keep[i] = (int32_t)(i % n_keep);
}

// keep[bh][first + j] = row0 + j for j < count: rows that are retained whatever they score
__global__ void append_rows(int32_t* keep, int pitch, int first, int count, int row0, size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) keep[(i / count) * pitch + first + (i % count)] = row0 + (int32_t)(i % count);
}

}  // namespace

hipError_t launch_append_rows(const Plan& pl, int32_t* keep, int first, int count, int row0, hipStream_t stream) {
  const size_t total = (size_t)pl.nb * pl.Hkv * count;
  hipLaunchKernelGGL(append_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, keep,
                     pl.keep_stride, first, count, row0, total);
  return hipGetLastError();
}

hipError_t launch_iota_keep(const Plan& pl, int32_t* keep, hipStream_t stream) {
  const size_t total = (size_t)pl.nb * pl.Hkv * pl.n_keep;
  hipLaunchKernelGGL(iota_keep, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, keep,
                     pl.n_keep, total);
  return hipGetLastError();
}

hipError_t launch_topk(const Plan& pl, const float* scores, int32_t* keep, hipStream_t stream) {
  if (pl.N <= pl.M) return launch_iota_keep(pl, keep, stream);
  const int nbh = pl.nb * pl.Hkv, N = pl.N, nk = pl.n_keep, pitch = pl.keep_stride;
  dim3 grid(nbh);
  if (N <= 1024)
    hipLaunchKernelGGL(topk_select<4>, grid, dim3(256), 0, stream, scores, keep, N, nk, pitch);
  else if (N <= 4096)
    hipLaunchKernelGGL(topk_select<16>, grid, dim3(256), 0, stream, scores, keep, N, nk, pitch);
  else if (N <= 8192)
    hipLaunchKernelGGL(topk_select<16>, grid, dim3(512), 0, stream, scores, keep, N, nk, pitch);
  else if (N <= 16384)
    hipLaunchKernelGGL(topk_select<16>, grid, dim3(1024), 0, stream, scores, keep, N, nk, pitch);
  else if (N <= 32768)
    hipLaunchKernelGGL(topk_select<32>, grid, dim3(1024), 0, stream, scores, keep, N, nk, pitch);
  else
    hipLaunchKernelGGL(topk_select<0>, grid, dim3(1024), 0, stream, scores, keep, N, nk, pitch);
  return hipGetLastError();
}

}  // namespace epicache
