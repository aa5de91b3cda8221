// Retention on ragged batches: every (batch item, KV head) has its own number of scored rows and
// every batch item its own budget, both read from device memory.
//
// Two rules (paper Sec. 3.1 Stage 2 for the first; App. A.2, last paragraph, for the second):
//   per head: head (b, h) keeps its min(M_b, n) best rows;
//   pooled:   the heads of item b form one pool whose min(Hkv * M_b, total) best entries are kept,
//             ties to the lower head, then to the lower row, so heads end up with different counts.
//
// Kernel 1 (one workgroup per head, or per item when pooled) finds the score threshold with a
// four-digit radix select over its pool, then counts, per head, the rows above the threshold and
// the rows equal to it, and hands every head its share of the ties in pool order.  It leaves one
// record per head: the threshold key, the number of ties kept, and the head's kept-row count.
// Kernel 2 (one workgroup per head) walks the head's row in index order and writes the kept
// indices ascending, exactly as the uniform selection does.
#include "epicache_internal.h"
#include "select_util.h"

namespace epicache {
namespace {

constexpr int kMaxPooledHeads = 1024;

struct HeadRecord {
  uint32_t thr;   // order key of the threshold score
  int32_t ties;   // rows equal to the threshold that are kept, lowest index first; -1: keep every row
};

__device__ __forceinline__ int item_budget(const Plan& pl, const int32_t* budgets, int b) {
  if (!budgets) return pl.M;
  const int m = budgets[b];
  return m < 1 ? 1 : (m > pl.M ? pl.M : m);
}

template <bool POOLED>
__global__ __launch_bounds__(1024) void ragged_threshold(const float* __restrict__ scores,
                                                         const int32_t* __restrict__ budgets,
                                                         HeadRecord* __restrict__ rec,
                                                         int32_t* __restrict__ n_kept, Plan pl) {
  constexpr int kSeg = POOLED ? kMaxPooledHeads : 1;
  __shared__ uint32_t hist_rep[256 * kHistCopies];  // one digit's histogram, every bin once per LDS bank
  __shared__ uint32_t hist[256];
  __shared__ int seg_len[kSeg];
  __shared__ uint32_t seg_gt[kSeg], seg_eq[kSeg];
  __shared__ unsigned long long pool_total;
  const int tid = threadIdx.x, lane = tid & 63;
  const int b = POOLED ? blockIdx.x : blockIdx.x / pl.Hkv;
  const int h_first = POOLED ? 0 : blockIdx.x % pl.Hkv;
  const int nh = POOLED ? pl.Hkv : 1;
  const int bh_first = b * pl.Hkv + h_first;
  const int M = item_budget(pl, budgets, b);

  if (tid == 0) pool_total = 0;
  for (int i = tid; i < 256 * kHistCopies; i += blockDim.x) hist_rep[i] = 0;
  __syncthreads();
  for (int s = tid; s < nh; s += blockDim.x) {
    const int n = ctx_rows(pl, bh_first + s);
    seg_len[s] = n;
    seg_gt[s] = 0;
    seg_eq[s] = 0;
    atomicAdd(&pool_total, (unsigned long long)n);
  }
  __syncthreads();
  const unsigned long long total = pool_total;
  const unsigned long long want = (unsigned long long)nh * (unsigned long long)M;
  if (want >= total) {  // everything fits: no head loses a row
    for (int s = tid; s < nh; s += blockDim.x) {
      rec[bh_first + s] = HeadRecord{0u, -1};
      n_kept[bh_first + s] = seg_len[s];
    }
    return;
  }

  // radix select of the want-th largest key of the pool, most significant digit first
  uint32_t prefix = 0, mask = 0;
  uint32_t kth = (uint32_t)want;  // < total < 2^31
#pragma unroll 1
  for (int pass = 0; pass < 4; pass++) {
    const int shift = 24 - 8 * pass;
    for (int s = 0; s < nh; s++) {
      const float* row = scores + (size_t)(bh_first + s) * pl.N;
      const int n = seg_len[s];
      for (int i = tid; i < n; i += blockDim.x) {
        const uint32_t key = order_key(row[i]);
        if ((key & mask) == prefix) hist_count(hist_rep, (key >> shift) & 255u, lane);
      }
    }
    __syncthreads();
    hist_fold(hist_rep, hist, tid);
    __syncthreads();
    uint32_t bin, above;
    locate_digit(hist, kth, lane, bin, above);
    prefix |= bin << shift;
    mask |= 255u << shift;
    kth -= above;
  }
  const uint32_t thr = prefix;
  const uint32_t need_eq = kth;  // ties kept over the whole pool, >= 1

  // per head: rows above the threshold and rows equal to it
  for (int s = 0; s < nh; s++) {
    const float* row = scores + (size_t)(bh_first + s) * pl.N;
    const int n = seg_len[s];
    uint32_t cgt = 0, ceq = 0;
    for (int i0 = tid - lane; i0 < n; i0 += blockDim.x) {  // whole waves stay in the loop for the ballots
      const int i = i0 + lane;
      const bool valid = i < n;
      const uint32_t key = valid ? order_key(row[i]) : 0u;
      cgt += __popcll(__ballot(valid && key > thr));
      ceq += __popcll(__ballot(valid && key == thr));
    }
    if (lane == 0) {
      if (cgt) atomicAdd(&seg_gt[s], cgt);
      if (ceq) atomicAdd(&seg_eq[s], ceq);
    }
  }
  __syncthreads();
  if (tid == 0) {  // ties are handed out in pool order: head 0 first
    uint32_t left = need_eq;
    for (int s = 0; s < nh; s++) {
      const uint32_t take = seg_eq[s] < left ? seg_eq[s] : left;
      left -= take;
      rec[bh_first + s] = HeadRecord{thr, (int32_t)take};
      n_kept[bh_first + s] = (int32_t)(seg_gt[s] + take);
    }
  }
}

__global__ __launch_bounds__(1024) void ragged_emit(const float* __restrict__ scores,
                                                    const HeadRecord* __restrict__ rec,
                                                    int32_t* __restrict__ keep, Plan pl) {
  __shared__ uint32_t wave_gt[16], wave_eq[16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nwaves = blockDim.x >> 6;
  const int bh = blockIdx.x;
  const int N = ctx_rows(pl, bh);
  const float* row = scores + (size_t)bh * pl.N;
  int32_t* out = keep + (size_t)bh * pl.keep_stride;
  const HeadRecord r = rec[bh];
  if (r.ties < 0) {  // nothing evicted from this head
    const int n = N < pl.keep_stride ? N : pl.keep_stride;
    for (int i = tid; i < n; i += blockDim.x) out[i] = i;
    return;
  }
  const uint32_t thr = r.thr, need_eq = (uint32_t)r.ties;
  const int cap = pl.keep_stride;

  // every wave owns a contiguous segment of the row, walked 64 rows at a time
  const int groups = (N + nwaves * 64 - 1) / (nwaves * 64);
  const int base = wave * groups * 64 + lane;
  uint32_t cgt = 0, ceq = 0;
  for (int j = 0; j < groups; j++) {
    const int i = base + j * 64;
    const bool valid = i < N;
    const uint32_t key = valid ? order_key(row[i]) : 0u;
    cgt += __popcll(__ballot(valid && key > thr));
    ceq += __popcll(__ballot(valid && key == thr));
  }
  if (lane == 0) wave_gt[wave] = cgt, wave_eq[wave] = ceq;
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; w++) gt_before += wave_gt[w], eq_before += wave_eq[w];
  for (int j = 0; j < groups; j++) {
    const int i = base + j * 64;
    const bool valid = i < N;
    const uint32_t key = valid ? order_key(row[i]) : 0u;
    const bool is_gt = valid && key > thr, is_eq = valid && key == thr;
    const uint64_t bgt = __ballot(is_gt), beq = __ballot(is_eq);
    const uint32_t my_gt = gt_before + lanes_below(bgt);
    const uint32_t my_eq = eq_before + lanes_below(beq);
    if (is_gt || (is_eq && my_eq < need_eq)) {
      const uint32_t pos = my_gt + min(my_eq, need_eq);
      if (pos < (uint32_t)cap) out[pos] = i;  // always true for records kernel 1 wrote for these scores
    }
    gt_before += __popcll(bgt);
    eq_before += __popcll(beq);
  }
}

}  // namespace

size_t select_ragged_record_bytes(const Plan& pl) { return (size_t)pl.nb * pl.Hkv * sizeof(HeadRecord); }

hipError_t launch_select_ragged(const Plan& pl, int select, const float* scores, const int32_t* budgets,
                                int32_t* keep, int32_t* n_kept, void* records, hipStream_t stream) {
  HeadRecord* rec = static_cast<HeadRecord*>(records);
  const int nbh = pl.nb * pl.Hkv;
  if (select == EPICACHE_SELECT_POOLED) {
    if (pl.Hkv > kMaxPooledHeads) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ragged_threshold<true>, dim3(pl.nb), dim3(1024), 0, stream, scores, budgets, rec,
                       n_kept, pl);
  } else {
    const int threads = pl.N <= 4096 ? 256 : pl.N <= 16384 ? 512 : 1024;
    hipLaunchKernelGGL(ragged_threshold<false>, dim3(nbh), dim3(threads), 0, stream, scores, budgets, rec,
                       n_kept, pl);
  }
  const int threads = pl.N <= 8192 ? 256 : 1024;
  hipLaunchKernelGGL(ragged_emit, dim3(nbh), dim3(threads), 0, stream, scores, rec, keep, pl);
  return hipGetLastError();
}

}  // namespace epicache
