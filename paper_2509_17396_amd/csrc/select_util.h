// Device helpers shared by the selection kernels (uniform top-M and ragged / pooled selection).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace epicache {

// Unsigned key whose integer order is the IEEE-754 total order of the float.
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Histogram of one radix digit in LDS.  The scores of a row share few values of the leading digits (sign and
// exponent), so with a plain 256-bin array most of a wave's 64 atomics would meet on one address, which LDS
// serialises.  Every bin is therefore kept in kHistCopies copies, one per LDS bank (copy = lane % 32): at most two
// lanes of an instruction meet on an address.  hist_rep holds 256 * kHistCopies counters, all zero before a pass.
constexpr int kHistCopies = 32;

__device__ __forceinline__ void hist_count(uint32_t* hist_rep, uint32_t digit, int lane) {
  atomicAdd(&hist_rep[digit * kHistCopies + (lane & (kHistCopies - 1))], 1u);
}

// Between two workgroup barriers, by every thread of a workgroup of at least 256: thread t < 256 folds the copies
// of bin t into hist[t] (reading them in a rotated order, so the lanes of a wave stay on different banks) and
// clears them for the next pass.
__device__ __forceinline__ void hist_fold(uint32_t* hist_rep, uint32_t* hist, int tid) {
  if (tid < 256) {
    uint32_t sum = 0;
#pragma unroll 8
    for (int c = 0; c < kHistCopies; c++) {
      uint32_t& slot = hist_rep[tid * kHistCopies + ((c + tid) & (kHistCopies - 1))];
      sum += slot;
      slot = 0;
    }
    hist[tid] = sum;
  }
}

// One radix digit of a select: given the 256-bin histogram of the digit among the keys that still
// match the prefix, find the bin that holds the kth largest (kth >= 1 counts from the top) and how
// many keys lie in the bins above it.  Every wave calls this with the same arguments and gets the
// same answer; lane l owns bins 255-4l .. 252-4l.
__device__ __forceinline__ void locate_digit(const uint32_t* hist, uint32_t kth, int lane, uint32_t& bin,
                                             uint32_t& above) {
  uint32_t c[4];
#pragma unroll
  for (int x = 0; x < 4; x++) c[x] = hist[255 - 4 * lane - x];
  const uint32_t mine = c[0] + c[1] + c[2] + c[3];
  uint32_t incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  const uint32_t excl = incl - mine;
  const bool here = excl < kth && kth <= incl;  // true in exactly one lane
  uint32_t b = 0, a = 0;
  if (here) {
    uint32_t run = excl;
#pragma unroll
    for (int x = 0; x < 4; x++) {
      if (run < kth && kth <= run + c[x]) {
        b = 255 - 4 * lane - x;
        a = run;
      }
      run += c[x];
    }
  }
  const uint64_t who = __ballot(here);
  const int src = __ffsll((unsigned long long)who) - 1;
  bin = __shfl(b, src);
  above = __shfl(a, src);
}

}  // namespace epicache
