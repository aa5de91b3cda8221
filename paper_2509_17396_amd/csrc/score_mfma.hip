// bf16 MFMA scoring kernels for gfx950 (head_dim 64 or 128).
//
// Eq. 1 needs every row's softmax normaliser over all N context keys before a
// single column value is final, and the R x N logits of one KV head do not fit
// on chip, so Q.K^T is evaluated twice:
//   pass 1 (score_stats):  per query row, a reference logit (the maximum, or a value
//                          within 2^60 in weight of it) and the sum of exp2 relative
//                          to it over the keys of one key split -> stats[bh][split][row]
//   pass 2 (score_reduce): per context key, reduce exp2(logit - lse_row) over
//                          all R = G*p rows (max or sum) -> scores[bh][key]
// Both use v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  The operand order
// is chosen so that the axis being reduced lies inside a lane's 16 accumulator
// values: pass 1 puts the keys on the MFMA row axis (a lane owns one query
// column and 16 keys), pass 2 puts the query rows there (a lane owns one key
// column and 16 query rows).  Only two lanes (l, l^32) ever need to be combined.
//
// Both passes are bound by the plain ALUs, not by the matrix cores: per logit
// the softmax costs a multiply-add, an exponential (half rate) and an add or
// max, about 4 issue slots, against 2 slots' worth of MFMA time.  Each wave
// therefore software-pipelines by hand: the MFMA chain of tile u+1 is issued
// one instruction at a time between slices of the softmax arithmetic of tile u.
//
// Accumulator layout of the 32x32 MFMA: lane l, value v holds
//   row = (v / 4) * 8 + (l / 32) * 4 + (v % 4),  column = l % 32.
// The contraction index a lane feeds is the same for the A and the B operand
// (16-byte chunk 2*j + l/32 of the head_dim row for MFMA j), which is all the
// hardware needs for a correct dot product.
//
// Staging: 64-row tiles (keys in pass 1, query rows in pass 2) go from global
// memory straight into LDS with global_load_lds_dwordx4 (lane l of a wave fills
// 16-byte slot l of a 1 KiB slab).  Each lane picks the global chunk that makes
// the LDS image XOR-swizzled, so the ds_read_b128 of the MFMA operands is free
// of bank conflicts without padding.
#include "epicache_internal.h"
#include "mfma_tiles.h"

namespace epicache {
namespace {

// ------------------------------------------------------------------ pass 1
// Softmax statistics of the previous accumulator tile, cut into slices that are
// issued between the MFMAs of the next tile.  16 values = 16 keys of one query row.
//
// Sentinels instead of infinities, so that no inf - inf can arise: a row that has
// seen no key yet has m = kNoMax; masked keys and the filler tile that precedes the
// first real one hold kMasked < kNoMax, so folding them in leaves (m, D) untouched
// (their exp2 underflows to exactly 0 and the max does not move).  Raw dot products
// are assumed to lie above kNoMax (-1e30).
struct RowStat {
  float m, D;  // reference (a raw dot product at or below the running maximum); running sum of exp2((dot - m) * c2)
};

__device__ __forceinline__ void stats_begin(const f32x16& P, const RowStat& st, float c2, float& mn,
                                            float& nmc, float& corr) {
  const float a0 = max3(P[0], P[1], P[2]), a1 = max3(P[3], P[4], P[5]), a2 = max3(P[6], P[7], P[8]);
  const float a3 = max3(P[9], P[10], P[11]), a4 = max3(P[12], P[13], P[14]);
  mn = max3(max3(a0, a1, a2), max3(a3, a4, P[15]), st.m);
  nmc = -mn * c2;
  corr = ex2((st.m - mn) * c2);  // exactly 1 when the max did not move
}

// Which accumulator values enter the arithmetic pipeline in each MFMA slot of a unit.  Independent vector
// instructions issue in the shadow of an MFMA, so the softmax arithmetic is spread evenly over the KS slots;
// and because dependent VALU / transcendental ops have several clocks of latency, it is staggered: the
// values that get their multiply-add in slot j get their exp2 in slot j+1 and are summed in slot j+2, so
// the instructions inside one slot never wait on each other.
template <int KS> struct Slots;
template <> struct Slots<8> {
  static constexpr int reduce[9] = {0, 2, 4, 6, 8, 10, 12, 14, 16};
};
template <> struct Slots<4> {
  static constexpr int reduce[5] = {0, 4, 8, 12, 16};
};

// pipeline stages over the value range [LO, HI); each pins its results at the point of issue
template <int LO, int HI>
__device__ __forceinline__ void stage_exp(float (&x)[16]) {
#pragma unroll
  for (int v = LO; v < HI; v++) x[v] = ex2(x[v]);
#pragma unroll
  for (int v = LO; v < HI; v++) pin(x[v]);
}
template <int LO, int HI>
__device__ __forceinline__ void stage_add(const float (&x)[16], float& s0, float& s1) {
#pragma unroll
  for (int v = LO; v < HI; v++) {
    if (v & 1) s1 += x[v]; else s0 += x[v];
  }
  if (HI > LO) pin(s0), pin(s1);
}
template <int LO, int HI>
__device__ __forceinline__ void stage_max(const float (&x)[16], float& s0, float& s1) {
#pragma unroll
  for (int v = LO; v < HI; v += 2) {  // two values per instruction, alternating between the two chains
    float& s = ((v - LO) & 2) ? s1 : s0;
    if (v + 1 < HI) s = vmax3(s, x[v], x[v + 1]);
    else s = vmax(s, x[v]);
  }
  if (HI > LO) pin(s0), pin(s1);
}

template <int LO, int HI>
__device__ __forceinline__ void stats_stage_fma(float (&x)[16], const f32x16& P, float c2, float nmc) {
#pragma unroll
  for (int v = LO; v < HI; v++) x[v] = fmaf(P[v], c2, nmc);
#pragma unroll
  for (int v = LO; v < HI; v++) pin(x[v]);
}

__device__ __forceinline__ float stats_group(const f32x16& P, int g, float c2, float nmc) {
  const float e0 = ex2(fmaf(P[4 * g + 0], c2, nmc)), e1 = ex2(fmaf(P[4 * g + 1], c2, nmc));
  const float e2 = ex2(fmaf(P[4 * g + 2], c2, nmc)), e3 = ex2(fmaf(P[4 * g + 3], c2, nmc));
  return (e0 + e1) + (e2 + e3);
}

// acc <- MFMA chain over head_dim (A rows = a-frag rows, B columns = b-frag rows), interleaved
// with folding P, the tile finished one unit earlier, into its row statistics.
// The reference st.m of a row only has to keep the exponentials in range, so the fast path does not look
// for the tile's maximum at all (12 of ~62 instructions per unit): it sums exp2((dot - st.m) * c2) as is and
// checks the sum.  A sum beyond kRebase (a dot product more than ~60 / c2 above the reference, or a row
// that has no reference yet: st.m = kNoMax sends every real dot product to +inf) takes the exact path
// below, which moves the reference to the true maximum.  Wave-uniform branch, taken for the first tile of
// a row and then only when the logits climb by a factor of 2^60 in weight.
constexpr float kRebase = 1.0e18f;

template <int KS, int J>
__device__ __forceinline__ void stats_slot(f32x16& acc, const bf16x8 (&a)[KS], const bf16x8 (&b)[KS],
                                           const f32x16& P, float c2, float nmc, float (&x)[16], float& s0,
                                           float& s1) {
  using SL = Slots<KS>;
  const f32x16 zero = {0};
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[J], b[J], J == 0 ? zero : acc, 0, 0, 0);
  fence_sched();
  stats_stage_fma<SL::reduce[J], SL::reduce[J + 1]>(x, P, c2, nmc);
  if constexpr (J >= 1) stage_exp<SL::reduce[J - 1], SL::reduce[J]>(x);
  if constexpr (J >= 2) stage_add<SL::reduce[J - 2], SL::reduce[J - 1]>(x, s0, s1);
  fence_sched();
}

__device__ __forceinline__ void stats_fold(const f32x16& P, RowStat& st, float c2);

// DEFER: the sum is taken as it is and only its running maximum over several units is kept in `worst`; the
// caller checks that once per key tile and, if it ever exceeded kRebase, redoes those units on the exact path.
template <int KS, bool DEFER = false>
__device__ __forceinline__ void stats_unit(f32x16& acc, const bf16x8 (&a)[KS], const bf16x8 (&b)[KS],
                                           const f32x16& P, RowStat& st, float c2, float* worst = nullptr) {
  using SL = Slots<KS>;
  float s0 = 0.f, s1 = 0.f, x[16];
  const float nmc = -st.m * c2;
  stats_slot<KS, 0>(acc, a, b, P, c2, nmc, x, s0, s1);
  stats_slot<KS, 1>(acc, a, b, P, c2, nmc, x, s0, s1);
  stats_slot<KS, 2>(acc, a, b, P, c2, nmc, x, s0, s1);
  stats_slot<KS, 3>(acc, a, b, P, c2, nmc, x, s0, s1);
  if constexpr (KS == 8) {
    stats_slot<KS, 4>(acc, a, b, P, c2, nmc, x, s0, s1);
    stats_slot<KS, 5>(acc, a, b, P, c2, nmc, x, s0, s1);
    stats_slot<KS, 6>(acc, a, b, P, c2, nmc, x, s0, s1);
    stats_slot<KS, 7>(acc, a, b, P, c2, nmc, x, s0, s1);
  }
  // drain the pipeline: last exp2 stage, last two sum stages
  stage_exp<SL::reduce[KS - 1], SL::reduce[KS]>(x);
  stage_add<SL::reduce[KS - 2], SL::reduce[KS - 1]>(x, s0, s1);
  stage_add<SL::reduce[KS - 1], SL::reduce[KS]>(x, s0, s1);
  const float D = st.D + (s0 + s1);
  if constexpr (DEFER) {
    st.D = D;  // +inf at worst (a row without a reference, or a logit 2^60 in weight above it): never NaN
    *worst = fmaxf(*worst, D);
  } else {
    if (__any(!(D <= kRebase))) stats_fold(P, st, c2);  // some row needs a new reference: exact path for the wave
    else st.D = D;
  }
  fence_sched();
}

// fold one finished tile into its row statistics, nothing to overlap with
__device__ __forceinline__ void stats_fold(const f32x16& P, RowStat& st, float c2) {
  float mn, nmc, corr;
  stats_begin(P, st, c2, mn, nmc, corr);
  const float s = (stats_group(P, 0, c2, nmc) + stats_group(P, 1, c2, nmc)) +
                  (stats_group(P, 2, c2, nmc) + stats_group(P, 3, c2, nmc));
  st.D = fmaf(st.D, corr, s);
  st.m = mn;
}

// NQ 32-row query sub-tiles per wave, NW waves per workgroup: 32*NQ*NW query rows per workgroup.
template <int HD, int NQ, int NW>
__global__ __launch_bounds__(NW * 64, (NW == 1 ? 1 : 2)) void score_stats(const bf16_t* __restrict__ q,
                                                          const bf16_t* __restrict__ k,
                                                          float2* __restrict__ stats, Plan pl) {
  using TL = Tile<HD>;
  using ST = Stager<HD, NW>;
  constexpr int KS = TL::kSteps;
  // the per-unit check of the running sums is deferred to once per tile where the registers allow it (the
  // three-sub-tile form sits at the 256-register limit as it is)
  constexpr bool kDeferCheck = NQ <= 2;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * TL::kTileBytes];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  // Workgroups are handed to the 8 XCDs round-robin by linear id.  The key splits (and row blocks) of one
  // (b, h) read the same query rows, so they are given ids that land on one XCD and share its L2:
  // id = xcd + 8 * (rb + RB * (split + S * (bh / 8))), bh % 8 = xcd.
  const int n_rb = (pl.R + 32 * NQ * NW - 1) / (32 * NQ * NW);
  const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
  const int rb = within % n_rb, split = (within / n_rb) % pl.n_splits;  // row blocks of a split side by side: one K fetch
  const int bh = (within / (pl.n_splits * n_rb)) * 8 + xcd;
  if (bh >= pl.nb * pl.Hkv) return;
  const int b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int row0 = rb * (32 * NQ * NW) + wave * (32 * NQ);
  const bool active = row0 < pl.R;  // waves without rows only help staging the key tiles
  const float c2 = pl.c2;

  const int N = ctx_rows(pl, bh);
  const int tiles = (N + kKeyTile - 1) / kKeyTile;
  const int t_begin = split * pl.tiles_per_split;
  if (t_begin >= tiles) {
    // a head shorter than the batch's longest: this split holds none of its keys and contributes
    // an empty sum under a maximum below every logit
    const int r_end = min(pl.R, (rb + 1) * (32 * NQ * NW));
    for (int r = rb * (32 * NQ * NW) + tid; r < r_end; r += NW * 64)
      stats[((size_t)bh * pl.n_splits + split) * pl.Rpad + r] = make_float2(kMasked, 0.f);
    return;
  }
  const int t_end = min(tiles, t_begin + pl.tiles_per_split);
  // a ragged last tile (N % 64 != 0) is handled after the pipelined loop over full tiles
  const int t_full = (t_end == tiles && N % kKeyTile != 0) ? t_end - 1 : t_end;

  // query fragments stay in registers for the whole key loop
  bf16x8 qf[NQ][KS];
#pragma unroll
  for (int s = 0; s < NQ; s++) {
    const int r = row0 + s * 32 + l32;
    const bool ok = r < pl.R;
    const int rr = ok ? r : 0;
    const bf16_t* qrow = q + b * pl.qsb + (int64_t)(h * pl.G + rr / pl.p) * pl.qsh +
                         (int64_t)(rr % pl.p) * pl.qst + hi * 8;
#pragma unroll
    for (int j = 0; j < KS; j++) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (ok) u = *reinterpret_cast<const uint4*>(qrow + j * 16);
      qf[s][j] = as_frag(u);
    }
  }

  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(k + b * pl.ksb + (int64_t)h * pl.ksh);
  const uint32_t kstride = (uint32_t)pl.kst * 2;
  uint32_t koff[ST::kPer];
  ST::offsets(koff, wave, lane, kstride);

  RowStat st[NQ];
#pragma unroll
  for (int s = 0; s < NQ; s++) st[s].m = kNoMax, st[s].D = 0.f;
  f32x16 accA, accB;
#pragma unroll
  for (int v = 0; v < 16; v++) accA[v] = accB[v] = kMasked;  // the tile "before the first": a no-op

  const uint32_t lds0 = lds_address(lds);
  if (t_begin < t_full) ST::run(lds0, kbase + (size_t)t_begin * kKeyTile * kstride, koff, wave);
  wait_vmem();
  __syncthreads();
  int buf = 0;
  // Units of one tile, in order: (ks, s) for key half ks in {0,1}, query sub-tile s in 0..NQ-1.
  // Unit u accumulates into accA (u even) or accB (u odd) while unit u-1 is folded into the
  // statistics of its query sub-tile.  2*NQ is even, so the parity carries over between tiles.
  for (int t = t_begin; t < t_full; t++) {
    const unsigned char* cur = lds + buf * TL::kTileBytes;
    if (t + 1 < t_full)
      ST::run(lds0 + (buf ^ 1) * TL::kTileBytes, kbase + (size_t)(t + 1) * kKeyTile * kstride, koff, wave);
    if (active) {
      bf16x8 kf[KS];  // one 32-key half at a time, refilled once its last MFMA has been issued
      read_frags<HD>(kf, cur, 0, l32, hi);
      if constexpr (kDeferCheck) {
        // The unit carried over from the previous tile is folded with its check at once (its keys are gone from
        // LDS).  The tile's own units 0 .. 2*NQ-2 are folded unchecked; one look at their largest sum decides
        // whether they are redone, from the row statistics as they were before them, on the exact path.  The
        // tile is still in LDS then, and neither kf nor accA is live any more.
        stats_unit<KS>(accA, kf, qf[0], accB, st[NQ - 1], c2);
        RowStat before[NQ];
#pragma unroll
        for (int s = 0; s < NQ; s++) before[s] = st[s];
        float worst = 0.f;
#pragma unroll
        for (int u = 1; u < 2 * NQ; u++) {
          const int s = u % NQ, sp = (u - 1) % NQ;
          if (u == NQ) read_frags<HD>(kf, cur, 1, l32, hi);
          if (u & 1) stats_unit<KS, true>(accB, kf, qf[s], accA, st[sp], c2, &worst);
          else       stats_unit<KS, true>(accA, kf, qf[s], accB, st[sp], c2, &worst);
        }
        if (__any(!(worst <= kRebase))) {
#pragma unroll
          for (int s = 0; s < NQ; s++) st[s] = before[s];
#pragma unroll
          for (int u = 0; u < 2 * NQ - 1; u++) {
            if (u == 0 || u == NQ) read_frags<HD>(kf, cur, u / NQ, l32, hi);
            mfma_chain<KS>(accA, kf, qf[u % NQ]);
            stats_fold(accA, st[u % NQ], c2);
          }
        }
      } else {
#pragma unroll
        for (int u = 0; u < 2 * NQ; u++) {
          const int s = u % NQ, sp = (u + NQ * 2 - 1) % NQ;
          if (u == NQ) read_frags<HD>(kf, cur, 1, l32, hi);
          if (u & 1) stats_unit<KS>(accB, kf, qf[s], accA, st[sp], c2);
          else       stats_unit<KS>(accA, kf, qf[s], accB, st[sp], c2);
        }
      }
    }
    wait_vmem();
    __syncthreads();
    buf ^= 1;
  }
  if (active) stats_fold(accB, st[NQ - 1], c2);  // last unit in flight (or the filler)

  if (t_full < t_end) {
    // ragged last tile: rows beyond N re-read the last key and are masked out of the statistics
    const int t = t_full;
    const int nrows = N - t * kKeyTile;  // 1..63
    const unsigned char* tile = kbase + (size_t)t * kKeyTile * kstride;
    __syncthreads();  // every wave is done reading both buffers
    ST::run_rows(lds0, wave, lane, [=](int row) { return tile + (size_t)min(row, nrows - 1) * kstride; });
    wait_vmem();
    __syncthreads();
    if (active) {
      for (int ks = 0; ks < 2; ks++) {
        bf16x8 kf[KS];
        read_frags<HD>(kf, lds, ks, l32, hi);
#pragma unroll
        for (int s = 0; s < NQ; s++) {
          f32x16 acc;
          mfma_chain<KS>(acc, kf, qf[s]);
#pragma unroll
          for (int v = 0; v < 16; v++)
            if (ks * 32 + (v >> 2) * 8 + hi * 4 + (v & 3) >= nrows) acc[v] = kMasked;
          stats_fold(acc, st[s], c2);
        }
      }
    }
  }

  if (pl.causal_patch && split == 0) {
    // the patch's own keys follow the context rows; the query of patch token t = r % p sees patch
    // keys 0..t (Sec. 2.3: the patch is appended after the block and attends causally)
    const int ptiles = (pl.p + kKeyTile - 1) / kKeyTile;
    for (int pt = 0; pt < ptiles; pt++) {
      const int nrows = min(kKeyTile, pl.p - pt * kKeyTile);
      const unsigned char* tile = kbase + (size_t)(N + pt * kKeyTile) * kstride;
      __syncthreads();  // every wave is done reading the buffer this tile lands in
      ST::run_rows(lds0, wave, lane, [=](int row) { return tile + (size_t)min(row, nrows - 1) * kstride; });
      wait_vmem();
      __syncthreads();
      if (active) {
        for (int ks = 0; ks < 2; ks++) {
          bf16x8 kf[KS];
          read_frags<HD>(kf, lds, ks, l32, hi);
#pragma unroll
          for (int s = 0; s < NQ; s++) {
            const int t_row = (row0 + s * 32 + l32) % pl.p;
            f32x16 acc;
            mfma_chain<KS>(acc, kf, qf[s]);
#pragma unroll
            for (int v = 0; v < 16; v++)
              if (pt * kKeyTile + ks * 32 + (v >> 2) * 8 + hi * 4 + (v & 3) > t_row) acc[v] = kMasked;
            stats_fold(acc, st[s], c2);
          }
        }
      }
    }
  }

  if (!active) return;
#pragma unroll
  for (int s = 0; s < NQ; s++) {
    // lanes l and l^32 hold the same query row over disjoint keys
    const float mo = __shfl_xor(st[s].m, 32), Do = __shfl_xor(st[s].D, 32);
    const float mn = fmaxf(st[s].m, mo);
    const float Dn = st[s].D * ex2((st[s].m - mn) * c2) + Do * ex2((mo - mn) * c2);
    const int r = row0 + s * 32 + l32;
    if (hi == 0 && r < pl.R)
      stats[((size_t)bh * pl.n_splits + split) * pl.Rpad + r] = make_float2(mn * c2, Dn);
  }
}

// ------------------------------------------------------- between the passes
// The key splits of pass 1 become one number per scoring row: minus the base-2 log-sum-exp, which is what pass 2
// adds to every scaled logit.  Done once per row here, not once per workgroup of pass 2: a head has up to a
// hundred such workgroups, and a dependent chain of small loads at the start of each cost them a fifth of their
// lifetime.  Rows beyond R get -inf (weight 0).
__global__ void combine_row_stats(const float2* __restrict__ stats, float* __restrict__ nlse, int n_splits,
                                  int R, int Rpad, size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const size_t bh = i / Rpad;
  const int r = (int)(i % Rpad);
  float val = -INFINITY;
  if (r < R) {
    const float2* st = stats + bh * n_splits * Rpad + r;
    float mx = st[0].x;
    for (int s = 1; s < n_splits; s++) mx = fmaxf(mx, st[(size_t)s * Rpad].x);
    float den = 0.f;
    for (int s = 0; s < n_splits; s++) {
      const float2 e = st[(size_t)s * Rpad];
      den += e.y * ex2(e.x - mx);
    }
    val = -(mx + __log2f(den));
  }
  nlse[i] = val;
}

// ------------------------------------------------------------------ pass 2
// Column reduction of the previous accumulator tile (16 query rows of one key),
// sliced like the statistics above.  nl[v] = -(base-2 lse) of the value's row.
template <int REDUCE>
__device__ __forceinline__ float col_group(const f32x16& P, const float (&nl)[16], int g, float c2) {
  const float x0 = fmaf(P[4 * g + 0], c2, nl[4 * g + 0]), x1 = fmaf(P[4 * g + 1], c2, nl[4 * g + 1]);
  const float x2 = fmaf(P[4 * g + 2], c2, nl[4 * g + 2]), x3 = fmaf(P[4 * g + 3], c2, nl[4 * g + 3]);
  if (REDUCE == EPICACHE_REDUCE_MAX) return vmax(vmax3(x0, x1, x2), x3);
  return (ex2(x0) + ex2(x1)) + (ex2(x2) + ex2(x3));
}

template <int REDUCE>
__device__ __forceinline__ float col_merge(float col, float a, float b, float c, float d) {
  if (REDUCE == EPICACHE_REDUCE_MAX) return vmax3(vmax3(a, b, c), d, col);
  return col + ((a + b) + (c + d));
}

template <int LO, int HI>
__device__ __forceinline__ void col_stage_fma(float (&x)[16], const f32x16& P, const float (&nl)[16], float c2) {
#pragma unroll
  for (int v = LO; v < HI; v++) x[v] = fmaf(P[v], c2, nl[v]);
#pragma unroll
  for (int v = LO; v < HI; v++) pin(x[v]);
}

template <int KS, int REDUCE, int J>
__device__ __forceinline__ void reduce_slot(f32x16& acc, const bf16x8 (&a)[KS], const bf16x8 (&b)[KS],
                                            const f32x16& P, const float (&nl)[16], float c2, float (&x)[16],
                                            float& s0, float& s1) {
  using SL = Slots<KS>;
  const f32x16 zero = {0};
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[J], b[J], J == 0 ? zero : acc, 0, 0, 0);
  fence_sched();
  col_stage_fma<SL::reduce[J], SL::reduce[J + 1]>(x, P, nl, c2);
  if constexpr (REDUCE == EPICACHE_REDUCE_MAX) {
    if constexpr (J >= 1) stage_max<SL::reduce[J - 1], SL::reduce[J]>(x, s0, s1);
  } else {
    if constexpr (J >= 1) stage_exp<SL::reduce[J - 1], SL::reduce[J]>(x);
    if constexpr (J >= 2) stage_add<SL::reduce[J - 2], SL::reduce[J - 1]>(x, s0, s1);
  }
  fence_sched();
}

// acc <- MFMA chain, interleaved with reducing P (the tile finished one unit earlier; nl = minus the
// base-2 log-sum-exp of each of its 16 rows) into `col`.
template <int KS, int REDUCE>
__device__ __forceinline__ void reduce_unit(f32x16& acc, const bf16x8 (&a)[KS], const bf16x8 (&b)[KS],
                                            const f32x16& P, const float (&nl)[16], float& col, float c2) {
  using SL = Slots<KS>;
  float x[16];
  float s0 = REDUCE == EPICACHE_REDUCE_MAX ? -INFINITY : 0.f, s1 = s0;
  reduce_slot<KS, REDUCE, 0>(acc, a, b, P, nl, c2, x, s0, s1);
  reduce_slot<KS, REDUCE, 1>(acc, a, b, P, nl, c2, x, s0, s1);
  reduce_slot<KS, REDUCE, 2>(acc, a, b, P, nl, c2, x, s0, s1);
  reduce_slot<KS, REDUCE, 3>(acc, a, b, P, nl, c2, x, s0, s1);
  if constexpr (KS == 8) {
    reduce_slot<KS, REDUCE, 4>(acc, a, b, P, nl, c2, x, s0, s1);
    reduce_slot<KS, REDUCE, 5>(acc, a, b, P, nl, c2, x, s0, s1);
    reduce_slot<KS, REDUCE, 6>(acc, a, b, P, nl, c2, x, s0, s1);
    reduce_slot<KS, REDUCE, 7>(acc, a, b, P, nl, c2, x, s0, s1);
  }
  if constexpr (REDUCE == EPICACHE_REDUCE_MAX) {
    stage_max<SL::reduce[KS - 1], SL::reduce[KS]>(x, s0, s1);
    col = vmax3(col, s0, s1);
  } else {
    stage_exp<SL::reduce[KS - 1], SL::reduce[KS]>(x);
    stage_add<SL::reduce[KS - 2], SL::reduce[KS - 1]>(x, s0, s1);
    stage_add<SL::reduce[KS - 1], SL::reduce[KS]>(x, s0, s1);
    col += s0 + s1;
  }
  fence_sched();
}

__device__ __forceinline__ void read_nlse(float (&nl)[16], const float* nlse, int row0, int hi) {
#pragma unroll
  for (int g4 = 0; g4 < 4; g4++) {
    const float4 x = *reinterpret_cast<const float4*>(nlse + row0 + g4 * 8 + hi * 4);
    nl[g4 * 4 + 0] = x.x, nl[g4 * 4 + 1] = x.y, nl[g4 * 4 + 2] = x.z, nl[g4 * 4 + 3] = x.w;
  }
}

template <int HD, int REDUCE>
__global__ __launch_bounds__(256, 2) void score_reduce(const bf16_t* __restrict__ q,
                                                       const bf16_t* __restrict__ k,
                                                       const float* __restrict__ nlse_rows,
                                                       float* __restrict__ scores, Plan pl) {
  using TL = Tile<HD>;
  constexpr int KS = TL::kSteps;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* lds = smem;                                            // 2 query tiles
  float* nlse = reinterpret_cast<float*>(smem + 2 * TL::kTileBytes);    // [Rpad + 64] minus base-2 lse
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  // XCD-aware ids as in pass 1: the key blocks of one (b, h) all stream the same query rows through LDS
  // and are given ids that land on one XCD: id = xcd + 8 * (key block + NKB * (bh / 8)), bh % 8 = xcd.
  const int n_kb = (pl.N + kKeysPerWG - 1) / kKeysPerWG;
  const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
  const int kb = within % n_kb;
  const int bh = (within / n_kb) * 8 + xcd;
  if (bh >= pl.nb * pl.Hkv) return;
  const int b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int N = ctx_rows(pl, bh);
  if (kb * kKeysPerWG >= N) return;  // a shorter head of a ragged batch: no keys here
  const int key0 = kb * kKeysPerWG + wave * 64;
  const float c2 = pl.c2;

  using ST = Stager<HD, 4>;
  const unsigned char* qbase = reinterpret_cast<const unsigned char*>(q + b * pl.qsb + (int64_t)(h * pl.G) * pl.qsh);
  const size_t qsh = (size_t)pl.qsh * 2;
  const uint32_t qstride = (uint32_t)pl.qst * 2;
  const int p = pl.p, last_row = pl.R - 1;
  const bool dense_tiles = p % 64 == 0;  // every 64-row tile lies inside one query head
  uint32_t qoff[ST::kPer];
  ST::offsets(qoff, wave, lane, qstride);
  const uint32_t lds0 = lds_address(lds);
  // dense tiles are staged in order, so the address of the next one is carried along instead of being derived
  // from the tile index with a division per tile
  const unsigned char* qtile = qbase;  // first row of the next tile to stage
  int qtile_row = 0;                   // that row's index within its query head
  auto stage_queries = [&](uint32_t dst, int t) {
    if (dense_tiles) {
      ST::run(dst, qtile, qoff, wave);
      qtile_row += 64;
      if (qtile_row == p) {
        qtile_row = 0;
        qtile += qsh - (size_t)(p - 64) * qstride;  // first row of the next query head
      } else {
        qtile += (size_t)64 * qstride;
      }
    } else {
      // rows beyond R re-read the last row; their -lse is -inf, so they contribute nothing
      ST::run_rows(dst, wave, lane, [=](int row) {
        const int r = min(t * 64 + row, last_row);
        return qbase + (size_t)(r / p) * qsh + (size_t)(r % p) * qstride;
      });
    }
  };
  stage_queries(lds0, 0);

  // minus the base-2 log-sum-exp of every query row of this head, then 64 rows of -inf (the "tile before the first")
  {
    const float4* src = reinterpret_cast<const float4*>(nlse_rows + (size_t)bh * pl.Rpad);
    for (int r4 = tid; r4 < (pl.Rpad + 64) / 4; r4 += 256)
      reinterpret_cast<float4*>(nlse)[r4] =
          r4 < pl.Rpad / 4 ? src[r4] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  }

  // key fragments of this wave stay in registers for the whole query loop
  const bf16_t* kbase = k + b * pl.ksb + (int64_t)h * pl.ksh;
  bf16x8 kf[2][KS];
#pragma unroll
  for (int s = 0; s < 2; s++) {
    const int key = min(key0 + s * 32 + l32, N - 1);
    const bf16_t* krow = kbase + (int64_t)key * pl.kst + hi * 8;
#pragma unroll
    for (int j = 0; j < KS; j++)
      kf[s][j] = as_frag(*reinterpret_cast<const uint4*>(krow + j * 16));
  }
  // The fragments are used here, i.e. loaded before the wait below.  Left to itself the compiler sinks these
  // loads behind the barrier, finds them outstanding at the loop's entry and puts a counted wait in front of the
  // first use of each inside the loop; from the second iteration on those waits only see the tile in flight and
  // make every wave wait for it a unit and a half after it was requested.
#pragma unroll
  for (int s = 0; s < 2; s++)
#pragma unroll
    for (int j = 0; j < KS; j++) asm volatile("" : "+v"(kf[s][j]));

  // SUM: running sum of weights.  MAX: running max of the base-2 log weight
  // (exp2 is monotone, so one exponential per key at the end is enough).
  float col[2];
  col[0] = col[1] = REDUCE == EPICACHE_REDUCE_MAX ? -INFINITY : 0.f;
  f32x16 accA, accB;
#pragma unroll
  for (int v = 0; v < 16; v++) accA[v] = accB[v] = 0.f;
  // "previous tile" of the very first unit: rows [Rpad, Rpad+64) of nlse are -inf, i.e. a no-op
  float nlP[16], nlC[16];

  wait_vmem();
  __syncthreads();  // query tile 0 and nlse[] are in LDS
  read_nlse(nlP, nlse, pl.Rpad, hi);

  const int qtiles = pl.Rpad / 64;
  int buf = 0;
  // Units of one query tile: (qs, s) for qs in {0,1} (32-row halves), s in {0,1} (key halves of the
  // wave): u = 2*qs + s accumulates into accA (u even) / accB (u odd) while unit u-1 is reduced.
  for (int t = 0; t < qtiles; t++) {
    const unsigned char* cur = lds + buf * TL::kTileBytes;
    if (t + 1 < qtiles) stage_queries(lds0 + (buf ^ 1) * TL::kTileBytes, t + 1);
    bf16x8 qf0[KS], qf1[KS];
    read_frags<HD>(qf0, cur, 0, l32, hi);
    read_frags<HD>(qf1, cur, 1, l32, hi);
    read_nlse(nlC, nlse, t * 64, hi);
    // unit 0: rows qs=0, keys s=0; previous unit = (prev tile, qs=1, s=1) with nlP
    reduce_unit<KS, REDUCE>(accA, qf0, kf[0], accB, nlP, col[1], c2);
    read_nlse(nlP, nlse, t * 64 + 32, hi);
    reduce_unit<KS, REDUCE>(accB, qf0, kf[1], accA, nlC, col[0], c2);
    reduce_unit<KS, REDUCE>(accA, qf1, kf[0], accB, nlC, col[1], c2);
    reduce_unit<KS, REDUCE>(accB, qf1, kf[1], accA, nlP, col[0], c2);
    wait_vmem();
    __syncthreads();
    buf ^= 1;
  }
  {  // drain: last unit (qs=1, s=1) sits in accB with nlP
    const float s0 = col_group<REDUCE>(accB, nlP, 0, c2), s1 = col_group<REDUCE>(accB, nlP, 1, c2);
    const float s2 = col_group<REDUCE>(accB, nlP, 2, c2), s3 = col_group<REDUCE>(accB, nlP, 3, c2);
    col[1] = col_merge<REDUCE>(col[1], s0, s1, s2, s3);
  }

#pragma unroll
  for (int s = 0; s < 2; s++) {
    // lanes l and l^32 hold the same key over disjoint query rows
    const float o = __shfl_xor(col[s], 32);
    float val;
    if (REDUCE == EPICACHE_REDUCE_MAX) val = ex2(fmaxf(col[s], o));
    else val = col[s] + o;
    const int key = key0 + s * 32 + l32;
    if (hi == 0 && key < N) scores[(size_t)bh * pl.N + key] = val;
  }
}

// ------------------------------------------------------- pass 2, streaming form
// For R <= 256 (all query rows of a KV head fit one workgroup): same data flow as pass 1 - query
// fragments stay in registers, 64-key tiles stream through LDS - with the operands swapped so that
// a lane owns one key column and 16 query rows.  Each wave reduces its own rows; the per-key
// partial results of the NW waves meet in LDS once per tile.  Reads K with fully coalesced
// 1 KiB bursts, which the key-stationary form above cannot do when R is small.
template <int KS, int REDUCE>
__device__ __forceinline__ void col_fold(const f32x16& P, const float (&nl)[16], float& col, float c2) {
  const float s0 = col_group<REDUCE>(P, nl, 0, c2), s1 = col_group<REDUCE>(P, nl, 1, c2);
  const float s2 = col_group<REDUCE>(P, nl, 2, c2), s3 = col_group<REDUCE>(P, nl, 3, c2);
  col = col_merge<REDUCE>(col, s0, s1, s2, s3);
}

template <int HD, int NQ, int NW, int REDUCE>
__global__ __launch_bounds__(NW * 64, (NW == 1 ? 1 : 2)) void score_reduce_stream(const bf16_t* __restrict__ q,
                                                                  const bf16_t* __restrict__ k,
                                                                  const float* __restrict__ nlse_rows,
                                                                  float* __restrict__ scores, Plan pl) {
  using TL = Tile<HD>;
  using ST = Stager<HD, NW>;
  constexpr int KS = TL::kSteps;
  constexpr int kRows = 32 * NQ * NW;
  constexpr float kNeutral = REDUCE == EPICACHE_REDUCE_MAX ? -INFINITY : 0.f;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * TL::kTileBytes];
  __shared__ __attribute__((aligned(16))) float nlse[kRows];
  __shared__ float part[2][NW][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int split = blockIdx.x, bh = blockIdx.y;
  const int b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int row0 = wave * (32 * NQ);
  const bool active = row0 < pl.R;
  const float c2 = pl.c2;

  const int N = ctx_rows(pl, bh);
  const int tiles = (N + kKeyTile - 1) / kKeyTile;
  const int t_begin = split * pl.reduce_tiles_per_split;
  const int t_end = min(tiles, t_begin + pl.reduce_tiles_per_split);
  if (t_begin >= t_end) return;  // a shorter head of a ragged batch: no keys in this split

  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(k + b * pl.ksb + (int64_t)h * pl.ksh);
  const uint32_t kstride = (uint32_t)pl.kst * 2;
  uint32_t koff[ST::kPer];
  ST::offsets(koff, wave, lane, kstride);
  const uint32_t lds0 = lds_address(lds);
  auto stage_keys = [&](uint32_t dst, int t) {
    const unsigned char* tile = kbase + (size_t)t * kKeyTile * kstride;
    const int nrows = N - t * kKeyTile;
    if (nrows >= kKeyTile) ST::run(dst, tile, koff, wave);
    else  // ragged last tile: rows beyond N re-read the last key; their results are never written
      ST::run_rows(dst, wave, lane, [=](int row) { return tile + (size_t)min(row, nrows - 1) * kstride; });
  };
  stage_keys(lds0, t_begin);

  // minus the base-2 log-sum-exp of this head's query rows; rows beyond R: weight exp2(-inf) = 0
  for (int r = tid; r < kRows; r += NW * 64)
    nlse[r] = r < pl.Rpad ? nlse_rows[(size_t)bh * pl.Rpad + r] : -INFINITY;

  // query fragments (A operand: rows = queries) stay in registers for the whole key loop
  bf16x8 qf[NQ][KS];
#pragma unroll
  for (int s = 0; s < NQ; s++) {
    const int r = row0 + s * 32 + l32;
    const bool ok = r < pl.R;
    const int rr = ok ? r : 0;
    const bf16_t* qrow = q + b * pl.qsb + (int64_t)(h * pl.G + rr / pl.p) * pl.qsh +
                         (int64_t)(rr % pl.p) * pl.qst + hi * 8;
#pragma unroll
    for (int j = 0; j < KS; j++) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (ok) u = *reinterpret_cast<const uint4*>(qrow + j * 16);
      qf[s][j] = as_frag(u);
    }
  }

  wait_vmem();
  __syncthreads();  // first key tile and nlse[] are in LDS

  // The pipeline runs across tile boundaries: the last unit of tile t-1 (in accB) is reduced while the first
  // chain of tile t is issued, so the column partials of a tile are complete one unit into the next tile and
  // its scores are written one barrier later than its keys were consumed.
  auto exchange = [&](const float (&c)[2], int t) {  // this wave's partials of tile t -> part[t & 1]
#pragma unroll
    for (int ks = 0; ks < 2; ks++) {
      // lanes l and l^32 hold the same key over disjoint query rows; the swap leaves the lower half's values
      // in both halves of one register and the upper half's in both halves of the other (vector ALU, no LDS)
      const unsigned int bits = __float_as_uint(c[ks]);
      const auto r = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
      const float lo = __uint_as_float(r[0]), up = __uint_as_float(r[1]);
      const float v = REDUCE == EPICACHE_REDUCE_MAX ? fmaxf(lo, up) : lo + up;
      if (hi == 0) part[t & 1][wave][ks * 32 + l32] = v;
    }
  };
  auto write_scores = [&](int t) {  // after the barrier that completes part[t & 1]
    if (tid < 64) {
      const int key = t * kKeyTile + tid;
      if (key < N) {
        float v = part[t & 1][0][tid];
#pragma unroll
        for (int w = 1; w < NW; w++)
          v = REDUCE == EPICACHE_REDUCE_MAX ? fmaxf(v, part[t & 1][w][tid]) : v + part[t & 1][w][tid];
        scores[(size_t)bh * pl.N + key] = REDUCE == EPICACHE_REDUCE_MAX ? ex2(v) : v;
      }
    }
  };

  int buf = 0;
  f32x16 accA, accB;                             // accB after a tile: its last unit, still to be reduced
#pragma unroll
  for (int v = 0; v < 16; v++) accB[v] = kMasked;  // before the first tile: a filler whose weights are 0; what it
                                                   // leaves in cs_prev is never exchanged
  float cs_prev[2] = {kNeutral, kNeutral};       // partials of the previous tile (keys ks*32 + l32)
  for (int t = t_begin; t < t_end; t++) {
    const unsigned char* cur = lds + buf * TL::kTileBytes;
    if (t + 1 < t_end) stage_keys(lds0 + (buf ^ 1) * TL::kTileBytes, t + 1);
    float cs[2] = {kNeutral, kNeutral};  // this wave's rows, keys ks*32 + l32 of the tile
    if (active) {
      // units (ks, s): key half ks, query sub-tile s; unit u accumulates into accA/accB (u even/odd)
      // while unit u-1 is reduced over its 16 rows into cs[ks of u-1]
      bf16x8 kf[KS];
      read_frags<HD>(kf, cur, 0, l32, hi);
#pragma unroll
      for (int u = 0; u < 2 * NQ; u++) {
        const int s = u % NQ, sp = (u + 2 * NQ - 1) % NQ, ksp = (u - 1) / NQ;
        if (u == NQ) read_frags<HD>(kf, cur, 1, l32, hi);
        float nl[16];  // minus lse of the 16 rows this lane holds of the previous unit
        read_nlse(nl, nlse, row0 + sp * 32, hi);
        if (u == 0) {
          reduce_unit<KS, REDUCE>(accA, qf[0], kf, accB, nl, cs_prev[1], c2);  // last unit of tile t-1
        } else if (u & 1) {
          reduce_unit<KS, REDUCE>(accB, qf[s], kf, accA, nl, cs[ksp], c2);
        } else {
          reduce_unit<KS, REDUCE>(accA, qf[s], kf, accB, nl, cs[ksp], c2);
        }
      }
    }
    if (t > t_begin) exchange(cs_prev, t - 1);
    wait_vmem();
    __syncthreads();  // tile t+1 staged, part[(t-1) & 1] complete; it is rewritten two barriers from now
    if (t > t_begin) write_scores(t - 1);
    cs_prev[0] = cs[0], cs_prev[1] = cs[1];
    buf ^= 1;
  }
  if (active) {
    float nl[16];
    read_nlse(nl, nlse, row0 + (NQ - 1) * 32, hi);
    col_fold<KS, REDUCE>(accB, nl, cs_prev[1], c2);  // last unit of the last tile: odd index, key half 1
  }
  exchange(cs_prev, t_end - 1);
  __syncthreads();
  write_scores(t_end - 1);
}

template <int HD, int NQ, int NW>
void launch_reduce_stream(const Plan& pl, const bf16_t* q, const bf16_t* k, const float* nlse,
                          float* scores, hipStream_t stream) {
  dim3 grid(pl.reduce_splits, pl.nb * pl.Hkv);
  if (pl.reduce == EPICACHE_REDUCE_MAX)
    hipLaunchKernelGGL((score_reduce_stream<HD, NQ, NW, EPICACHE_REDUCE_MAX>), grid, dim3(NW * 64), 0,
                       stream, q, k, nlse, scores, pl);
  else
    hipLaunchKernelGGL((score_reduce_stream<HD, NQ, NW, EPICACHE_REDUCE_SUM>), grid, dim3(NW * 64), 0,
                       stream, q, k, nlse, scores, pl);
}

template <int HD, int NQ, int NW>
void launch_stats(const Plan& pl, const bf16_t* q, const bf16_t* k, float2* stats, hipStream_t stream) {
  const int rows_per_wg = 32 * NQ * NW;
  const int n_rb = (pl.R + rows_per_wg - 1) / rows_per_wg;
  const int bh8 = (pl.nb * pl.Hkv + 7) / 8 * 8;  // ids whose bh falls beyond the batch exit at once
  dim3 grid((unsigned)(pl.n_splits * n_rb * bh8));
  hipLaunchKernelGGL((score_stats<HD, NQ, NW>), grid, dim3(NW * 64), 0, stream, q, k, stats, pl);
}

template <int HD>
hipError_t launch_hd(const Plan& pl, const bf16_t* q, const bf16_t* k, float* scores,
                     float2* stats, float* nlse, bool stats_ready, hipStream_t stream) {
  using TL = Tile<HD>;
  const int nbh = pl.nb * pl.Hkv;
  if (!stats_ready) switch (pl.stats_rows_per_wg) {
    case 256: launch_stats<HD, 2, 4>(pl, q, k, stats, stream); break;
    case 192: launch_stats<HD, 3, 2>(pl, q, k, stats, stream); break;
    case 128: launch_stats<HD, 1, 4>(pl, q, k, stats, stream); break;
    case 64: launch_stats<HD, 1, 2>(pl, q, k, stats, stream); break;
    default: launch_stats<HD, 1, 1>(pl, q, k, stats, stream); break;
  }
  {
    const size_t total = (size_t)nbh * pl.Rpad;
    hipLaunchKernelGGL(combine_row_stats, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, stats, nlse,
                       pl.n_splits, pl.R, pl.Rpad, total);
  }
  if (pl.R <= pl.stats_rows_per_wg) {
    switch (pl.stats_rows_per_wg) {
      case 256: launch_reduce_stream<HD, 2, 4>(pl, q, k, nlse, scores, stream); break;
      case 192: launch_reduce_stream<HD, 3, 2>(pl, q, k, nlse, scores, stream); break;
      case 128: launch_reduce_stream<HD, 1, 4>(pl, q, k, nlse, scores, stream); break;
      case 64: launch_reduce_stream<HD, 1, 2>(pl, q, k, nlse, scores, stream); break;
      default: launch_reduce_stream<HD, 1, 1>(pl, q, k, nlse, scores, stream); break;
    }
    return hipGetLastError();
  }
  dim3 g2((unsigned)(((pl.N + kKeysPerWG - 1) / kKeysPerWG) * ((nbh + 7) / 8 * 8)));
  const size_t smem = 2 * TL::kTileBytes + (size_t)(pl.Rpad + 64) * sizeof(float);
  auto launch = [&](auto kernel) -> hipError_t {
    if (smem > 64 * 1024) {
      // very long patches: one normaliser per row no longer fits the default 64 KB of dynamic LDS
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, g2, dim3(256), smem, stream, q, k, nlse, scores, pl);
    return hipGetLastError();
  };
  if (pl.reduce == EPICACHE_REDUCE_MAX) return launch(score_reduce<HD, EPICACHE_REDUCE_MAX>);
  return launch(score_reduce<HD, EPICACHE_REDUCE_SUM>);
}

}  // namespace

hipError_t launch_score_mfma(const Plan& pl, const void* q, const void* k, float* scores,
                             float2* stats, float* nlse, bool stats_ready, hipStream_t stream) {
  const bf16_t* qq = static_cast<const bf16_t*>(q);
  const bf16_t* kk = static_cast<const bf16_t*>(k);
  if (pl.d == 128) return launch_hd<128>(pl, qq, kk, scores, stats, nlse, stats_ready, stream);
  if (pl.d == 64) return launch_hd<64>(pl, qq, kk, scores, stats, nlse, stats_ready, stream);
  return hipErrorInvalidValue;
}

}  // namespace epicache
