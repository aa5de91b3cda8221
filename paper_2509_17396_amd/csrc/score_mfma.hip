// bf16 MFMA scoring kernels for gfx950 (head_dim 64 or 128).
//
// Eq. 1 needs every row's softmax normaliser over all N context keys before a
// single column value is final, and the R x N logits of one KV head do not fit
// on chip, so Q.K^T is evaluated twice:
//   pass 1 (score_stats):  per query row, running (max, sum of exp2) over the
//                          keys of one key split  -> stats[bh][split][row]
//   pass 2 (score_reduce): per context key, reduce exp2(logit - lse_row) over
//                          all R = G*p rows (max or sum) -> scores[bh][key]
// Both use v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  The operand order
// is chosen so that the axis being reduced lies inside a lane's 16 accumulator
// values: pass 1 puts the keys on the MFMA row axis (a lane owns one query
// column and 16 keys), pass 2 puts the query rows there (a lane owns one key
// column and 16 query rows).  Only two lanes (l, l^32) ever need to be combined.
//
// Accumulator layout of the 32x32 MFMA used throughout: lane l, value v holds
//   row = (v / 4) * 8 + (l / 32) * 4 + (v % 4),  column = l % 32.
// The contraction index each lane feeds is the same for the A and the B
// operand (16-byte chunk 2*j + l/32 of the head_dim row for MFMA j), which is
// all the hardware needs for a correct dot product.
#include "epicache_internal.h"

namespace epicache {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint16_t bf16_t;  // raw storage

__device__ __forceinline__ bf16x8 as_frag(uint4 u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int HD>
struct Tile {
  static constexpr int kSteps = HD / 16;           // MFMAs per 32x32 output tile
  static constexpr int kChunks = HD / 8;           // 16-byte chunks per row
  static constexpr int kRowBytes = HD * 2 + 16;    // LDS row pitch: +16 B keeps ds_read_b128 conflict free
  static constexpr int kTileBytes = 64 * kRowBytes;
  static constexpr int kLoads = 64 * kChunks / 256;  // 16-byte global loads per thread per 64-row tile
};

// ------------------------------------------------------------------ pass 1
template <int HD>
__global__ __launch_bounds__(256, 2) void score_stats(const bf16_t* __restrict__ q,
                                                      const bf16_t* __restrict__ k,
                                                      float2* __restrict__ stats, Plan pl) {
  using TL = Tile<HD>;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * TL::kTileBytes];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, hi = lane >> 5;
  const int split = blockIdx.x, rb = blockIdx.y, bh = blockIdx.z;
  const int b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int row0 = rb * kRowsPerWG + wave * 64;
  const bool active = row0 < pl.R;  // inactive waves only help staging the key tiles

  const int tiles = (pl.N + kKeyTile - 1) / kKeyTile;
  const int t_begin = split * pl.tiles_per_split;
  const int t_end = min(tiles, t_begin + pl.tiles_per_split);

  // query fragments stay in registers for the whole key loop
  bf16x8 qf[2][TL::kSteps];
#pragma unroll
  for (int s = 0; s < 2; s++) {
    const int r = row0 + s * 32 + l32;
    const bool ok = active && r < pl.R;
    const int rr = ok ? r : 0;
    const bf16_t* qrow = q + b * pl.qsb + (int64_t)(h * pl.G + rr / pl.p) * pl.qsh +
                         (int64_t)(rr % pl.p) * pl.qst;
#pragma unroll
    for (int j = 0; j < TL::kSteps; j++) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (ok) u = *reinterpret_cast<const uint4*>(qrow + j * 16 + hi * 8);
      qf[s][j] = as_frag(u);
    }
  }

  const bf16_t* kbase = k + b * pl.ksb + (int64_t)h * pl.ksh;
  uint4 stage[TL::kLoads];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int i = 0; i < TL::kLoads; i++) {
      const int c = tid + i * 256;
      const int row = c / TL::kChunks, ch = c % TL::kChunks;
      const int key = min(t * kKeyTile + row, pl.N - 1);  // tail rows are masked below
      stage[i] = *reinterpret_cast<const uint4*>(kbase + (int64_t)key * pl.kst + ch * 8);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TL::kLoads; i++) {
      const int c = tid + i * 256;
      const int row = c / TL::kChunks, ch = c % TL::kChunks;
      *reinterpret_cast<uint4*>(lds + buf * TL::kTileBytes + row * TL::kRowBytes + ch * 16) = stage[i];
    }
  };

  float m[2] = {-INFINITY, -INFINITY};  // running max of the raw dot products
  float D[2] = {0.f, 0.f};              // running sum of exp2((dot - m) * c2)
  const float c2 = pl.c2;

  if (t_begin < t_end) load_tile(t_begin);
  int buf = 0;
  for (int t = t_begin; t < t_end; t++) {
    store_tile(buf);
    __syncthreads();
    if (t + 1 < t_end) load_tile(t + 1);
    if (active) {
      const bool tail = (t + 1) * kKeyTile > pl.N;
#pragma unroll
      for (int ks = 0; ks < 2; ks++) {
        bf16x8 kf[TL::kSteps];
        const unsigned char* src = lds + buf * TL::kTileBytes + (ks * 32 + l32) * TL::kRowBytes + hi * 16;
#pragma unroll
        for (int j = 0; j < TL::kSteps; j++)
          kf[j] = as_frag(*reinterpret_cast<const uint4*>(src + j * 32));
#pragma unroll
        for (int s = 0; s < 2; s++) {
          f32x16 acc = {0};
#pragma unroll
          for (int j = 0; j < TL::kSteps; j++)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[s][j], acc, 0, 0, 0);
          if (tail) {
            const int kb = t * kKeyTile + ks * 32 + hi * 4;
#pragma unroll
            for (int v = 0; v < 16; v++)
              if (kb + (v >> 2) * 8 + (v & 3) >= pl.N) acc[v] = -INFINITY;
          }
          float tmax = acc[0];
#pragma unroll
          for (int v = 1; v < 16; v++) tmax = fmaxf(tmax, acc[v]);
          const float mn = fmaxf(m[s], tmax);
          const float mref = mn == -INFINITY ? 0.f : mn;  // all 16 keys masked and nothing seen yet
          const float mc = mref * c2;
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; v++) sum += fast_exp2(fmaf(acc[v], c2, -mc));
          D[s] = D[s] * fast_exp2(fmaf(m[s], c2, -mc)) + sum;
          m[s] = mn;
        }
      }
    }
    buf ^= 1;
  }

  if (!active) return;
#pragma unroll
  for (int s = 0; s < 2; s++) {
    // lanes l and l^32 hold the same query row over disjoint keys
    const float mo = __shfl_xor(m[s], 32), Do = __shfl_xor(D[s], 32);
    const float mn = fmaxf(m[s], mo);
    const float mref = mn == -INFINITY ? 0.f : mn;
    const float Dn = D[s] * fast_exp2((m[s] - mref) * c2) + Do * fast_exp2((mo - mref) * c2);
    const int r = row0 + s * 32 + l32;
    if (hi == 0 && r < pl.R)
      stats[((size_t)bh * pl.n_splits + split) * pl.Rpad + r] = make_float2(mn * c2, Dn);
  }
}

// ------------------------------------------------------------------ pass 2
template <int HD, int REDUCE>
__global__ __launch_bounds__(256, 2) void score_reduce(const bf16_t* __restrict__ q,
                                                       const bf16_t* __restrict__ k,
                                                       const float2* __restrict__ stats,
                                                       float* __restrict__ scores, Plan pl) {
  using TL = Tile<HD>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* lds = smem;                                            // 2 query tiles
  float* nlse = reinterpret_cast<float*>(smem + 2 * TL::kTileBytes);    // [Rpad] minus base-2 lse
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, hi = lane >> 5;
  const int bh = blockIdx.y, b = bh / pl.Hkv, h = bh % pl.Hkv;
  const int key0 = blockIdx.x * kKeysPerWG + wave * 64;
  const float c2 = pl.c2;

  // combine the key splits of pass 1 into one log-sum-exp per query row
  for (int r = tid; r < pl.Rpad; r += 256) {
    float val = -INFINITY;  // padding rows: weight exp2(-inf) = 0
    if (r < pl.R) {
      const float2* st = stats + (size_t)bh * pl.n_splits * pl.Rpad + r;
      float mx = -INFINITY;
      for (int s = 0; s < pl.n_splits; s++) mx = fmaxf(mx, st[(size_t)s * pl.Rpad].x);
      float den = 0.f;
      for (int s = 0; s < pl.n_splits; s++) {
        const float2 e = st[(size_t)s * pl.Rpad];
        den += e.y * fast_exp2(e.x - mx);
      }
      val = -(mx + __log2f(den));
    }
    nlse[r] = val;
  }

  // key fragments of this wave stay in registers for the whole query loop
  const bf16_t* kbase = k + b * pl.ksb + (int64_t)h * pl.ksh;
  bf16x8 kf[2][TL::kSteps];
#pragma unroll
  for (int s = 0; s < 2; s++) {
    const int key = min(key0 + s * 32 + l32, pl.N - 1);
    const bf16_t* krow = kbase + (int64_t)key * pl.kst + hi * 8;
#pragma unroll
    for (int j = 0; j < TL::kSteps; j++)
      kf[s][j] = as_frag(*reinterpret_cast<const uint4*>(krow + j * 16));
  }

  const bf16_t* qbase = q + b * pl.qsb + (int64_t)(h * pl.G) * pl.qsh;
  uint4 stage[TL::kLoads];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int i = 0; i < TL::kLoads; i++) {
      const int c = tid + i * 256;
      const int row = c / TL::kChunks, ch = c % TL::kChunks;
      const int r = t * 64 + row;
      uint4 u = make_uint4(0, 0, 0, 0);
      if (r < pl.R)
        u = *reinterpret_cast<const uint4*>(qbase + (int64_t)(r / pl.p) * pl.qsh +
                                            (int64_t)(r % pl.p) * pl.qst + ch * 8);
      stage[i] = u;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TL::kLoads; i++) {
      const int c = tid + i * 256;
      const int row = c / TL::kChunks, ch = c % TL::kChunks;
      *reinterpret_cast<uint4*>(lds + buf * TL::kTileBytes + row * TL::kRowBytes + ch * 16) = stage[i];
    }
  };

  // SUM: running sum of weights.  MAX: running max of the base-2 log weight
  // (exp2 is monotone, so one exponential per key at the end is enough).
  float col[2];
  col[0] = col[1] = REDUCE == EPICACHE_REDUCE_MAX ? -INFINITY : 0.f;

  const int qtiles = pl.Rpad / 64;
  load_tile(0);
  int buf = 0;
  for (int t = 0; t < qtiles; t++) {
    store_tile(buf);
    __syncthreads();  // also orders the nlse[] writes above before their first use
    if (t + 1 < qtiles) load_tile(t + 1);
#pragma unroll
    for (int qs = 0; qs < 2; qs++) {
      bf16x8 qf[TL::kSteps];
      const unsigned char* src = lds + buf * TL::kTileBytes + (qs * 32 + l32) * TL::kRowBytes + hi * 16;
#pragma unroll
      for (int j = 0; j < TL::kSteps; j++)
        qf[j] = as_frag(*reinterpret_cast<const uint4*>(src + j * 32));
      float nl[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; g4++) {
        const float4 x = *reinterpret_cast<const float4*>(nlse + t * 64 + qs * 32 + g4 * 8 + hi * 4);
        nl[g4 * 4 + 0] = x.x, nl[g4 * 4 + 1] = x.y, nl[g4 * 4 + 2] = x.z, nl[g4 * 4 + 3] = x.w;
      }
#pragma unroll
      for (int s = 0; s < 2; s++) {
        f32x16 acc = {0};
#pragma unroll
        for (int j = 0; j < TL::kSteps; j++)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[j], kf[s][j], acc, 0, 0, 0);
        if (REDUCE == EPICACHE_REDUCE_MAX) {
          float x = col[s];
#pragma unroll
          for (int v = 0; v < 16; v++) x = fmaxf(x, fmaf(acc[v], c2, nl[v]));
          col[s] = x;
        } else {
          float x = 0.f;
#pragma unroll
          for (int v = 0; v < 16; v++) x += fast_exp2(fmaf(acc[v], c2, nl[v]));
          col[s] += x;
        }
      }
    }
    buf ^= 1;
  }

#pragma unroll
  for (int s = 0; s < 2; s++) {
    // lanes l and l^32 hold the same key over disjoint query rows
    const float o = __shfl_xor(col[s], 32);
    float val;
    if (REDUCE == EPICACHE_REDUCE_MAX) val = fast_exp2(fmaxf(col[s], o));
    else val = col[s] + o;
    const int key = key0 + s * 32 + l32;
    if (hi == 0 && key < pl.N) scores[(size_t)bh * pl.N + key] = val;
  }
}

template <int HD>
hipError_t launch_hd(const Plan& pl, const bf16_t* q, const bf16_t* k, float* scores,
                     float2* stats, hipStream_t stream) {
  using TL = Tile<HD>;
  const int nbh = pl.nb * pl.Hkv;
  dim3 g1(pl.n_splits, (pl.R + kRowsPerWG - 1) / kRowsPerWG, nbh);
  hipLaunchKernelGGL(score_stats<HD>, g1, dim3(256), 0, stream, q, k, stats, pl);
  dim3 g2((pl.N + kKeysPerWG - 1) / kKeysPerWG, nbh);
  const size_t smem = 2 * TL::kTileBytes + (size_t)pl.Rpad * sizeof(float);
  if (pl.reduce == EPICACHE_REDUCE_MAX)
    hipLaunchKernelGGL((score_reduce<HD, EPICACHE_REDUCE_MAX>), g2, dim3(256), smem, stream, q, k,
                       stats, scores, pl);
  else
    hipLaunchKernelGGL((score_reduce<HD, EPICACHE_REDUCE_SUM>), g2, dim3(256), smem, stream, q, k,
                       stats, scores, pl);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_mfma(const Plan& pl, const void* q, const void* k, float* scores,
                             float2* stats, hipStream_t stream) {
  const bf16_t* qq = static_cast<const bf16_t*>(q);
  const bf16_t* kk = static_cast<const bf16_t*>(k);
  if (pl.d == 128) return launch_hd<128>(pl, qq, kk, scores, stats, stream);
  if (pl.d == 64) return launch_hd<64>(pl, qq, kk, scores, stats, stream);
  return hipErrorInvalidValue;
}

}  // namespace epicache
