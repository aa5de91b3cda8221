// Attention output of the patch tokens (paper Sec. 2.3: the patched prompt is appended after the block and
// attends back to it): for every patch query t of every query head,
//   O_t = sum_i softmax_i(scale * q_t . k_i) v_i,   lse_t = log sum_i exp(scale * q_t . k_i),
// over the N context rows and, with causal_patch, the patch rows 0..t that follow them in K and V.
// The normalisers are exactly what the single-pass scoring takes, so this call followed by the scoring on
// supplied normalisers is the patch's whole pass through the layer plus Eq. 1.
//
// bf16, head_dim 128: one wave owns 32 query rows; 64-key tiles of K and of V stream HBM -> LDS
// (direct loads, double buffered).  Per 32-key half: S^T = K Q^T on the matrix cores (a lane owns one query
// column and 16 keys, as in the scoring statistics pass), an online softmax whose row maximum is shared by
// the two lanes of a row, the weights rounded to bf16, and O^T += V^T P^T.  The V^T operand (8 consecutive
// keys of one head_dim column per lane) comes out of the row-major V tile with the transposing LDS load:
// 16 lanes that point at 4 keys x 16 columns get, lane i, the 4 keys of column i.
// Anything else (fp32 inputs, other head dims): a plain fp32 kernel.
#include <hip/hip_bf16.h>

#include <type_traits>

#include "mfma_tiles.h"

namespace epicache {
namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kHD = 128;
constexpr float kLazyBits = 8.f;
using TL = Tile<kHD>;

// V tiles use their own swizzle: 16-byte chunk c of key row r sits at position c ^ (4 * (r % 4)), so the four
// key rows that one transposing load touches fall into four different 64-byte bank groups.
__device__ __forceinline__ int swz_v(int r) { return 4 * (r & 3); }

template <int NW>
struct StagerV {
  static constexpr int kSlabs = TL::kTileBytes / 1024;
  static constexpr int kPer = (kSlabs + NW - 1) / NW;
  template <typename RowPtr>
  __device__ static __forceinline__ void run_rows(uint32_t lds_tile, int wave, int lane, RowPtr row_ptr) {
#pragma unroll
    for (int i = 0; i < kPer; i++) {
      if (kSlabs % NW == 0 || wave + i * NW < kSlabs) {
        const int row = (wave + i * NW) * TL::kRowsPerSlab + lane / TL::kChunks;
        dma16_lane_ptr(lds_tile + (wave + i * NW) * 1024,
                       row_ptr(row) + (((lane % TL::kChunks) ^ swz_v(row)) * 16));
      }
    }
  }
};

// A operand of O^T += V^T P^T for head_dim block `dblk` (32 columns) and the 16-key step `kstep` of the
// 32-key half `ks`: lane (m = l % 32, hi = l / 32) needs keys {4 hi .. 4 hi + 3} and {8 + 4 hi .. 8 + 4 hi + 3}
// (+ 16 kstep + 32 ks) of column 32 dblk + m, the key order in which the softmax weights sit in the lane.
__device__ __forceinline__ bf16x8 read_vt_frag(const unsigned char* vtile, int ks, int kstep, int dblk, int lane) {
  const int s = lane & 15, gh = (lane >> 4) & 1, hi = lane >> 5;
  const int chunk = 4 * dblk + 2 * gh + ((s & 3) >> 1);      // 16-byte chunk of the row this lane points into
  const int half = (s & 1) * 8;
  s16x4 part[2];
#pragma unroll
  for (int g = 0; g < 2; g++) {
    const int row = 32 * ks + 16 * kstep + 8 * g + 4 * hi + (s >> 2);
    const unsigned char* p = vtile + row * TL::kRowBytes + ((chunk ^ swz_v(row)) * 16) + half;
    part[g] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)LDS_PTR(p));
  }
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  const s16x8 both = {part[0][0], part[0][1], part[0][2], part[0][3], part[1][0], part[1][1], part[1][2], part[1][3]};
  return __builtin_bit_cast(bf16x8, both);
}

// max(x[l], x[l ^ 32]) in every lane, on the vector ALU: the swap leaves the lower half's values in both
// halves of one register and the upper half's in both halves of the other.
__device__ __forceinline__ float max_across_halves(float x) {
  const unsigned int u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// The row maximum is taken with compiler-visible max operations, not the hand-written v_max3_f32 of the scoring
// kernels: the compiler's hazard pass does not treat inline assembly as a vector ALU instruction, so a
// hand-written v_max3_f32 scheduled straight behind the S chain read the accumulators before the matrix core
// had written them (no wait states inserted).  The stale maximum is still a valid reference, so results stayed
// inside the tolerance but differed from run to run in the last bf16 bit.
// Two waves per SIMD (a cap of 256 registers per wave): two workgroups per CU when a workgroup has 3 or 4 waves,
// one when it has 8; the 2-wave form keeps the uncapped allocation.
template <int NW>
__global__ __launch_bounds__(NW * 64, (NW >= 3 && NW < 8) ? 2 : 1) void patch_attention_mfma(const bf16_t* __restrict__ q,
                                                                   const bf16_t* __restrict__ k,
                                                                   const bf16_t* __restrict__ v,
                                                                   bf16_t* __restrict__ out,
                                                                   float* __restrict__ lse_out, Plan pl) {
  using ST = Stager<kHD, NW>;
  using SV = StagerV<NW>;
  constexpr int KS = TL::kSteps;  // 8
  __shared__ __attribute__((aligned(1024))) unsigned char lds_k[2 * TL::kTileBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char lds_v[2 * TL::kTileBytes];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  // XCD-aware ids: the row blocks of one (b, h) read the same K and V and land on one XCD
  const int n_rb = (pl.R + 32 * NW - 1) / (32 * NW);
  const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
  const int rb = within % n_rb;
  const int bh = (within / n_rb) * 8 + xcd;
  if (bh >= pl.nb * pl.Hkv) return;
  const int b = bh / pl.Hkv, h = bh % pl.Hkv;
  // the 32-row blocks are dealt evenly to the n_rb workgroups of a head: workgroups that do the same amount of
  // work stream K and V at the same pace, so the second one finds the tiles in the XCD's L2
  const int blocks_per_rb = ((pl.R + 31) / 32 + n_rb - 1) / n_rb;
  const int row0 = (rb * blocks_per_rb + wave) * 32;
  const bool active = wave < blocks_per_rb && row0 < pl.R;  // waves without rows only help staging the tiles
  const float c2 = pl.c2;
  const int N = ctx_rows(pl, bh);  // this head's own context length in a ragged batch
  const int n_keys = N + (pl.causal_patch ? pl.p : 0);  // context rows, then the patch's own rows
  const int tiles = (n_keys + kKeyTile - 1) / kKeyTile;

  const int r = row0 + l32;            // this lane's query row
  const bool row_ok = r < pl.R;
  const int rr = row_ok ? r : 0;
  const int t_row = rr % pl.p;         // patch token index: sees patch keys 0..t_row
  if (n_keys == 0) {  // a head without a single key (workgroup-uniform): O = 0, lse = -inf
    if (active && row_ok) {
      const int hq = h * pl.G + r / pl.p;
      const size_t orow = ((size_t)b * pl.Hq + hq) * pl.p + t_row;
      if (hi == 0) lse_out[orow] = -INFINITY;
      uint4* o4 = reinterpret_cast<uint4*>(out + orow * kHD + hi * 64);
#pragma unroll
      for (int j = 0; j < 8; j++) o4[j] = make_uint4(0, 0, 0, 0);
    }
    return;
  }
  bf16x8 qf[KS];
  {
    const bf16_t* qrow = q + b * pl.qsb + (int64_t)(h * pl.G + rr / pl.p) * pl.qsh + (int64_t)t_row * pl.qst + hi * 8;
#pragma unroll
    for (int j = 0; j < KS; j++) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (row_ok) u = *reinterpret_cast<const uint4*>(qrow + j * 16);
      qf[j] = as_frag(u);
    }
  }

  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(k + b * pl.ksb + (int64_t)h * pl.ksh);
  const unsigned char* vbase = reinterpret_cast<const unsigned char*>(v + b * pl.ksb + (int64_t)h * pl.ksh);
  const uint32_t kstride = (uint32_t)pl.kst * 2;
  const uint32_t ldsk0 = lds_address(lds_k), ldsv0 = lds_address(lds_v);
  auto stage = [&](int buf, int t) {
    const int first = t * kKeyTile;
    const int nrows = min(kKeyTile, n_keys - first);  // rows beyond the last key re-read it; their weight is 0
    const unsigned char* kt = kbase + (size_t)first * kstride;
    const unsigned char* vt = vbase + (size_t)first * kstride;
    ST::run_rows(ldsk0 + buf * TL::kTileBytes, wave, lane,
                 [=](int row) { return kt + (size_t)min(row, nrows - 1) * kstride; });
    SV::run_rows(ldsv0 + buf * TL::kTileBytes, wave, lane,
                 [=](int row) { return vt + (size_t)min(row, nrows - 1) * kstride; });
  };

  f32x16 o[4];  // O^T: head_dim block x 16 values (head_dim (v/4)*8 + hi*4 + v%4 of the block), this lane's row
#pragma unroll
  for (int d = 0; d < 4; d++)
#pragma unroll
    for (int i = 0; i < 16; i++) o[d][i] = 0.f;
  const float lazy = kLazyBits / c2;  // in units of the raw dot product
  float m = kNoMax, l = 0.f;  // running row maximum (raw dot products, shared by lanes l and l^32) and this lane's sum

  stage(0, 0);
  wait_vmem();
  __syncthreads();
  // One 64-key tile out of buffer BUF.  The buffer index is a compile-time constant (the tile loop below is
  // unrolled by two) so that every LDS address is a loop-invariant lane offset plus an immediate.
  auto tile_step = [&](auto buf_c, int t) {
    constexpr int BUF = decltype(buf_c)::value;
    const unsigned char* ktile = lds_k + BUF * TL::kTileBytes;
    const unsigned char* vtile = lds_v + BUF * TL::kTileBytes;
    if (t + 1 < tiles) stage(BUF ^ 1, t + 1);
    if (active) {
      const int first = t * kKeyTile;
      const bool plain = first + kKeyTile <= N;  // every key of the tile is a context key: no masking
      bf16x8 kf[KS];
      read_frags<kHD>(kf, ktile, 0, l32, hi);
#pragma unroll
      for (int ks = 0; ks < 2; ks++) {
        f32x16 sacc;
        mfma_chain<KS>(sacc, kf, qf);
        // LDS reads that the arithmetic below can hide: the key fragments of the second half and the eight
        // V^T fragments of this half
        if (ks == 0) read_frags<kHD>(kf, ktile, 1, l32, hi);
        bf16x8 vf[4][2];
#pragma unroll
        for (int d = 0; d < 4; d++)
#pragma unroll
          for (int st = 0; st < 2; st++) vf[d][st] = read_vt_frag(vtile, ks, st, d, lane);
        if (!plain) {
#pragma unroll
          for (int i = 0; i < 16; i++) {
            const int key = first + ks * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
            const bool visible = key < N || (key < n_keys && key - N <= t_row);
            if (!visible) sacc[i] = kMasked;
          }
        }
        // row maximum over this lane's 16 keys, then over the two lanes of the row
        const float a0 = max3(sacc[0], sacc[1], sacc[2]), a1 = max3(sacc[3], sacc[4], sacc[5]);
        const float a2 = max3(sacc[6], sacc[7], sacc[8]), a3 = max3(sacc[9], sacc[10], sacc[11]);
        const float a4 = max3(sacc[12], sacc[13], sacc[14]);
        const float mn = max_across_halves(max3(max3(a0, a1, a2), max3(a3, a4, sacc[15]), m));
        // The reference m only has to keep the exponentials in range, so it follows the maximum lazily: sums
        // and outputs move to a new reference only when some row's maximum exceeds the current one by more than
        // 2^kLazyBits in weight (weights then stay below that factor; fp32 sums and bf16 weights keep their
        // relative precision).  Without the slack ~60 % of the 32-key steps of a 4096-key context rescale.
        if (__any(mn > m + lazy)) {
          const float corr = ex2((m - mn) * c2);
          l *= corr;
#pragma unroll
          for (int d = 0; d < 4; d++)
#pragma unroll
            for (int i = 0; i < 16; i++) o[d][i] *= corr;
          m = mn;
        }
        const float nmc = -m * c2;
        float e[16];
#pragma unroll
        for (int i = 0; i < 16; i++) e[i] = ex2(fmaf(sacc[i], c2, nmc));
        l += ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7])) +
             (((e[8] + e[9]) + (e[10] + e[11])) + ((e[12] + e[13]) + (e[14] + e[15])));
        // weights to bf16: values 0..7 are the keys of the first 16-key step, 8..15 of the second
        bf16x8 pf[2];
#pragma unroll
        for (int st = 0; st < 2; st++) {
          typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
          u32x4 packed;
#pragma unroll
          for (int j = 0; j < 4; j++) {
            const f32x2 pair = {e[8 * st + 2 * j], e[8 * st + 2 * j + 1]};
            packed[j] = __builtin_bit_cast(unsigned int, __builtin_convertvector(pair, bf16x2));
          }
          pf[st] = __builtin_bit_cast(bf16x8, packed);
        }
#pragma unroll
        for (int st = 0; st < 2; st++)
#pragma unroll
          for (int d = 0; d < 4; d++)  // four independent accumulators back to back
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[d][st], pf[st], o[d], 0, 0, 0);
      }
    }
    wait_vmem();
    __syncthreads();
  };
  for (int t = 0; t < tiles; t += 2) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < tiles) tile_step(std::integral_constant<int, 1>{}, t + 1);
  }

  if (!active) return;
  const float l_row = l + __shfl_xor(l, 32);
  const float inv = 1.0f / l_row;
  if (row_ok) {
    const int hq = h * pl.G + r / pl.p;
    if (hi == 0) lse_out[((size_t)b * pl.Hq + hq) * pl.p + t_row] = (m * c2 + __log2f(l_row)) * 0.69314718055994530942f;
    bf16_t* orow = out + (((size_t)b * pl.Hq + hq) * pl.p + t_row) * kHD;
#pragma unroll
    for (int d = 0; d < 4; d++) {
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const f32x2 p0 = {o[d][4 * g + 0] * inv, o[d][4 * g + 1] * inv};
        const f32x2 p1 = {o[d][4 * g + 2] * inv, o[d][4 * g + 3] * inv};
        uint2 w;
        w.x = __builtin_bit_cast(unsigned int, __builtin_convertvector(p0, bf16x2));
        w.y = __builtin_bit_cast(unsigned int, __builtin_convertvector(p1, bf16x2));
        *reinterpret_cast<uint2*>(orow + d * 32 + g * 8 + hi * 4) = w;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------- plain fp32 form
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__hip_bfloat16 x) { return __bfloat162float(x); }
__device__ __forceinline__ void from_f32(float& dst, float x) { dst = x; }
__device__ __forceinline__ void from_f32(__hip_bfloat16& dst, float x) { dst = __float2bfloat16(x); }

// One workgroup per query row.  Keys are taken 256 at a time: thread i scores key i, the chunk's maximum
// and sum update the running pair, then thread c accumulates head_dim column c over the chunk's keys.
template <typename T>
__global__ __launch_bounds__(256) void patch_attention_plain(const T* __restrict__ q, const T* __restrict__ k,
                                                             const T* __restrict__ v, T* __restrict__ out,
                                                             float* __restrict__ lse_out, Plan pl) {
  __shared__ float qs[256], w[256], red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = blockIdx.x % pl.p, hq = (blockIdx.x / pl.p) % pl.Hq, b = blockIdx.x / (pl.p * pl.Hq);
  const int h = hq / pl.G;
  const T* qrow = q + b * pl.qsb + (int64_t)hq * pl.qsh + (int64_t)t * pl.qst;
  for (int c = tid; c < pl.d; c += 256) qs[c] = to_f32(qrow[c]);
  __syncthreads();
  const T* kbase = k + b * pl.ksb + (int64_t)h * pl.ksh;
  const T* vbase = v + b * pl.ksb + (int64_t)h * pl.ksh;
  const int n_keys = ctx_rows(pl, b * pl.Hkv + h) + (pl.causal_patch ? t + 1 : 0);
  float m = -INFINITY, l = 0.f, acc = 0.f;  // acc: column tid of the output, relative to the reference m
  auto block_reduce = [&](float x, bool is_max) {
    for (int off = 32; off >= 1; off >>= 1) {
      const float o = __shfl_xor(x, off);
      x = is_max ? fmaxf(x, o) : x + o;
    }
    __syncthreads();  // red[] of the previous reduction has been read by everyone
    if (lane == 0) red[wave] = x;
    __syncthreads();
    return is_max ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : (red[0] + red[1]) + (red[2] + red[3]);
  };
  for (int k0 = 0; k0 < n_keys; k0 += 256) {
    const int i = k0 + tid;
    float z = -INFINITY;
    if (i < n_keys) {
      const T* krow = kbase + (int64_t)i * pl.kst;
      float dot = 0.f;
      for (int c = 0; c < pl.d; c++) dot = fmaf(qs[c], to_f32(krow[c]), dot);
      z = dot * pl.c2;
    }
    const float mn = fmaxf(m, block_reduce(z, true));
    const float e = i < n_keys ? exp2f(z - mn) : 0.f;
    const float corr = exp2f(m - mn);  // first chunk: exp2(-inf) = 0 times 0
    const float s = block_reduce(e, false);
    l = l * corr + s;
    acc *= corr;
    m = mn;
    w[tid] = e;
    __syncthreads();
    if (tid < pl.d) {
      const int cnt = min(256, n_keys - k0);
      for (int j = 0; j < cnt; j++) acc = fmaf(w[j], to_f32(vbase[(int64_t)(k0 + j) * pl.kst + tid]), acc);
    }
    __syncthreads();  // w[] is rewritten by the next chunk
  }
  const size_t orow = ((size_t)b * pl.Hq + hq) * pl.p + t;
  if (tid < pl.d) from_f32(out[orow * pl.d + tid], n_keys > 0 ? acc / l : 0.f);  // no key at all: O = 0, lse = -inf
  if (tid == 0) lse_out[orow] = n_keys > 0 ? (m + log2f(l)) * 0.69314718055994530942f : -INFINITY;
}

template <int NW>
void launch_mfma(const Plan& pl, const void* q, const void* k, const void* v, void* out, float* lse,
                 hipStream_t stream) {
  const int n_rb = (pl.R + 32 * NW - 1) / (32 * NW);
  const int bh8 = (pl.nb * pl.Hkv + 7) / 8 * 8;
  hipLaunchKernelGGL((patch_attention_mfma<NW>), dim3((unsigned)(n_rb * bh8)), dim3(NW * 64), 0, stream,
                     static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k), static_cast<const bf16_t*>(v),
                     static_cast<bf16_t*>(out), lse, pl);
}

}  // namespace

hipError_t launch_patch_attention(const Plan& pl, const void* q, const void* k, const void* v, void* out,
                                  float* lse, hipStream_t stream) {
  if (pl.dtype == EPICACHE_DTYPE_BF16 && pl.d == kHD) {
    // waves per workgroup (32 rows each): as many as R fills, so that K and V tiles are staged by as few row
    // blocks as possible.  Eight waves (one workgroup per CU) halve the L2 -> LDS traffic of four and are 2-3 %
    // faster from 256 rows on, although the tile barrier then stops both waves of every SIMD at once.
    const int best = pl.R <= 64 ? 2 : pl.R <= 96 ? 3 : pl.R < 256 ? 4 : 8;
    if (best == 8) launch_mfma<8>(pl, q, k, v, out, lse, stream);
    else if (best == 4) launch_mfma<4>(pl, q, k, v, out, lse, stream);
    else if (best == 3) launch_mfma<3>(pl, q, k, v, out, lse, stream);
    else launch_mfma<2>(pl, q, k, v, out, lse, stream);
    return hipGetLastError();
  }
  const unsigned rows = (unsigned)((size_t)pl.nb * pl.Hq * pl.p);
  if (pl.dtype == EPICACHE_DTYPE_F32)
    hipLaunchKernelGGL(patch_attention_plain<float>, dim3(rows), dim3(256), 0, stream, static_cast<const float*>(q),
                       static_cast<const float*>(k), static_cast<const float*>(v), static_cast<float*>(out), lse, pl);
  else
    hipLaunchKernelGGL(patch_attention_plain<__hip_bfloat16>, dim3(rows), dim3(256), 0, stream,
                       static_cast<const __hip_bfloat16*>(q), static_cast<const __hip_bfloat16*>(k),
                       static_cast<const __hip_bfloat16*>(v), static_cast<__hip_bfloat16*>(out), lse, pl);
  return hipGetLastError();
}

}  // namespace epicache
