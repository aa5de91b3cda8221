// Device helpers shared by the bf16 MFMA kernels (scoring passes, patch attention): vector types, the
// direct global->LDS staging of 64-row tiles with an XOR-swizzled LDS image, MFMA operand fragments.
#pragma once

#include "epicache_internal.h"

namespace epicache {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint16_t bf16_t;  // raw storage

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ bf16x8 as_frag(uint4 u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
// The bare instructions: fmaxf() on values that went through pin() gets a canonicalising v_max x, x
// in front of every operand, which doubled the ALU work of the max reduction.  The compiler's hazard pass does
// not see inline assembly as a vector ALU instruction and inserts no wait states for it: these must never be
// the first reader of an MFMA result (12 wait states after an 8-pass MFMA on gfx950) or of a transcendental's
// result.  The callers read values that a compiler-visible instruction has already read or produced;
// tests/test_isa_hazards.py checks the generated ISA for it.
__device__ __forceinline__ float vmax(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ void fence_sched() { __builtin_amdgcn_sched_barrier(0); }
// Keeps the computation of x above this point: without it the optimiser sinks a slice of
// arithmetic down to its first use, past the MFMAs it is meant to fill the shadow of.
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)


template <int HD>
struct Tile {
  static constexpr int kSteps = HD / 16;          // MFMAs per 32x32 output tile
  static constexpr int kChunks = HD / 8;          // 16-byte chunks per row
  static constexpr int kRowBytes = HD * 2;
  static constexpr int kTileBytes = 64 * kRowBytes;
  static constexpr int kSlabs = kTileBytes / 1024;   // 1 KiB wave-wide direct loads per tile
  static constexpr int kRowsPerSlab = 1024 / kRowBytes;
  // XOR swizzle: chunk c of row r sits at position c ^ swz(r)
  __device__ static __forceinline__ int swz(int r) { return (r / (16 / kChunks)) % kChunks; }
};

// 16 bytes per lane, global memory -> LDS without passing through registers: lane l of the wave
// writes LDS bytes [lds_addr + 16*l, +16).  Issued as inline assembly so that the compiler's
// wait-count pass does not serialise later ds_reads of the *other* LDS buffer behind these loads;
// completion is awaited explicitly (wait_vmem) before the barrier that publishes the tile.
// M0 is on the clobber lists: the statements overwrite it, and the compiler (which sets M0 itself right before
// its own users of it) must not assume a value survives them.  Clang flags any reserved register on a clobber
// list; for M0 the entry is exactly the definition that has to be declared.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16_uniform_base(uint32_t lds_addr, const void* base, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(base)
               : "memory", "m0");
}
__device__ __forceinline__ void dma16_lane_ptr(uint32_t lds_addr, const void* ptr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr), "v"(ptr)
               : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)LDS_PTR(p);
}

// Staging of one ROWS-row tile, global -> LDS, by NW waves.  Rows are `stride` bytes apart.
// Wave w issues the 1 KiB slabs w, w + NW, w + 2*NW, ...; `wave` must be wave-uniform.
template <int HD, int NW, int ROWS = 64>
struct Stager {
  using TL = Tile<HD>;
  static constexpr int kSlabs = ROWS * TL::kRowBytes / 1024;  // 1 KiB wave-wide direct loads per tile
  static constexpr int kPer = (kSlabs + NW - 1) / NW;          // direct loads per wave and tile (at most)
  // byte offset, from the first row of a tile, of the chunk that lane `lane` fetches in load i
  __device__ static __forceinline__ void offsets(uint32_t (&off)[kPer], int wave, int lane, uint32_t stride) {
#pragma unroll
    for (int i = 0; i < kPer; i++) {
      const int row = (wave + i * NW) * TL::kRowsPerSlab + lane / TL::kChunks;
      off[i] = row * stride + (((lane % TL::kChunks) ^ TL::swz(row)) * 16);
    }
  }
  // all 64 rows exist: tile base (wave-uniform) + per-lane offsets
  __device__ static __forceinline__ void run(uint32_t lds_tile, const unsigned char* base,
                                             const uint32_t (&off)[kPer], int wave) {
#pragma unroll
    for (int i = 0; i < kPer; i++)
      if (kSlabs % NW == 0 || wave + i * NW < kSlabs)
        dma16_uniform_base(lds_tile + (wave + i * NW) * 1024, base, off[i]);
  }
  // general form: `row_ptr(r)` gives the address of row r of the tile (clamping, ragged strides)
  template <typename RowPtr>
  __device__ static __forceinline__ void run_rows(uint32_t lds_tile, int wave, int lane, RowPtr row_ptr) {
#pragma unroll
    for (int i = 0; i < kPer; i++) {
      if (kSlabs % NW == 0 || wave + i * NW < kSlabs) {
        const int row = (wave + i * NW) * TL::kRowsPerSlab + lane / TL::kChunks;
        dma16_lane_ptr(lds_tile + (wave + i * NW) * 1024,
                       row_ptr(row) + (((lane % TL::kChunks) ^ TL::swz(row)) * 16));
      }
    }
  }
};

// MFMA operand fragments of one 32-row sub-tile of a staged tile.
template <int HD>
__device__ __forceinline__ void read_frags(bf16x8 (&f)[HD / 16], const unsigned char* lds_tile, int sub,
                                           int l32, int hi) {
  using TL = Tile<HD>;
  const int row = sub * 32 + l32;
  const unsigned char* base = lds_tile + row * TL::kRowBytes;
  const int s = TL::swz(row);
#pragma unroll
  for (int j = 0; j < TL::kSteps; j++)
    f[j] = as_frag(*reinterpret_cast<const uint4*>(base + (((2 * j + hi) ^ s) * 16)));
}

// Finite sentinels instead of infinities keep the running-max updates branch-free and NaN-free:
// kNoMax is the "no key seen yet" maximum, kMasked (< kNoMax) the logit of a key that must not count.
// Their products with c2 = scale * log2(e) must stay finite (no inf - inf in the exponent arithmetic), which
// holds for every scale the host accepts (<= 1e6); raw dot products are assumed to lie above kNoMax.
constexpr float kNoMax = -1.0e30f;
constexpr float kMasked = -2.0e30f;

template <int KS>
__device__ __forceinline__ void mfma_chain(f32x16& acc, const bf16x8 (&a)[KS], const bf16x8 (&b)[KS]) {
  const f32x16 zero = {0};
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], zero, 0, 0, 0);
#pragma unroll
  for (int j = 1; j < KS; j++) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], acc, 0, 0, 0);
}

}  // namespace epicache
