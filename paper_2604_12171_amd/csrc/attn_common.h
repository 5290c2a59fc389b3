// Device helpers shared by the decode and prefill attention kernels (gfx950).
#pragma once
#include "internal.h"
#include "scan.h"

namespace pipelive {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int lane) {
  uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, lane);
  uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}

// max of a value with the lane 16 (32) positions away: one v_permlane16_swap
// (v_permlane32_swap) of gfx950 instead of a trip through the LDS crossbar.
// The swap of (x, x) leaves lane i's own value in one result and lane i^16's
// (i^32's) in the other.
__device__ __forceinline__ float xor16_max(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// max(a, b) for values that are never NaN, as the bare instruction: fmaxf() would first quiet each
// operand that the compiler cannot prove canonical (one more instruction per operand).
__device__ __forceinline__ float max_no_nan(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// The maximum over the four 16-lane rows of a and of b, per lane position inside the row, for both
// values at once: the first swap pairs the rows of a and b (rows 0, 2 then hold a's pair maxima, rows
// 1, 3 b's), the second joins the two halves, the third hands every row both results.  Three swaps
// and two maxima instead of four and four.  Inputs must not be NaN.
__device__ __forceinline__ void rows_max_pair(float a, float b, float &ma, float &mb) {
  const auto r1 = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  const float y = max_no_nan(__uint_as_float(r1[0]), __uint_as_float(r1[1]));
  const auto r2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  const float z = max_no_nan(__uint_as_float(r2[0]), __uint_as_float(r2[1]));
  const auto r3 = __builtin_amdgcn_permlane16_swap(__float_as_uint(z), __float_as_uint(z), false, false);
  ma = __uint_as_float(r3[0]);
  mb = __uint_as_float(r3[1]);
}

// two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, bf16x2));
}

// Softmax weights as MFMA operands: p = hi + lo with hi = bf16(p) (nearest) and
// lo = bf16(p - hi); the pair keeps 16 mantissa bits of the fp32 weight.
__device__ __forceinline__ void split_weights(const float (&pv)[8], u32x4 &ph, u32x4 &pl) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = pack_bf16_rne(pv[2 * i], pv[2 * i + 1]);
    const float r0 = pv[2 * i] - __uint_as_float(h[i] << 16);
    const float r1 = pv[2 * i + 1] - __uint_as_float(h[i] & 0xFFFF0000u);
    l[i] = pack_bf16_rne(r0, r1);
  }
  ph = (u32x4){h[0], h[1], h[2], h[3]};
  pl = (u32x4){l[0], l[1], l[2], l[3]};
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float o) {
  uint32_t u = __float_as_uint(o);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}


constexpr int kTile = 32;      // tokens per tile
constexpr int kSubTiles = 32;  // tiles whose block addresses are resolved at once

// KV blocks are reached through 64-bit addresses read from the block list; the
// explicit global address space keeps the loads global_load (not flat_load).
typedef const u32x4 __attribute__((address_space(1))) *global_u4;
typedef const u32x2 __attribute__((address_space(1))) *global_u2;

template <int D>
struct KRegs {
  u32x4 k[2][D / 32];
  int nvalid[2];
};
template <int D>
struct VRegs {
  u32x2 v[D / 16][2];
};

// In-block layout: a block of BS tokens is a sequence of sub-blocks of
// SB = min(BS, 32) tokens; a sub-block holds K[Hkv][D/8][SB][8] and then
// V[Hkv][D][SB] (bf16), so the operands of one 32-token tile are two runs of
// contiguous memory per KV head whatever the block size.
template <int BS>
struct SubBlock {
  static constexpr int SB = BS < kTile ? BS : kTile;
  __device__ static uint32_t bytes(int Hkv, int D) { return (uint32_t)(2 * Hkv * SB * D * 2); }
};

// K and V are read once per launch, so their loads are nontemporal: the lines are
// streamed past the L2 instead of displacing each other there (measured on MI355X:
// 8-11 % shorter decode launches than with ordinary loads).
//
// Issue the K loads of one tile.  a0/a1 are the (wave-uniform) addresses of
// the sub-blocks holding its two 16-token halves (the same sub-block twice
// when SB = 32; both always valid memory: a half without tokens re-reads the
// first half's sub-block and is masked), nv0/nv1 the number of valid tokens in
// each half.
template <int D, int BS>
__device__ __forceinline__ void load_k(KRegs<D> &t, uint64_t a0, uint64_t a1, int nv0, int nv1, int g,
                                       int r, int qg) {
  constexpr int NC = D / 32;
  constexpr int SB = SubBlock<BS>::SB;
  constexpr int KHEAD = SB * D * 2;
#pragma unroll
  for (int T = 0; T < 2; ++T) {
    const uint64_t addr = T ? a1 : a0;
    const int nv = T ? nv1 : nv0;
    t.nvalid[T] = nv > 0 ? nv : 0;
    const int toff = (SB == kTile) ? 16 * T : 0;
    const uint64_t kb = addr + (uint64_t)g * KHEAD + (uint32_t)((qg * SB + toff + r) * 16);
#pragma unroll
    for (int c = 0; c < NC; ++c) t.k[T][c] = __builtin_nontemporal_load((global_u4)(kb + (uint32_t)(4 * c * SB * 16)));
  }
}

template <int D, int BS>
__device__ __forceinline__ void load_v(VRegs<D> &t, uint64_t a0, uint64_t a1, int g, int Hkv, int r,
                                       int qg) {
  constexpr int ND = D / 16;
  constexpr int SB = SubBlock<BS>::SB;
  constexpr int KHEAD = SB * D * 2;
#pragma unroll
  for (int T = 0; T < 2; ++T) {
    const uint64_t addr = T ? a1 : a0;
    const int toff = (SB == kTile) ? 16 * T : 0;
    const uint64_t vb = addr + (uint64_t)(Hkv + g) * KHEAD + (uint32_t)((r * SB + toff + 4 * qg) * 2);
#pragma unroll
    for (int c = 0; c < ND; ++c) t.v[c][T] = __builtin_nontemporal_load((global_u2)(vb + (uint32_t)(16 * c * SB * 2)));
  }
}

}  // namespace pipelive
