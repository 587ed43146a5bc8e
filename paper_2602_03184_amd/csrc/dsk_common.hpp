// Shared device helpers for the DynSplit-KV gfx950 kernels: bf16 unpacking, 64-lane
// wavefront reductions, order-preserving float keys.  Device code only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dsk.h"

#define DSK_WAVE 64

namespace dsk {

// ---- bf16 <-> f32 (bf16 is the upper half of an f32) ---------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// exact when the float already holds a bf16 value
__device__ __forceinline__ uint32_t pack_bf16_exact(float lo, float hi) {
  return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
}

// nearest bf16 value (ties to even) of a finite float, returned as a float
__device__ __forceinline__ float bf16_round_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xFFFF0000u);
}

// 8 bf16 values (one 16-byte vector) widened to fp32
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
  f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
  f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
  f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

// ---- keeping a batch of independent loads in flight together -------------------------------
// The compiler sinks loads towards their first use, which turns a batch of independent loads
// into a chain of memory round trips in latency-bound kernels.  pin_loaded(x) is an empty asm
// that takes x in and out and clobbers "memory": no load written before it in the source can be
// moved below it, so every load of the batch is issued before the first pin, and the compiler
// (which still tracks these ordinary loads) places its own s_waitcnt in front of each pin.
template <typename T>
__device__ __forceinline__ void pin_loaded(T& v) {
  asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w)::"memory");
}

// ---- wavefront (64 lanes) helpers ------------------------------------------------------
__device__ __forceinline__ float shfl_xor_f(float v, int mask) { return __shfl_xor(v, mask, DSK_WAVE); }
__device__ __forceinline__ int shfl_xor_i(int v, int mask) { return __shfl_xor(v, mask, DSK_WAVE); }

// Cross-lane moves inside a row of 16 lanes run on the vector ALU's data-parallel-primitive path
// (no trip through the LDS crossbar).  Controls: quad_perm [1,0,3,2] and [2,3,0,1] swap
// neighbours / pairs, the mirrors reverse 8 or 16 lanes -- after the two quad steps all four
// lanes of a quad agree, so the mirrors complete an all-reduce over the row.
constexpr int kDppSwap1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppSwap2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <- lane 7-i  (within 8)
constexpr int kDppMirror = 0x140;      // lane i <- lane 15-i (within 16)
constexpr int kDppRowShr = 0x110;      // + n: lane i <- lane i-n within the row
constexpr int kDppBcast15 = 0x142;     // lane 15 of a row -> every lane of the next row
constexpr int kDppBcast31 = 0x143;     // lane 31 -> every lane of rows 2 and 3

template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v))); }

// sum over aligned groups of 16 lanes (a K/V row is spread over 16 lanes x 8 channels);
// every lane of the group ends with the same bits as a xor-butterfly would give
__device__ __forceinline__ float group16_sum(float v) {
  v += dpp_f<kDppSwap1>(v);
  v += dpp_f<kDppSwap2>(v);
  v += dpp_f<kDppHalfMirror>(v);
  v += dpp_f<kDppMirror>(v);
  return v;
}
__device__ __forceinline__ float group16_max(float v) {
  v = fmaxf(v, dpp_f<kDppSwap1>(v));
  v = fmaxf(v, dpp_f<kDppSwap2>(v));
  v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f<kDppMirror>(v));
  return v;
}
__device__ __forceinline__ int group16_sum_i(int v) {
  v += dpp_i<kDppSwap1>(v);
  v += dpp_i<kDppSwap2>(v);
  v += dpp_i<kDppHalfMirror>(v);
  v += dpp_i<kDppMirror>(v);
  return v;
}
// Full-wavefront reductions: rows reduced as above, the four row results combined through
// scalar registers.  Every lane must be active.
__device__ __forceinline__ float rows4_f(float v, int r) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16 * r)); }
__device__ __forceinline__ float wave_sum(float v) {
  v = group16_sum(v);
  return (rows4_f(v, 0) + rows4_f(v, 1)) + (rows4_f(v, 2) + rows4_f(v, 3));
}
__device__ __forceinline__ float wave_max(float v) {
  v = group16_max(v);
  return fmaxf(fmaxf(rows4_f(v, 0), rows4_f(v, 1)), fmaxf(rows4_f(v, 2), rows4_f(v, 3)));
}
__device__ __forceinline__ int wave_sum_i(int v) {
  v = group16_sum_i(v);
  return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
         (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}
__device__ __forceinline__ uint32_t wave_min_u(uint32_t v) {
  uint32_t o;
  o = (uint32_t)dpp_i<kDppSwap1>((int)v); v = o < v ? o : v;
  o = (uint32_t)dpp_i<kDppSwap2>((int)v); v = o < v ? o : v;
  o = (uint32_t)dpp_i<kDppHalfMirror>((int)v); v = o < v ? o : v;
  o = (uint32_t)dpp_i<kDppMirror>((int)v); v = o < v ? o : v;
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  const uint32_t ab = a < b ? a : b, cd = c < d ? c : d;
  return ab < cd ? ab : cd;
}
__device__ __forceinline__ uint32_t wave_max_u(uint32_t v) { return ~wave_min_u(~v); }

// inclusive prefix sum across the 64 lanes (all active): shifts by 1, 2, 4, 8 inside each row
// (lanes without a source add 0), then lane 15 of rows 0 and 2 is added to rows 1 and 3, and
// lane 31 to rows 2 and 3
__device__ __forceinline__ int wave_incl_scan_i(int v, int /*lane*/) {
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 1, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 2, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 4, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 8, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppBcast15, 0xA, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppBcast31, 0xC, 0xF, false);
  return v;
}

// ---- order-preserving key of a float: a > b  <=>  key(a) > key(b); -0 folded into +0 ---
__device__ __forceinline__ uint32_t float_key(float s) {
  uint32_t u = __float_as_uint(s + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ void set_status(int32_t* dev_status, int32_t code) {
  if (dev_status) atomicCAS(dev_status, 0, code);
}

}  // namespace dsk
