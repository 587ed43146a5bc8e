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

// sum over aligned groups of 16 lanes (a K/V row is spread over 16 lanes x 8 channels)
__device__ __forceinline__ float group16_sum(float v) {
  v += shfl_xor_f(v, 1);
  v += shfl_xor_f(v, 2);
  v += shfl_xor_f(v, 4);
  v += shfl_xor_f(v, 8);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  v = group16_sum(v);
  v += shfl_xor_f(v, 16);
  v += shfl_xor_f(v, 32);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 1; m < DSK_WAVE; m <<= 1) v = fmaxf(v, shfl_xor_f(v, m));
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int m = 1; m < DSK_WAVE; m <<= 1) v += shfl_xor_i(v, m);
  return v;
}
// inclusive prefix sum across the 64 lanes
__device__ __forceinline__ int wave_incl_scan_i(int v, int lane) {
#pragma unroll
  for (int d = 1; d < DSK_WAVE; d <<= 1) {
    int o = __shfl_up(v, d, DSK_WAVE);
    if (lane >= d) v += o;
  }
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
