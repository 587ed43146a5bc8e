// V2F compression (Sec. 4.2, KVCache Compression): element-wise min and max of K (or V)
// over the tokens of every variable-length block.  One wavefront per (head, block):
// a 128-channel bf16 row is 256 B = 16 lanes x 16 B, so the 64 lanes cover 4 token rows
// per load instruction; rows stream from HBM fully coalesced and each is read once.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kSumThreads = 256;
constexpr int kSumWaves = kSumThreads / DSK_WAVE;
constexpr int kSumUnroll = 8;  // row-groups of 4 rows in flight per wave

// min / max (or mean) of rows [0, len) of one head, `base` pointing at row 0 of the block, written
// to the 512-byte record `o`.  All 64 lanes of a wavefront call it with wave-uniform arguments.
template <bool MEAN>
__device__ __forceinline__ void summarize_block(const uint16_t* base, int len, int64_t stride_tok, unsigned ustride,
                                                uint16_t* o, int g, int c) {
  // MEAN: mn[] holds this lane's running sums instead
  float mn[8], mx[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) { mn[k] = MEAN ? 0.0f : __builtin_inff(); mx[k] = -__builtin_inff(); }
  for (int r0 = 0; r0 < len; r0 += 4 * kSumUnroll) {
    // scalar 64-bit base of this row batch + 32-bit lane offsets (stride_tok <= 2^24, host-checked)
    const char* rb = reinterpret_cast<const char*>(base + (int64_t)r0 * stride_tok);
    const int last = len - 1 - r0;
    uint4 v[kSumUnroll];
#pragma unroll
    for (int u = 0; u < kSumUnroll; ++u) {
      int r = 4 * u + g;
      r = r < last ? r : last;     // a repeated row changes neither min nor max
      const unsigned byte_off = ((unsigned)r * ustride + (unsigned)(c * 8)) * 2u;
      v[u] = *reinterpret_cast<const uint4*>(rb + byte_off);
    }
#pragma unroll
    for (int u = 0; u < kSumUnroll; ++u) {
      float f[8];
      unpack8(v[u], f);
      if constexpr (MEAN) {
        const bool real = 4 * u + g <= last;         // a repeated row must not be added again
#pragma unroll
        for (int k = 0; k < 8; ++k) mn[k] += real ? f[k] : 0.0f;
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) { mn[k] = fminf(mn[k], f[k]); mx[k] = fmaxf(mx[k], f[k]); }
      }
    }
  }
  if constexpr (MEAN) {
    // fixed order: rows of a lane group in token order, then (g0 + g1) + (g2 + g3); the mean
    // rounded to nearest-even bf16 goes into both rows of the record
    const float inv_den = (float)len;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      mn[k] += shfl_xor_f(mn[k], 16);
      mn[k] += shfl_xor_f(mn[k], 32);
      mn[k] = bf16_round_rne(mn[k] / inv_den);
      mx[k] = mn[k];
    }
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      mn[k] = fminf(mn[k], shfl_xor_f(mn[k], 16)); mx[k] = fmaxf(mx[k], shfl_xor_f(mx[k], 16));
      mn[k] = fminf(mn[k], shfl_xor_f(mn[k], 32)); mx[k] = fmaxf(mx[k], shfl_xor_f(mx[k], 32));
    }
  }
  if (g == 0) {
    reinterpret_cast<uint4*>(o)[c] = make_uint4(pack_bf16_exact(mn[0], mn[1]), pack_bf16_exact(mn[2], mn[3]),
                                                pack_bf16_exact(mn[4], mn[5]), pack_bf16_exact(mn[6], mn[7]));
  } else if (g == 1) {
    reinterpret_cast<uint4*>(o)[16 + c] = make_uint4(pack_bf16_exact(mx[0], mx[1]), pack_bf16_exact(mx[2], mx[3]),
                                                     pack_bf16_exact(mx[4], mx[5]), pack_bf16_exact(mx[6], mx[7]));
  }
}

// 8 waves per SIMD (32 per CU) so that one launch keeps every wave of the grid resident
template <bool MEAN>
__global__ __launch_bounds__(kSumThreads) void summaries_kernel(
    const uint16_t* __restrict__ X, int64_t stride_tok, int64_t stride_head, int Hkv,
    const int32_t* __restrict__ block_start, const int32_t* __restrict__ cu_blocks, int B,
    const int32_t* __restrict__ blk_range, int cap, int out_rows, int total_tokens, uint16_t* __restrict__ out,
    int32_t* dev_status) {
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DSK_WAVE);   // wave-uniform: scalar registers
  const int g = lane >> 4;   // row group 0..3
  const int c = lane & 15;   // 16-byte column 0..15
  // blocks [i_lo, i_lo + nblk): the whole table, or the range an incremental update rewrote
  int i_lo = 0;
  int nblk = 0;
  if (blk_range != nullptr) {
    i_lo = blk_range[0];
    int i_hi = blk_range[1];
    if (i_hi > cap) i_hi = cap;
    if (i_lo < 0) i_lo = 0;
    nblk = i_hi - i_lo;
  } else {
    nblk = cu_blocks[B];
    if (nblk > cap) nblk = cap;
  }
  if (nblk <= 0) return;
  const int64_t items = (int64_t)Hkv * nblk;
  const int64_t nwaves = (int64_t)gridDim.x * kSumWaves;
  int64_t item = (int64_t)blockIdx.x * kSumWaves + wave;
  if (item >= items) return;
  int h = (int)(item / nblk);
  int i = i_lo + (int)(item - (int64_t)h * nblk);
  int s = __builtin_amdgcn_readfirstlane(block_start[i]);
  int e = __builtin_amdgcn_readfirstlane(block_start[i + 1]);
  const unsigned ustride = (unsigned)stride_tok;
  for (;;) {
    // the bounds of this wave's next item travel with the rows of the current one
    const int64_t nitem = item + nwaves;
    const int64_t pitem = nitem < items ? nitem : item;
    const int nh = (int)(pitem / nblk);
    const int ni = i_lo + (int)(pitem - (int64_t)nh * nblk);
    const int ns = __builtin_amdgcn_readfirstlane(block_start[ni]);
    const int ne = __builtin_amdgcn_readfirstlane(block_start[ni + 1]);
    const int len = e - s;
    uint16_t* o = out + ((int64_t)h * out_rows + i) * (2 * DSK_HEAD_DIM);   // out_rows records per head (>= cap)
    if (s < 0 || len <= 0 || e > total_tokens) {   // malformed table: defined output, flag it
      if (lane < 32) reinterpret_cast<uint4*>(o)[lane] = make_uint4(0, 0, 0, 0);
      if (lane == 0) set_status(dev_status, DSK_ERR_SHAPE);
    } else {
      const uint16_t* base = X + (int64_t)h * stride_head + (int64_t)s * stride_tok;   // uniform
      summarize_block<MEAN>(base, len, stride_tok, ustride, o, g, c);
    }
    if (nitem >= items) break;
    item = nitem; h = nh; i = ni; s = ns; e = ne;
  }
}

template <bool MEAN>
static hipError_t launch_summaries_impl(const dsk_compress_args& a, hipStream_t st) {
  const int64_t max_items = (int64_t)a.Hkv * a.max_blocks_total;
  if (max_items <= 0) return hipSuccess;
  int64_t wgs = (max_items + kSumWaves - 1) / kSumWaves;
  const int64_t max_wgs = 256 * 8;   // 8 workgroups (32 waves) per CU keeps HBM requests deep
  if (wgs > max_wgs) wgs = max_wgs;
  const int out_rows = a.sum_stride_blocks > 0 ? a.sum_stride_blocks : a.max_blocks_total;
  summaries_kernel<MEAN><<<dim3((unsigned)wgs), dim3(kSumThreads), 0, st>>>(
      static_cast<const uint16_t*>(a.K), a.k_stride_tok, a.k_stride_head, a.Hkv, a.block_start,
      a.cu_blocks, a.B, nullptr, a.max_blocks_total, out_rows, a.total_tokens, static_cast<uint16_t*>(a.ksum),
      a.dev_status);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  if (a.vsum != nullptr) {
    summaries_kernel<MEAN><<<dim3((unsigned)wgs), dim3(kSumThreads), 0, st>>>(
        static_cast<const uint16_t*>(a.V), a.v_stride_tok, a.v_stride_head, a.Hkv, a.block_start,
        a.cu_blocks, a.B, nullptr, a.max_blocks_total, out_rows, a.total_tokens, static_cast<uint16_t*>(a.vsum),
        a.dev_status);
    err = hipGetLastError();
  }
  return err;
}

hipError_t launch_summaries(const dsk_compress_args& a, hipStream_t st) {
  return a.summary_mode == DSK_SUMMARY_MEAN ? launch_summaries_impl<true>(a, st) : launch_summaries_impl<false>(a, st);
}

hipError_t launch_summaries_range(const void* X, int64_t stride_tok, int64_t stride_head, int Hkv,
                                  const int32_t* block_start, const int32_t* blk_range, int max_blocks_in_range,
                                  int cap, int total_tokens, int summary_mode, void* out, int32_t* dev_status,
                                  hipStream_t st) {
  const int64_t max_items = (int64_t)Hkv * max_blocks_in_range;
  if (max_items <= 0) return hipSuccess;
  int64_t wgs = (max_items + kSumWaves - 1) / kSumWaves;
  if (wgs > 256 * 8) wgs = 256 * 8;
  if (summary_mode == DSK_SUMMARY_MEAN)
    summaries_kernel<true><<<dim3((unsigned)wgs), dim3(kSumThreads), 0, st>>>(
        static_cast<const uint16_t*>(X), stride_tok, stride_head, Hkv, block_start, nullptr, 0, blk_range, cap, cap,
        total_tokens, static_cast<uint16_t*>(out), dev_status);
  else
    summaries_kernel<false><<<dim3((unsigned)wgs), dim3(kSumThreads), 0, st>>>(
        static_cast<const uint16_t*>(X), stride_tok, stride_head, Hkv, block_start, nullptr, 0, blk_range, cap, cap,
        total_tokens, static_cast<uint16_t*>(out), dev_status);
  return hipGetLastError();
}

// Summaries of the blocks a batched incremental update rewrote.  ranges[s] = {first rewritten
// entry, end, first K/V row of sequence s, its length}; block_start counts from the sequence's first
// token.  grid: (rewritten block, sequence, group of kSumWaves heads): one wavefront per head.
template <bool MEAN>
__global__ __launch_bounds__(kSumThreads) void summaries_batch_ranges_kernel(
    const uint16_t* __restrict__ X, int64_t stride_tok, int64_t stride_head, int Hkv,
    const int32_t* __restrict__ block_start, const int4* __restrict__ ranges, int out_rows,
    uint16_t* __restrict__ out, int32_t* dev_status) {
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DSK_WAVE);
  const int g = lane >> 4, c = lane & 15;
  const int4 rg = ranges[blockIdx.y];
  const int i = rg.x + (int)blockIdx.x;
  if (i >= rg.y || i >= out_rows) return;
  const int s = __builtin_amdgcn_readfirstlane(block_start[i]);
  const int e = __builtin_amdgcn_readfirstlane(block_start[i + 1]);
  const int len = e - s;
  const int h = (int)blockIdx.z * kSumWaves + wave;
  if (h < Hkv) {
    uint16_t* o = out + ((int64_t)h * out_rows + i) * (2 * DSK_HEAD_DIM);
    if (s < 0 || len <= 0 || e > rg.w) {           // malformed table: defined output, flag it
      if (lane < 32) reinterpret_cast<uint4*>(o)[lane] = make_uint4(0, 0, 0, 0);
      if (lane == 0) set_status(dev_status, DSK_ERR_SHAPE);
    } else {
      const uint16_t* base = X + (int64_t)h * stride_head + ((int64_t)rg.z + s) * stride_tok;
      summarize_block<MEAN>(base, len, stride_tok, (unsigned)stride_tok, o, g, c);
    }
  }
}

hipError_t launch_summaries_batch_ranges(const void* X, int64_t stride_tok, int64_t stride_head, int Hkv, int B,
                                         const int32_t* block_start, const void* ranges, int max_blocks_in_range,
                                         int out_rows, int summary_mode, void* out, int32_t* dev_status,
                                         hipStream_t st) {
  if (max_blocks_in_range <= 0 || B <= 0) return hipSuccess;
  const dim3 grid((unsigned)max_blocks_in_range, (unsigned)B, (unsigned)((Hkv + kSumWaves - 1) / kSumWaves));
  if (summary_mode == DSK_SUMMARY_MEAN)
    summaries_batch_ranges_kernel<true><<<grid, dim3(kSumThreads), 0, st>>>(
        static_cast<const uint16_t*>(X), stride_tok, stride_head, Hkv, block_start, static_cast<const int4*>(ranges),
        out_rows, static_cast<uint16_t*>(out), dev_status);
  else
    summaries_batch_ranges_kernel<false><<<grid, dim3(kSumThreads), 0, st>>>(
        static_cast<const uint16_t*>(X), stride_tok, stride_head, Hkv, block_start, static_cast<const int4*>(ranges),
        out_rows, static_cast<uint16_t*>(out), dev_status);
  return hipGetLastError();
}

}  // namespace dsk
