// Block scores (Sec. 4.2, Top-k Block Selection; App. B.2 Step 1):
//   score[hq, i] = sum_d max(q_d*kmax[hk,i,d], q_d*kmin[hk,i,d]) = q+ . kmax + q- . kmin
// with q+ = max(q,0), q- = min(q,0): one dot product of length 2D against the 512-byte
// (min,max) summary of the block.  Memory-bound: every summary is read once per step and
// shared by the G query heads of its KV head.  A half-wavefront (32 lanes x 16 B) covers one
// summary, so a wavefront scores two blocks per load.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kScoreThreads = 256;
constexpr int kScoreBlocksPerWg = 64;   // 4 waves x 2 half-waves x 8 blocks

template <int G>
__global__ __launch_bounds__(kScoreThreads) void scores_kernel(
    const uint16_t* __restrict__ ksum, const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_blocks,
    int B, int Hq, int cap, float* __restrict__ scores) {
  const int hk = blockIdx.y;
  int nblk = cu_blocks[B];
  if (nblk > cap) nblk = cap;
  const int half = threadIdx.x >> 5;          // 0..7 within the workgroup
  const int c = threadIdx.x & 31;             // 16-byte column of the summary
  const int is_max = c >> 4;                  // lanes 0-15: kmin, 16-31: kmax
  const int d0 = (c & 15) * 8;
  const int first = blockIdx.x * kScoreBlocksPerWg;
  const uint16_t* kh = ksum + (int64_t)hk * cap * (2 * DSK_HEAD_DIM);

  int cur_s = -1;
  float qs[G][8];
  for (int it = 0; it < kScoreBlocksPerWg / 8; ++it) {
    const int i = first + it * 8 + half;      // all 32 lanes of a half-wave share i
    if (i >= nblk) break;
    // sequence of block i (blocks of a sequence are contiguous)
    int s = cur_s < 0 ? 0 : cur_s;
    while (s + 1 < B && cu_blocks[s + 1] <= i) ++s;
    if (s != cur_s) {
      cur_s = s;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const uint4 qv = *reinterpret_cast<const uint4*>(q + ((int64_t)s * Hq + hk * G + g) * DSK_HEAD_DIM + d0);
        float f[8];
        unpack8(qv, f);
#pragma unroll
        for (int k = 0; k < 8; ++k) qs[g][k] = is_max ? fmaxf(f[k], 0.0f) : fminf(f[k], 0.0f);
      }
    }
    const uint4 kv = *reinterpret_cast<const uint4*>(kh + (int64_t)i * (2 * DSK_HEAD_DIM) + c * 8);
    float f[8];
    unpack8(kv, f);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float acc = 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = fmaf(qs[g][k], f[k], acc);
      acc = group16_sum(acc);
      acc += shfl_xor_f(acc, 16);
      if (c == 0) scores[(int64_t)(hk * G + g) * cap + i] = acc;
    }
  }
}

// any group width: q is re-read per block (it stays in the vector cache)
__global__ __launch_bounds__(kScoreThreads) void scores_kernel_anyg(
    const uint16_t* __restrict__ ksum, const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_blocks,
    int B, int Hq, int G, int cap, float* __restrict__ scores) {
  const int hk = blockIdx.y;
  int nblk = cu_blocks[B];
  if (nblk > cap) nblk = cap;
  const int half = threadIdx.x >> 5;
  const int c = threadIdx.x & 31;
  const int is_max = c >> 4;
  const int d0 = (c & 15) * 8;
  const int first = blockIdx.x * kScoreBlocksPerWg;
  const uint16_t* kh = ksum + (int64_t)hk * cap * (2 * DSK_HEAD_DIM);
  int s = 0;
  for (int it = 0; it < kScoreBlocksPerWg / 8; ++it) {
    const int i = first + it * 8 + half;
    if (i >= nblk) break;
    while (s + 1 < B && cu_blocks[s + 1] <= i) ++s;
    const uint4 kv = *reinterpret_cast<const uint4*>(kh + (int64_t)i * (2 * DSK_HEAD_DIM) + c * 8);
    float f[8];
    unpack8(kv, f);
    for (int g = 0; g < G; ++g) {
      const uint4 qv = *reinterpret_cast<const uint4*>(q + ((int64_t)s * Hq + hk * G + g) * DSK_HEAD_DIM + d0);
      float qf[8];
      unpack8(qv, qf);
      float acc = 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = fmaf(is_max ? fmaxf(qf[k], 0.0f) : fminf(qf[k], 0.0f), f[k], acc);
      acc = group16_sum(acc);
      acc += shfl_xor_f(acc, 16);
      if (c == 0) scores[(int64_t)(hk * G + g) * cap + i] = acc;
    }
  }
}

hipError_t launch_scores(const dsk_select_args& a, float* scores, hipStream_t st) {
  if (a.max_blocks_total <= 0) return hipSuccess;
  const int G = a.Hq / a.Hkv;
  const dim3 grid((unsigned)((a.max_blocks_total + kScoreBlocksPerWg - 1) / kScoreBlocksPerWg), (unsigned)a.Hkv);
  const dim3 block(kScoreThreads);
  const uint16_t* ksum = static_cast<const uint16_t*>(a.ksum);
  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  switch (G) {
    case 1: scores_kernel<1><<<grid, block, 0, st>>>(ksum, q, a.cu_blocks, a.B, a.Hq, a.max_blocks_total, scores); break;
    case 2: scores_kernel<2><<<grid, block, 0, st>>>(ksum, q, a.cu_blocks, a.B, a.Hq, a.max_blocks_total, scores); break;
    case 4: scores_kernel<4><<<grid, block, 0, st>>>(ksum, q, a.cu_blocks, a.B, a.Hq, a.max_blocks_total, scores); break;
    case 8: scores_kernel<8><<<grid, block, 0, st>>>(ksum, q, a.cu_blocks, a.B, a.Hq, a.max_blocks_total, scores); break;
    default:
      scores_kernel_anyg<<<grid, block, 0, st>>>(ksum, q, a.cu_blocks, a.B, a.Hq, G, a.max_blocks_total, scores);
  }
  return hipGetLastError();
}

}  // namespace dsk
