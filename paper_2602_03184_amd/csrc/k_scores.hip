// Block scores (Sec. 4.2, Top-k Block Selection; App. B.2 Step 1):
//   score[hq, i] = sum_d max(q_d*kmax[hk,i,d], q_d*kmin[hk,i,d]) = q+ . kmax + q- . kmin
// with q+ = max(q,0), q- = min(q,0): one dot product of length 2D against the 512-byte
// (min,max) summary of the block.  Memory-bound: every summary is read once per step and
// shared by the G query heads of its KV head.  A half-wavefront (32 lanes x 16 B) covers one
// summary; it takes 8 (4 for G = 8) consecutive blocks, issues all their loads first, and
// reduces the blocks x heads partial sums over its 32 lanes with a transposing butterfly
// (each exchange halves the values a lane still carries), so a lane ends up owning the
// finished score of one (block, head) pair.
#include "dsk_attn_fold.hpp"
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kScoreThreads = 256;
constexpr int kHalvesPerWg = kScoreThreads / 32;
__host__ __device__ constexpr int score_blocks_per_half(int G) { return G >= 8 ? 4 : 8; }

// value of lane (lane ^ M) of the same half-wave: on the vector ALU's data-parallel path for
// M < 16 (quad permutes and row mirrors; a mirror of 8 followed by a reversal inside quads flips
// lane bit 2, a mirror of 16 followed by a mirror of 8 flips bit 3), through the LDS crossbar for 16
constexpr int kDppQuadReverse = 0x1B;  // quad_perm [3,2,1,0]
template <int M>
__device__ __forceinline__ float xchg_half_wave(float v) {
  if constexpr (M == 1) return dpp_f<kDppSwap1>(v);
  else if constexpr (M == 2) return dpp_f<kDppSwap2>(v);
  else if constexpr (M == 4) return dpp_f<kDppQuadReverse>(dpp_f<kDppHalfMirror>(v));
  else if constexpr (M == 8) return dpp_f<kDppHalfMirror>(dpp_f<kDppMirror>(v));
  else return shfl_xor_f(v, M);
}

// Sum V (a power of two, <= 32) per-lane values over the 32 lanes of a half-wave.  While more
// than one value is left, a step over lane bit M halves them: the lane keeps the upper half of
// the value indices if its bit M is set (the lower half otherwise) and adds what its partner
// (lane ^ M) carried for that half; afterwards plain exchanges finish the sum.  Steps run from
// lane bit 0 upwards, so that the steps with many values to exchange are the cheap ones.  On
// return v[0] is the finished sum of original value index `idx` (built MSB-first from the lane
// bits of the halving steps, i.e. from the low log2(V) lane bits, bit 0 first).
template <int N, int V, int M>
__device__ __forceinline__ void half_wave_reduce(float (&v)[N], int lane, int& idx) {
  if constexpr (M <= 16) {
    if constexpr (V >= 2) {
      const bool up = (lane & M) != 0;
#pragma unroll
      for (int x = 0; x < V / 2; ++x) {
        const float send = up ? v[x] : v[x + V / 2];
        const float keep = up ? v[x + V / 2] : v[x];
        v[x] = keep + xchg_half_wave<M>(send);
      }
      idx = idx * 2 + (up ? 1 : 0);
      half_wave_reduce<N, V / 2, M * 2>(v, lane, idx);
    } else {
      v[0] += xchg_half_wave<M>(v[0]);
      half_wave_reduce<N, 1, M * 2>(v, lane, idx);
    }
  }
}

// value index = block_in_group * G + g.  GROUPMAX: one row per KV head, the largest of the G
// heads' scores (selection shared by the group); the G values of a block sit in lanes that
// differ only in log2(G) consecutive lane bits, so the maximum is a few exchanges.
template <int G, bool GROUPMAX = false>
__global__ __launch_bounds__(kScoreThreads) void scores_kernel(
    const uint16_t* __restrict__ ksum, const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_blocks,
    const int32_t* __restrict__ blocks_used, int B, int Hq, int cap, int bound, int stride,
    float* __restrict__ scores, float* __restrict__ user) {
  constexpr int NB = score_blocks_per_half(G);
  constexpr int V = NB * G;
  static_assert(V <= 32 && (V & (V - 1)) == 0, "one finished value per lane");
  const int hk = blockIdx.y;
  const int half = threadIdx.x >> 5;          // 0..7 within the workgroup
  const int c = threadIdx.x & 31;             // 16-byte column of the summary
  const bool is_max = c >= 16;                // lanes 0-15: kmin, 16-31: kmax
  const int d0 = (c & 15) * 8;
  const int i0 = (blockIdx.x * kHalvesPerWg + half) * NB;   // first block of this half-wave
  const uint16_t* kh = ksum + (int64_t)hk * cap * (2 * DSK_HEAD_DIM) + c * 8;

  // Tables with a region per sequence: the entries between a sequence's last block and the next
  // region hold no summary.  A half-wave whose blocks all lie in such a gap leaves before it loads
  // anything (one round trip for the region bounds, taken in this layout only); what a straddling
  // group computes for gap entries is never read by the selection.
  if (blocks_used != nullptr && B <= 32) {
    const int cs = c < B ? c : B - 1;
    const int st_c = cu_blocks[cs];
    const int end_c = st_c + blocks_used[cs];
    const int hs = threadIdx.x & 32;
    const int sq = __popcll((__ballot(c < B && st_c <= i0) >> hs) & 0xFFFFFFFFull) - 1;   // region of block i0
    if (sq >= 0) {
      const int end = __shfl(end_c, hs + sq, DSK_WAVE);
      const int next = sq + 1 < B ? __shfl(st_c, hs + sq + 1, DSK_WAVE) : 0x7FFFFFFF;
      if (i0 >= end && i0 + NB - 1 < next) return;
    }
  }

  // Sequence starts 1..32 and the block count go out first: loads return in order, so their
  // values can be used while the summaries issued behind them are still in flight.
  const int start_first = cu_blocks[1 + c < B ? 1 + c : B];
  int nblk = cu_blocks[B];
  // `bound` (<= cap) is the host's upper bound on the block count: the summary loads are
  // addressed without waiting for the device's count, all NB of them in flight together
  uint4 kv[NB];
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    int i = i0 + u;
    i = i < bound ? i : bound - 1;            // past the end: re-read the last record, result dropped
    kv[u] = *reinterpret_cast<const uint4*>(kh + (int64_t)i * (2 * DSK_HEAD_DIM));
  }
  if (nblk > bound) nblk = bound;
  // sequence of the group (blocks of a sequence are contiguous; a group rarely straddles two):
  // number of sequence starts at or before its first / last block, counted by the 32 lanes of
  // the half-wave at once
  const int ilast = (i0 + NB - 1 < nblk) ? i0 + NB - 1 : nblk - 1;
  const int half_shift = threadIdx.x & 32;    // this half-wave's 32 bits of a ballot
  int s_first, s_last;
  {
    const bool have = 1 + c < B;
    s_first = __popcll((__ballot(have && start_first <= i0) >> half_shift) & 0xFFFFFFFFull);
    s_last = __popcll((__ballot(have && start_first <= ilast) >> half_shift) & 0xFFFFFFFFull);
  }
  // queries of that sequence (exact when B <= 33; corrected below otherwise)
  uint4 qv[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qv[g] = *reinterpret_cast<const uint4*>(q + ((int64_t)s_first * Hq + hk * G + g) * DSK_HEAD_DIM + d0);
#pragma unroll
  for (int u = 0; u < NB; ++u) pin_loaded(kv[u]);
#pragma unroll
  for (int g = 0; g < G; ++g) pin_loaded(qv[g]);
  if (i0 >= nblk) return;                     // whole half-waves leave together
  if (B > 33) {                               // more sequence starts than one ballot covers
    const int s_before = s_first;
    for (int sb = 33; sb < B; sb += 32) {
      const int sidx = sb + c;
      const int start = cu_blocks[sidx < B ? sidx : B];
      const bool have = sidx < B;
      s_first += __popcll((__ballot(have && start <= i0) >> half_shift) & 0xFFFFFFFFull);
      s_last += __popcll((__ballot(have && start <= ilast) >> half_shift) & 0xFFFFFFFFull);
    }
    if (s_first != s_before) {
#pragma unroll
      for (int g = 0; g < G; ++g)
        qv[g] = *reinterpret_cast<const uint4*>(q + ((int64_t)s_first * Hq + hk * G + g) * DSK_HEAD_DIM + d0);
    }
  }
  // One pass per sequence the group touches (nearly always one): the group's summaries stay in
  // registers, only the queries change, and a pass writes the blocks of its own sequence.  The
  // summation tree is the same in every pass, so a block's score does not depend on the batch
  // it was computed in.
  int s = s_first;
  int cur = i0;                                // first block not yet written
  for (;;) {
    int seg_end = ilast + 1;
    if (s != s_last) {                         // the sequence ends inside the group
      seg_end = cu_blocks[s + 1];
      seg_end = seg_end < ilast + 1 ? seg_end : ilast + 1;
    }
    if (seg_end > cur) {
      // q+ (lanes holding kmax) or q- (lanes holding kmin) as packed bf16 pairs: the halves whose
      // sign does not fit are zeroed, both are exact in bf16; the products then run on the packed
      // bf16 dot instruction with neither operand widened
      uint32_t qp[G][4];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const uint32_t wds[4] = {qv[g].x, qv[g].y, qv[g].z, qv[g].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t neg = ((uint32_t)((int32_t)(wds[k] << 16) >> 31) & 0xFFFFu) |
                               ((uint32_t)((int32_t)wds[k] >> 31) & 0xFFFF0000u);   // ones over negative halves
          qp[g][k] = wds[k] & (is_max ? ~neg : neg);
        }
      }
      float v[V];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float acc = dot2_bf16(qp[g][0], kv[u].x, 0.0f);
          acc = dot2_bf16(qp[g][1], kv[u].y, acc);
          acc = dot2_bf16(qp[g][2], kv[u].z, acc);
          v[u * G + g] = dot2_bf16(qp[g][3], kv[u].w, acc);
        }
      }
      int idx = 0;
      half_wave_reduce<V, V, 1>(v, c, idx);
      const bool writer = c < V;                     // lanes differing only in non-halving (high) bits hold copies
      const int u = idx / G, g = idx % G;
      if constexpr (GROUPMAX) {
        // the G heads of a block: value indices that differ in their low log2(G) bits, i.e. lanes
        // that differ in lane bits log2(V / G) .. log2(V) - 1
        float best = v[0];
#pragma unroll
        for (int m = V / G; m < V; m <<= 1) best = fmaxf(best, shfl_xor_f(best, m));
        if (writer && g == 0 && i0 + u >= cur && i0 + u < seg_end) {
          scores[(int64_t)hk * stride + i0 + u] = best;
          if (user) user[(int64_t)hk * cap + i0 + u] = best;
        }
      } else if (writer && i0 + u >= cur && i0 + u < seg_end) {
        scores[(int64_t)(hk * G + g) * stride + i0 + u] = v[0];
        if (user) user[(int64_t)(hk * G + g) * cap + i0 + u] = v[0];
      }
      cur = seg_end;
    }
    if (s == s_last) break;
    ++s;
#pragma unroll
    for (int g = 0; g < G; ++g)
      qv[g] = *reinterpret_cast<const uint4*>(q + ((int64_t)s * Hq + hk * G + g) * DSK_HEAD_DIM + d0);
  }
}

// any group width: one block per half-wave step, q re-read per block (it stays in the vector cache)
__global__ __launch_bounds__(kScoreThreads) void scores_kernel_anyg(
    const uint16_t* __restrict__ ksum, const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_blocks,
    int B, int Hq, int G, int cap, int stride, bool group_max, float* __restrict__ scores,
    float* __restrict__ user) {
  const int hk = blockIdx.y;
  int nblk = cu_blocks[B];
  if (nblk > cap) nblk = cap;
  const int half = threadIdx.x >> 5;
  const int c = threadIdx.x & 31;
  const bool is_max = c >= 16;
  const int d0 = (c & 15) * 8;
  const int first = (blockIdx.x * kHalvesPerWg + half) * 8;
  const uint16_t* kh = ksum + (int64_t)hk * cap * (2 * DSK_HEAD_DIM);
  int s = 0;
  for (int it = 0; it < 8; ++it) {
    const int i = first + it;
    if (i >= nblk) break;
    while (s + 1 < B && cu_blocks[s + 1] <= i) ++s;
    const uint4 kv = *reinterpret_cast<const uint4*>(kh + (int64_t)i * (2 * DSK_HEAD_DIM) + c * 8);
    float f[8];
    unpack8(kv, f);
    float best = -__builtin_inff();
    for (int g = 0; g < G; ++g) {
      const uint4 qv = *reinterpret_cast<const uint4*>(q + ((int64_t)s * Hq + hk * G + g) * DSK_HEAD_DIM + d0);
      float qf[8];
      unpack8(qv, qf);
      float acc = 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = fmaf(is_max ? fmaxf(qf[k], 0.0f) : fminf(qf[k], 0.0f), f[k], acc);
      acc = group16_sum(acc);
      acc += shfl_xor_f(acc, 16);
      best = fmaxf(best, acc);
      if (c == 0 && !group_max) {
        scores[(int64_t)(hk * G + g) * stride + i] = acc;
        if (user) user[(int64_t)(hk * G + g) * cap + i] = acc;
      }
    }
    if (c == 0 && group_max) {
      scores[(int64_t)hk * stride + i] = best;
      if (user) user[(int64_t)hk * cap + i] = best;
    }
  }
}

hipError_t launch_scores(const dsk_select_args& a, float* scores, int stride, hipStream_t st) {
  if (a.max_blocks_total <= 0) return hipSuccess;
  const int G = a.Hq / a.Hkv;
  const int per_wg = kHalvesPerWg * score_blocks_per_half(G);
  const int bound = a.max_blocks_used > 0 ? a.max_blocks_used : a.max_blocks_total;
  const dim3 grid((unsigned)((bound + per_wg - 1) / per_wg), (unsigned)a.Hkv);
  const dim3 block(kScoreThreads);
  const uint16_t* ksum = static_cast<const uint16_t*>(a.ksum);
  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  const bool shared = (a.flags & DSK_SELECT_SHARED_BY_KV_GROUP) != 0 && G > 1;
#define DSK_SCORE_ARGS ksum, q, a.cu_blocks, a.blocks_used, a.B, a.Hq, a.max_blocks_total, bound, stride, scores, a.scores
  switch (shared ? -G : G) {
    case 1: scores_kernel<1><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    case 2: scores_kernel<2><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    case 4: scores_kernel<4><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    case 8: scores_kernel<8><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    case -2: scores_kernel<2, true><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    case -4: scores_kernel<4, true><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    case -8: scores_kernel<8, true><<<grid, block, 0, st>>>(DSK_SCORE_ARGS); break;
    default:
      scores_kernel_anyg<<<grid, block, 0, st>>>(ksum, q, a.cu_blocks, a.B, a.Hq, G, a.max_blocks_total, stride, shared,
                                                 scores, a.scores);
  }
#undef DSK_SCORE_ARGS
  return hipGetLastError();
}

}  // namespace dsk
