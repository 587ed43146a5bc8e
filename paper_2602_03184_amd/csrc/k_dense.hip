// Full attention of a decode query over the whole cache: the full-KV baseline of the latency
// comparison (Sec. 5, GPU Inference analysis, Figure 8).  Split-K flash-decode with the same
// row fold as the sparse gather kernel; HBM-bound (every K/V byte once), so no MFMA: at
// Hq/Hkv = 4 it is 4 flop per byte, a sixth of what the vector ALUs deliver at that byte rate.
// A workgroup owns a contiguous token range of one (sequence, KV head) and folds GT query heads
// of the GQA group against every 32-row tile it loads, so that K and V are read once per group.
#include "dsk_attn_fold.hpp"
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kDenseWaves = 4;
constexpr int kDenseThreads = kDenseWaves * DSK_WAVE;
constexpr int kDenseStep = kDenseWaves * 32;              // token ranges are multiples of this

template <int GT, int NS>
__global__ __launch_bounds__(kDenseThreads) void dense_attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    int64_t kst, int64_t ksh, int64_t vst, int64_t vsh, int Hq, int G, int total_tokens,
    const int32_t* __restrict__ cu_seqlens, int tokens_per_split, int nsplit, float scale_log2,
    float2* __restrict__ part_ml, float* __restrict__ part_acc, float* __restrict__ out,
    uint16_t* __restrict__ out_bf16, float* __restrict__ lse) {
  __shared__ float sm_m[kDenseWaves];
  __shared__ float sm_l[kDenseWaves];
  __shared__ float sm_acc[kDenseWaves][DSK_HEAD_DIM];

  const int split = blockIdx.x;
  const int tiles_g = (G + GT - 1) / GT;          // passes over K/V per KV head
  const int hk = blockIdx.y / tiles_g;
  const int g0 = (blockIdx.y - hk * tiles_g) * GT;  // first query head of the group in this pass
  const int s = blockIdx.z;
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int grp = lane >> 4;
  const int c = lane & 15;

  const int seq0 = cu_seqlens[s];
  int L = cu_seqlens[s + 1] - seq0;
  if (seq0 < 0 || L < 0 || seq0 > total_tokens - L) L = 0;     // malformed table: treated as empty
  // the host's max_seqlen sized the split: a longer sequence on the device is cut to the tokens the
  // nsplit ranges cover, so that the merge finds exactly the partials that were written
  if (L > nsplit * (int64_t)tokens_per_split) L = nsplit * tokens_per_split;
  const int ng = (G - g0 < GT) ? G - g0 : GT;                  // heads of this pass that exist
  if (L <= 0) {
    if (split == 0 && threadIdx.x < DSK_HEAD_DIM) {
      for (int j = 0; j < ng; ++j) {
        const int64_t sh = (int64_t)s * Hq + hk * G + g0 + j;
        store_attn_out(out, out_bf16, sh * DSK_HEAD_DIM + threadIdx.x, 0.0f);
        if (threadIdx.x == 0 && lse) lse[sh] = -__builtin_inff();
      }
    }
    return;
  }
  const int t0 = split * tokens_per_split;
  if (t0 >= L) return;                                         // uniform over the workgroup
  const int t1 = t0 + tokens_per_split < L ? t0 + tokens_per_split : L;
  const int used = (L + tokens_per_split - 1) / tokens_per_split;

  QRow qf[GT];
  WaveState st[GT];
#pragma unroll
  for (int j = 0; j < GT; ++j) {
    const int gq = g0 + (j < ng ? j : 0);                      // absent heads shadow head g0, never written
    const uint4 qv = *reinterpret_cast<const uint4*>(q + ((int64_t)s * Hq + hk * G + gq) * DSK_HEAD_DIM + c * 8);
    qf[j] = make_qrow(qv);
    st[j].m = -__builtin_inff();
    st[j].l = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) st[j].acc[i] = 0.0f;
  }
  const uint16_t* Kh = K + (int64_t)hk * ksh + (int64_t)seq0 * kst + c * 8;
  const uint16_t* Vh = V + (int64_t)hk * vsh + (int64_t)seq0 * vst + c * 8;

  constexpr int kTile = 4 * NS;                                // rows a wavefront loads at once
  for (int r0 = t0 + wave * kTile; r0 < t1; r0 += kDenseWaves * kTile) {
    const int nvalid = t1 - r0 < kTile ? t1 - r0 : kTile;
    uint4 kv[NS], vv[NS];
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      int r = 4 * u + grp;
      r = r < nvalid ? r : nvalid - 1;                         // padding rows re-read a real row
      kv[u] = *reinterpret_cast<const uint4*>(Kh + (int64_t)(r0 + r) * kst);
    }
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      int r = 4 * u + grp;
      r = r < nvalid ? r : nvalid - 1;
      vv[u] = *reinterpret_cast<const uint4*>(Vh + (int64_t)(r0 + r) * vst);
    }
#pragma unroll
    for (int j = 0; j < GT; ++j) fold_loaded<NS>(st[j], qf[j], kv, vv, nvalid, grp, scale_log2);
  }

  // per head: lane groups -> wave -> workgroup partial, fixed order
#pragma unroll
  for (int j = 0; j < GT; ++j) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      st[j].acc[i] += shfl_xor_f(st[j].acc[i], 16);
      st[j].acc[i] += shfl_xor_f(st[j].acc[i], 32);
    }
    st[j].l += shfl_xor_f(st[j].l, 16);
    st[j].l += shfl_xor_f(st[j].l, 32);
    if (j > 0) __syncthreads();                                // the previous head's reads are done
    if (lane == 0) { sm_m[wave] = st[j].m; sm_l[wave] = st[j].l; }
    if (grp == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) sm_acc[wave][c * 8 + i] = st[j].acc[i];
    }
    __syncthreads();
    const int d = threadIdx.x;
    if (d < DSK_HEAD_DIM && j < ng) {
      float M = sm_m[0];
#pragma unroll
      for (int w = 1; w < kDenseWaves; ++w) M = fmaxf(M, sm_m[w]);
      float l = 0.0f, a = 0.0f;
#pragma unroll
      for (int w = 0; w < kDenseWaves; ++w) {
        const float f = sm_m[w] == -__builtin_inff() ? 0.0f : exp2f(sm_m[w] - M);   // wave without rows
        l = fmaf(sm_l[w], f, l);
        a = fmaf(sm_acc[w][d], f, a);
      }
      const int64_t sh = (int64_t)s * Hq + hk * G + g0 + j;
      if (used == 1) {
        store_attn_out(out, out_bf16, sh * DSK_HEAD_DIM + d, l > 0.0f ? a / l : 0.0f);
        if (d == 0 && lse) lse[sh] = l > 0.0f ? (M + log2f(l)) * kLn2 : -__builtin_inff();
      } else {
        const int64_t p = sh * nsplit + split;
        part_acc[p * DSK_HEAD_DIM + d] = a;
        if (d == 0) part_ml[p] = make_float2(M, l);
      }
    }
  }
}

DenseWs dense_ws_layout(const dsk_dense_attn_args& a) {
  DenseWs ws;
  const int G = a.Hq / a.Hkv;
  ws.group_tile = (G % 4 == 0) ? 4 : (G % 2 == 0 ? 2 : 1);
  const int64_t passes = (int64_t)a.B * a.Hkv * ((G + ws.group_tile - 1) / ws.group_tile);
  // about 4096 workgroups (16 per CU) when the cache is long enough, 128 tokens at least each;
  // at most kDenseMaxSplit ranges per sequence, since the merge runs one workgroup per head and
  // its time grows with the partials it reads (measured: 32 beats 16, 24, 64, 128 and 256 at
  // batch 1 with 32K and 128K tokens)
  constexpr int64_t kDenseMaxSplit = 32;
  int64_t want_split = (4096 + passes - 1) / passes;
  if (want_split < 1) want_split = 1;
  if (want_split > kDenseMaxSplit) want_split = kDenseMaxSplit;
  int64_t tps = ((int64_t)a.max_seqlen + want_split - 1) / want_split;
  tps = (tps + kDenseStep - 1) / kDenseStep * kDenseStep;
  if (tps < kDenseStep) tps = kDenseStep;
  ws.tokens_per_split = (int)tps;
  ws.nsplit = (int)(((int64_t)a.max_seqlen + tps - 1) / tps);
  if (ws.nsplit < 1) ws.nsplit = 1;
  const size_t n = (size_t)a.B * a.Hq * ws.nsplit;
  ws.part_ml = 0;
  ws.part_acc = align_up(n * sizeof(float2));
  ws.total = ws.part_acc + align_up(n * DSK_HEAD_DIM * sizeof(float));
  return ws;
}

hipError_t launch_dense_attn(const dsk_dense_attn_args& a, const DenseWs& ws, hipStream_t st) {
  unsigned char* w = static_cast<unsigned char*>(a.workspace);
  float2* part_ml = reinterpret_cast<float2*>(w + ws.part_ml);
  float* part_acc = reinterpret_cast<float*>(w + ws.part_acc);
  const float scale = a.scale != 0.0f ? a.scale : 0.08838834764831845f;   // 128^-1/2
  const int G = a.Hq / a.Hkv;
  const int tiles_g = (G + ws.group_tile - 1) / ws.group_tile;
  const dim3 grid((unsigned)ws.nsplit, (unsigned)(a.Hkv * tiles_g), (unsigned)a.B);
  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  const uint16_t* K = static_cast<const uint16_t*>(a.K);
  const uint16_t* V = static_cast<const uint16_t*>(a.V);
#define DSK_DENSE_ARGS                                                                                        \
  q, K, V, a.k_stride_tok, a.k_stride_head, a.v_stride_tok, a.v_stride_head, a.Hq, G, a.total_tokens,         \
      a.cu_seqlens, ws.tokens_per_split, ws.nsplit, scale * kLog2e, part_ml, part_acc, a.out,         \
      static_cast<uint16_t*>(a.out_bf16), a.lse
  // 32-row tiles: 16- and 8-row tiles raise occupancy but were measured slower (the per-tile
  // rescale of four heads' states is vector-ALU work the kernel has little room for)
  if (ws.group_tile == 4) dense_attn_kernel<4, 8><<<grid, dim3(kDenseThreads), 0, st>>>(DSK_DENSE_ARGS);
  else if (ws.group_tile == 2) dense_attn_kernel<2, 8><<<grid, dim3(kDenseThreads), 0, st>>>(DSK_DENSE_ARGS);
  else dense_attn_kernel<1, 8><<<grid, dim3(kDenseThreads), 0, st>>>(DSK_DENSE_ARGS);
#undef DSK_DENSE_ARGS
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || ws.nsplit <= 1) return err;
  return launch_attn_merge(part_ml, part_acc, nullptr, a.cu_seqlens, a.B, a.Hq, 1, 0x7FFFFFFF, ws.nsplit,
                           ws.tokens_per_split, a.out, static_cast<uint16_t*>(a.out_bf16), a.lse, st);
}

}  // namespace dsk
