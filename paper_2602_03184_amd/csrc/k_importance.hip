// Delimiter importance via attention dependency (Alg. 1 and the equation of Sec. 3) on one
// layer, for the sampled candidates, followed by the class-mean -> weight-in-tenths map.
//
// For a sampled candidate at position t the W queries that follow it, for the G query heads of
// one KV head, form a [W*G x D] block; its logits against keys 0..t+W are a real dense
// contraction, so they run on the matrix cores: S^T tile [32 keys x 32 query rows] =
// K tile [32 x 128] . Q^T [128 x 32] as 8 MFMA 32x32x16 bf16 steps.  Keys are the MFMA "A" rows
// so that a lane ends up holding 16 keys of ONE query row: the softmax statistics (running max,
// total mass, mass on the retained region O_t, mass on the discarded region D_t) then
// accumulate per lane with no cross-lane traffic until the very end.  K rows are read straight
// from HBM into the A-operand layout: the contraction index is permuted so that lane half
// hf = lane/32 owns channels [64*hf, 64*hf+64) of its key row, i.e. eight contiguous 16-byte
// loads; Q^T (staged in LDS once per workgroup) is read with the same permutation, so the sum
// over channels is unchanged.  Every key tile a wavefront fetches is multiplied with the query
// windows of 3 or 4 sample slots (fetching a tile per sample made the operand loads, one key row
// per lane, the bound), the next tile is requested before the current one is used, and tiles that
// lie wholly in a sample's discarded region (nearly all of them) take an unmasked path: one running
// sum feeds the total and the discarded mass.  With that a wavefront no longer waits for loads;
// what remains is the vector-ALU work of the running softmax (16 exponentials and about 90 other
// instructions per lane and product, next to 8 MFMAs), two wavefronts per SIMD.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr float kImpLog2e = 1.4426950408889634f;

struct RowStat {       // online-softmax statistics of one query row over a subset of keys
  float m;             // running max of logits (log2 units)
  float zt, zo, zd;    // sum of 2^(z-m): all causal keys, retained region, discarded region
};

__device__ __forceinline__ void stat_merge(RowStat& a, const RowStat& b) {
  const float m = fmaxf(a.m, b.m);
  const float fa = a.m == -__builtin_inff() ? 0.0f : exp2f(a.m - m);
  const float fb = b.m == -__builtin_inff() ? 0.0f : exp2f(b.m - m);
  a.zt = a.zt * fa + b.zt * fb;
  a.zo = a.zo * fa + b.zo * fb;
  a.zd = a.zd * fa + b.zd * fb;
  a.m = m;
}

// Sample slots sharing the key tiles a wavefront loads (consecutive slots: mostly the same class,
// neighbouring positions).  Their Q^T operands live in LDS (rows of 128 channels padded to 136 so
// that the 16-byte reads of 16 consecutive query rows cover all banks), which leaves the registers
// to the key tiles and the statistics.
// 4 slots per group with 8 wavefronts when the launch is small (one sequence: 32 groups x 8 KV heads
// fill the 256 CUs in one round, 90 instead of 118 us at 128 windows), 3 with 4 wavefronts when
// there are many workgroups anyway (4 and 6 were measured there: 617 and 551 against 554 us).
constexpr int kImpQRow = DSK_HEAD_DIM + 8;   // bf16 elements per query row in LDS

// grid: (group of kImpSamples sample slots, kv head, sequence)
template <int kImpThreads, int kImpSamples>
__global__ __launch_bounds__(kImpThreads) void importance_kernel(
    const uint16_t* __restrict__ K, int64_t kst, int64_t ksh, const uint16_t* __restrict__ qwin,
    const int32_t* __restrict__ samp_pos, const int32_t* __restrict__ cu_seqlens, int n_samp, int W, int R,
    int Hq, int G, float alpha, float scale_log2, float* __restrict__ imp_part, int Hkv) {
  constexpr int kImpWaves = kImpThreads / DSK_WAVE;
  __shared__ RowStat sm_stat[kImpSamples][kImpWaves][32];
  __shared__ float sm_val[kImpSamples][32];
  __shared__ __attribute__((aligned(16))) uint16_t sm_q[kImpSamples][32][kImpQRow];
  const int hk = blockIdx.y;
  const int s = blockIdx.z;
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int col = lane & 31;        // query row of the tile this lane accumulates
  const int hf = lane >> 5;         // channel half / key sub-row selector

  const int seq0 = cu_seqlens[s];
  const int L = cu_seqlens[s + 1] - seq0;
  int jn[kImpSamples], t[kImpSamples], o_lo[kImpSamples], d_hi[kImpSamples], last_key[kImpSamples];
  bool have[kImpSamples];
  int n_tiles = 0;
#pragma unroll
  for (int p = 0; p < kImpSamples; ++p) {
    jn[p] = blockIdx.x * kImpSamples + p;
    const int tg = jn[p] < n_samp ? samp_pos[(int64_t)s * n_samp + jn[p]] : -1;
    t[p] = tg - seq0;
    have[p] = tg >= 0 && t[p] >= 0 && t[p] < L;
    if (!have[p]) t[p] = 0;
    o_lo[p] = t[p] - R + 1 > 0 ? t[p] - R + 1 : 0;          // retained region [o_lo, t]
    d_hi[p] = t[p] - R > 0 ? t[p] - R : 0;                  // discarded region [0, d_hi]
    last_key[p] = have[p] ? (t[p] + W < L - 1 ? t[p] + W : L - 1) : -1;
    const int nt = last_key[p] / 32 + 1;
    if (have[p] && nt > n_tiles) n_tiles = nt;
    if (!have[p] && jn[p] < n_samp && threadIdx.x == 0)     // no such sample
      imp_part[((int64_t)s * n_samp + jn[p]) * Hkv + hk] = 0.0f;
  }
  if (n_tiles == 0) return;                                 // uniform over the workgroup
  const int rows = W * G;                                   // query rows of one (sample, kv head)
  const uint16_t* Kh = K + (int64_t)hk * ksh + (int64_t)seq0 * kst + hf * 64;
  float total[kImpSamples];
#pragma unroll
  for (int p = 0; p < kImpSamples; ++p) total[p] = 0.0f;

  for (int row0 = 0; row0 < rows; row0 += 32) {
    // Q^T operands of the group's samples -> LDS: row r of sample p is query row row0 + r (window
    // position w = row / G, head g = row % G), zero for rows or samples that do not exist
    for (int idx = threadIdx.x; idx < kImpSamples * 32 * 16; idx += kImpThreads) {
      const int p = idx / (32 * 16);
      const int r = (idx / 16) & 31;
      const int c16 = idx & 15;
      const int rowq = row0 + r;
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (rowq < rows && have[p]) {
        const int wq_ = rowq / G, gq_ = rowq % G;
        raw = *reinterpret_cast<const uint4*>(
            qwin + ((((int64_t)s * n_samp + jn[p]) * W + wq_) * Hq + hk * G + gq_) * DSK_HEAD_DIM + c16 * 8);
      }
      *reinterpret_cast<uint4*>(&sm_q[p][r][c16 * 8]) = raw;
    }
    const int row = row0 + col;
    const bool row_ok = row < rows;
    const int w = row_ok ? row / G : 0;
    int qpos[kImpSamples];
    RowStat st[kImpSamples];
#pragma unroll
    for (int p = 0; p < kImpSamples; ++p) {
      qpos[p] = t[p] + 1 + w;               // position of this query; attends keys 0..qpos
      st[p].m = -__builtin_inff();
      st[p].zt = st[p].zo = st[p].zd = 0.0f;
    }
    __syncthreads();
    // the rows of the wave's next tile are requested before the current tile is multiplied
    uint4 knext[8];
    {
      int krow = wave * 32 + col;           // A operand row of this lane
      krow = krow < L ? krow : L - 1;       // stay inside the sequence; masked below
      const uint16_t* kp = Kh + (int64_t)krow * kst;
#pragma unroll
      for (int u = 0; u < 8; ++u) knext[u] = *reinterpret_cast<const uint4*>(kp + u * 8);
    }
    for (int tile = wave; tile < n_tiles; tile += kImpWaves) {
      const int k0 = tile * 32;
      uint4 kraw[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) kraw[u] = knext[u];
      {
        int krow = k0 + kImpWaves * 32 + col;
        krow = krow < L ? krow : L - 1;     // past the last tile: a harmless re-read inside the sequence
        const uint16_t* kp = Kh + (int64_t)krow * kst;
#pragma unroll
        for (int u = 0; u < 8; ++u) knext[u] = *reinterpret_cast<const uint4*>(kp + u * 8);
      }
#pragma unroll
      for (int p = 0; p < kImpSamples; ++p) {
        if (k0 > last_key[p]) continue;     // this sample's keys ended before the tile (uniform)
        f32x16_t acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          // lane (col, hf) supplies channels [64*hf + 8u, +8) of query row col
          const bf16x8_t qb = *reinterpret_cast<const bf16x8_t*>(&sm_q[p][col][hf * 64 + u * 8]);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8_t*>(&kraw[u]), qb, acc, 0, 0, 0);
        }
        // acc[r] = logit of key k0 + 8*(r/4) + 4*hf + r%4 against query row `col`
        if (k0 + 31 <= d_hi[p]) {
          // the whole tile lies in the discarded region (hence before every query of the window
          // and outside the retained region): no masks, one sum feeds both totals
          float amax = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) amax = fmaxf(amax, acc[r]);
          const float mn = fmaxf(st[p].m, amax * scale_log2);
          const float f = __builtin_amdgcn_exp2f(st[p].m - mn);   // 0 while st.m is still -inf
          float esum = 0.0f;
#pragma unroll
          for (int r = 0; r < 16; ++r) esum += __builtin_amdgcn_exp2f(fmaf(acc[r], scale_log2, -mn));
          st[p].zt = fmaf(st[p].zt, f, esum);
          st[p].zd = fmaf(st[p].zd, f, esum);
          st[p].zo *= f;
          st[p].m = mn;
          continue;
        }
        float z[16];
        float tmax = -__builtin_inff();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kpos = k0 + 8 * (r / 4) + 4 * hf + (r % 4);
          z[r] = (kpos <= qpos[p] && kpos <= last_key[p]) ? acc[r] * scale_log2 : -__builtin_inff();
          tmax = fmaxf(tmax, z[r]);
        }
        if (tmax != -__builtin_inff()) {
          const float mn = fmaxf(st[p].m, tmax);
          const float f = st[p].m == -__builtin_inff() ? 0.0f : exp2f(st[p].m - mn);
          st[p].zt *= f; st[p].zo *= f; st[p].zd *= f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kpos = k0 + 8 * (r / 4) + 4 * hf + (r % 4);
            const float e = __builtin_amdgcn_exp2f(z[r] - mn);   // z <= mn; 0 for masked keys (-inf)
            st[p].zt += e;
            st[p].zo += (kpos >= o_lo[p] && kpos <= t[p]) ? e : 0.0f;
            st[p].zd += (kpos <= d_hi[p]) ? e : 0.0f;
          }
          st[p].m = mn;
        }
      }
    }
    // halves of a wave hold disjoint keys of the same row; then waves; fixed order
#pragma unroll
    for (int p = 0; p < kImpSamples; ++p) {
      RowStat other;
      other.m = shfl_xor_f(st[p].m, 32);
      other.zt = shfl_xor_f(st[p].zt, 32);
      other.zo = shfl_xor_f(st[p].zo, 32);
      other.zd = shfl_xor_f(st[p].zd, 32);
      if (hf == 0) {
        stat_merge(st[p], other);
        sm_stat[p][wave][col] = st[p];
      }
    }
    __syncthreads();
    if (threadIdx.x < 32 * kImpSamples) {
      const int p = threadIdx.x >> 5;
      RowStat a = sm_stat[p][0][col];
#pragma unroll
      for (int wv = 1; wv < kImpWaves; ++wv) stat_merge(a, sm_stat[p][wv][col]);
      const float v = (row0 + col < rows && a.zt > 0.0f) ? (a.zo - alpha * a.zd) / a.zt : 0.0f;
      sm_val[p][col] = v;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
      for (int p = 0; p < kImpSamples; ++p)
        for (int c2 = 0; c2 < 32; ++c2) total[p] += sm_val[p][c2];   // fixed order
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
#pragma unroll
    for (int p = 0; p < kImpSamples; ++p)
      if (have[p]) imp_part[((int64_t)s * n_samp + jn[p]) * Hkv + hk] = total[p];
  }
}

// one wavefront per (class, sequence), one lane per sample of the class (M <= 64): the lanes sum
// their KV-head partials side by side (same order per sample as a serial loop), lane 0 then adds
// the sample scores in sample order
__global__ __launch_bounds__(DSK_WAVE) void importance_finalize_kernel(
    const float* __restrict__ imp_part, const int32_t* __restrict__ samp_pos, int n_class, int M, int Hkv,
    int Hq, int W, float alpha, uint8_t* __restrict__ class_weight_q, float* __restrict__ class_mean,
    float* __restrict__ samp_score, float* __restrict__ samp_score_sum, int layers) {
  __shared__ float sm_score[kMaxSamplesPerClass];
  __shared__ int sm_have[kMaxSamplesPerClass];
  const int c = blockIdx.x;
  const int s = blockIdx.y;
  const int m = threadIdx.x;
  const int n_samp = n_class * M;
  if (m < M) {
    const int64_t js = (int64_t)s * n_samp + c * M + m;
    const bool have = samp_pos[js] >= 0;
    float st = 0.0f;
    if (have) {
      for (int hk = 0; hk < Hkv; ++hk) st += imp_part[js * Hkv + hk];
      st /= (float)(Hq * W);
    }
    if (samp_score) samp_score[js] = have ? st : __builtin_nanf("");
    if (samp_score_sum != nullptr && have) {      // expectation over layers: this layer joins the running sum
      const float tot = samp_score_sum[js] + st;
      samp_score_sum[js] = tot;
      st = tot / (float)layers;
    }
    sm_score[m] = st;
    sm_have[m] = have ? 1 : 0;
  }
  __syncthreads();
  if (m != 0) return;
  float sum = 0.0f;
  int cnt = 0;
  for (int i = 0; i < M; ++i)
    if (sm_have[i]) { sum += sm_score[i]; ++cnt; }
  const int64_t cs = (int64_t)s * n_class + c;
  if (cnt > 0) {
    const float mean = sum / (float)cnt;
    float w = (mean + alpha) / (1.0f + alpha);
    w = fminf(1.0f, fmaxf(0.0f, w));
    class_weight_q[cs] = (uint8_t)floorf(10.0f * w + 0.5f);
    if (class_mean) class_mean[cs] = mean;
  } else if (class_mean) {
    class_mean[cs] = __builtin_nanf("");
  }
}

hipError_t launch_importance(const dsk_compress_args& a, const CompressWs& ws, hipStream_t st) {
  float* imp_part = reinterpret_cast<float*>(static_cast<unsigned char*>(a.workspace) + ws.imp_part);
  const int n_samp = a.n_class * a.M;
  const float scale = a.imp_scale != 0.0f ? a.imp_scale : 0.08838834764831845f;   // 128^-1/2
  const int64_t heads_seqs = (int64_t)a.Hkv * a.B;
#define DSK_IMP_ARGS                                                                                          \
  static_cast<const uint16_t*>(a.K), a.k_stride_tok, a.k_stride_head, static_cast<const uint16_t*>(a.qwin),    \
      a.samp_pos, a.cu_seqlens, n_samp, a.W, a.R, a.Hq, a.Hq / a.Hkv, a.alpha_imp, scale * kImpLog2e, imp_part, \
      a.Hkv
  if ((int64_t)((n_samp + 3) / 4) * heads_seqs < 1024) {
    const dim3 grid((unsigned)((n_samp + 3) / 4), (unsigned)a.Hkv, (unsigned)a.B);
    importance_kernel<512, 4><<<grid, dim3(512), 0, st>>>(DSK_IMP_ARGS);
  } else {
    const dim3 grid((unsigned)((n_samp + 2) / 3), (unsigned)a.Hkv, (unsigned)a.B);
    importance_kernel<256, 3><<<grid, dim3(256), 0, st>>>(DSK_IMP_ARGS);
  }
#undef DSK_IMP_ARGS
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  importance_finalize_kernel<<<dim3((unsigned)a.n_class, (unsigned)a.B), dim3(DSK_WAVE), 0, st>>>(
      imp_part, a.samp_pos, a.n_class, a.M, a.Hkv, a.Hq, a.W, a.alpha_imp, a.class_weight_q, a.class_mean,
      a.samp_score, a.samp_score_sum, a.imp_layers > 0 ? a.imp_layers : 1);
  return hipGetLastError();
}

}  // namespace dsk
