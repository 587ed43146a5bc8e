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
// loads; Q^T uses the same permutation, so the sum over channels is unchanged.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kImpThreads = 512;   // 8 waves share the key tiles of a sample (256 and 1024 threads measured slower)
constexpr int kImpWaves = kImpThreads / DSK_WAVE;
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

// grid: (sample slot c*M+m, kv head, sequence)
__global__ __launch_bounds__(kImpThreads) void importance_kernel(
    const uint16_t* __restrict__ K, int64_t kst, int64_t ksh, const uint16_t* __restrict__ qwin,
    const int32_t* __restrict__ samp_pos, const int32_t* __restrict__ cu_seqlens, int n_samp, int W, int R,
    int Hq, int G, float alpha, float scale_log2, float* __restrict__ imp_part, int Hkv) {
  __shared__ RowStat sm_stat[kImpWaves][32];
  __shared__ float sm_val[32];
  const int j = blockIdx.x;
  const int hk = blockIdx.y;
  const int s = blockIdx.z;
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int col = lane & 31;        // query row of the tile this lane accumulates
  const int hf = lane >> 5;         // channel half / key sub-row selector
  float* out = imp_part + ((int64_t)s * n_samp + j) * Hkv + hk;

  const int seq0 = cu_seqlens[s];
  const int L = cu_seqlens[s + 1] - seq0;
  const int tg = samp_pos[(int64_t)s * n_samp + j];
  const int t = tg - seq0;
  if (tg < 0 || t < 0 || t >= L) {          // no such sample
    if (threadIdx.x == 0) *out = 0.0f;
    return;
  }
  const int rows = W * G;                   // query rows of this (sample, kv head)
  const int o_lo = t - R + 1 > 0 ? t - R + 1 : 0;   // retained region [o_lo, t]
  const int d_hi = t - R > 0 ? t - R : 0;           // discarded region [0, d_hi]
  const int last_key = t + W < L - 1 ? t + W : L - 1;
  const int n_tiles = last_key / 32 + 1;
  const uint16_t* Kh = K + (int64_t)hk * ksh + (int64_t)seq0 * kst + hf * 64;
  float total = 0.0f;

  for (int row0 = 0; row0 < rows; row0 += 32) {
    // Q^T operand: lane (col, hf) holds channels [64*hf, 64*hf+64) of query row row0+col
    const int row = row0 + col;
    const bool row_ok = row < rows;
    const int w = row_ok ? row / G : 0;
    const int g = row_ok ? row % G : 0;
    const int qpos = t + 1 + w;             // position of this query; attends keys 0..qpos
    bf16x8_t qv[8];
    {
      const uint16_t* qp = qwin + ((((int64_t)s * n_samp + j) * W + w) * Hq + hk * G + g) * DSK_HEAD_DIM + hf * 64;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        uint4 raw = *reinterpret_cast<const uint4*>(qp + u * 8);
        if (!row_ok) raw = make_uint4(0, 0, 0, 0);
        qv[u] = *reinterpret_cast<bf16x8_t*>(&raw);
      }
    }
    RowStat st;
    st.m = -__builtin_inff();
    st.zt = st.zo = st.zd = 0.0f;
    for (int tile = wave; tile < n_tiles; tile += kImpWaves) {
      const int k0 = tile * 32;
      int krow = k0 + col;                  // A operand row of this lane
      krow = krow < L ? krow : L - 1;       // stay inside the sequence; masked below
      const uint16_t* kp = Kh + (int64_t)krow * kst;
      uint4 kraw[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) kraw[u] = *reinterpret_cast<const uint4*>(kp + u * 8);
      f32x16_t acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8_t*>(&kraw[u]), qv[u], acc, 0, 0, 0);
      // acc[r] = logit of key k0 + 8*(r/4) + 4*hf + r%4 against query row `col`
      float z[16];
      float tmax = -__builtin_inff();
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kpos = k0 + 8 * (r / 4) + 4 * hf + (r % 4);
        z[r] = (kpos <= qpos && kpos <= last_key) ? acc[r] * scale_log2 : -__builtin_inff();
        tmax = fmaxf(tmax, z[r]);
      }
      if (tmax != -__builtin_inff()) {
        const float mn = fmaxf(st.m, tmax);
        const float f = st.m == -__builtin_inff() ? 0.0f : exp2f(st.m - mn);
        st.zt *= f; st.zo *= f; st.zd *= f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kpos = k0 + 8 * (r / 4) + 4 * hf + (r % 4);
          const float e = __builtin_amdgcn_exp2f(z[r] - mn);   // z <= mn; 0 for masked keys (-inf)
          st.zt += e;
          st.zo += (kpos >= o_lo && kpos <= t) ? e : 0.0f;
          st.zd += (kpos <= d_hi) ? e : 0.0f;
        }
        st.m = mn;
      }
    }
    // halves of a wave hold disjoint keys of the same row; then waves; fixed order
    RowStat other;
    other.m = shfl_xor_f(st.m, 32);
    other.zt = shfl_xor_f(st.zt, 32);
    other.zo = shfl_xor_f(st.zo, 32);
    other.zd = shfl_xor_f(st.zd, 32);
    if (hf == 0) {
      stat_merge(st, other);
      sm_stat[wave][col] = st;
    }
    __syncthreads();
    if (threadIdx.x < 32) {
      RowStat a = sm_stat[0][col];
#pragma unroll
      for (int wv = 1; wv < kImpWaves; ++wv) stat_merge(a, sm_stat[wv][col]);
      const float v = (row0 + col < rows && a.zt > 0.0f) ? (a.zo - alpha * a.zd) / a.zt : 0.0f;
      sm_val[col] = v;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int c2 = 0; c2 < 32; ++c2) total += sm_val[c2];   // fixed order
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = total;
}

// one workgroup per sequence, one thread per delimiter class
__global__ __launch_bounds__(DSK_MAX_CLASSES) void importance_finalize_kernel(
    const float* __restrict__ imp_part, const int32_t* __restrict__ samp_pos, int n_class, int M, int Hkv,
    int Hq, int W, float alpha, uint8_t* __restrict__ class_weight_q, float* __restrict__ class_mean,
    float* __restrict__ samp_score) {
  const int s = blockIdx.x;
  const int c = threadIdx.x;
  if (c >= n_class) return;
  const int n_samp = n_class * M;
  float sum = 0.0f;
  int cnt = 0;
  for (int m = 0; m < M; ++m) {
    const int64_t js = (int64_t)s * n_samp + c * M + m;
    const bool have = samp_pos[js] >= 0;
    float st = 0.0f;
    if (have) {
      for (int hk = 0; hk < Hkv; ++hk) st += imp_part[js * Hkv + hk];
      st /= (float)(Hq * W);
      sum += st;
      ++cnt;
    }
    if (samp_score) samp_score[js] = have ? st : __builtin_nanf("");
  }
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
  const dim3 grid((unsigned)n_samp, (unsigned)a.Hkv, (unsigned)a.B);
  importance_kernel<<<grid, dim3(kImpThreads), 0, st>>>(
      static_cast<const uint16_t*>(a.K), a.k_stride_tok, a.k_stride_head, static_cast<const uint16_t*>(a.qwin),
      a.samp_pos, a.cu_seqlens, n_samp, a.W, a.R, a.Hq, a.Hq / a.Hkv, a.alpha_imp, scale * kImpLog2e, imp_part,
      a.Hkv);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  importance_finalize_kernel<<<dim3((unsigned)a.B), dim3(DSK_MAX_CLASSES), 0, st>>>(
      imp_part, a.samp_pos, a.n_class, a.M, a.Hkv, a.Hq, a.W, a.alpha_imp, a.class_weight_q, a.class_mean,
      a.samp_score);
  return hipGetLastError();
}

}  // namespace dsk
