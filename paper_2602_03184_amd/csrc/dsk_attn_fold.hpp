// Online-softmax state of one wavefront and the fold of up to 32 loaded K/V rows into it;
// shared by the sparse gather kernel and the full-attention baseline.
#pragma once

#include "dsk_common.hpp"

namespace dsk {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct WaveState {
  float m;        // running max of the logits, in log2 units (wave-uniform)
  float l;        // this lane group's part of the denominator
  float acc[8];   // this lane group's part of the numerator, channels 8c..8c+7
};

// A query row's 8 channels of one lane, kept as 4 packed bf16 pairs: q.K runs on the packed
// bf16 dot instruction (two exact bf16 products added into an fp32 accumulator), which needs
// neither operand widened.
struct QRow {
  uint32_t p[4];
};
__device__ __forceinline__ QRow make_qrow(const uint4& v) { return QRow{{v.x, v.y, v.z, v.w}}; }

typedef __bf16 dsk_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dsk_bf16x2, a), __builtin_bit_cast(dsk_bf16x2, b), acc,
                                         false);
}
__device__ __forceinline__ float dot8_bf16(const QRow& q, const uint4& k) {
  float d = dot2_bf16(q.p[0], k.x, 0.0f);
  d = dot2_bf16(q.p[1], k.y, d);
  d = dot2_bf16(q.p[2], k.z, d);
  return dot2_bf16(q.p[3], k.w, d);
}

// 2^x for x <= 0 on the hardware exponential alone: results below the normal range come out as
// 0, which is what a softmax weight that small is worth; -inf gives 0.
__device__ __forceinline__ float exp2_nonpos(float x) { return __builtin_amdgcn_exp2f(x); }

// one channel of a finished attention output: fp32 always, a nearest-even bf16 copy on request
__device__ __forceinline__ void store_attn_out(float* __restrict__ out, uint16_t* __restrict__ out_bf16, int64_t idx,
                                               float v) {
  out[idx] = v;
  if (out_bf16 != nullptr) out_bf16[idx] = (uint16_t)(__float_as_uint(bf16_round_rne(v)) >> 16);
}

// Fold 4*NS already-loaded token rows (K rows kv, V rows vv; row 4u+g in kv[u] of lane group g)
// into the state.  Rows >= nvalid are padding (their loads were redirected to a real row).
template <int NS>
__device__ __forceinline__ void fold_loaded(WaveState& st, const QRow& qf, const uint4 (&kv)[NS],
                                            const uint4 (&vv)[NS], int nvalid, int g, float scale_log2) {
  float z[NS];
  float mloc = -__builtin_inff();
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    const float d = group16_sum(dot8_bf16(qf, kv[u])) * scale_log2;
    z[u] = (4 * u + g < nvalid) ? d : -__builtin_inff();
    mloc = fmaxf(mloc, z[u]);
  }
  mloc = fmaxf(fmaxf(rows4_f(mloc, 0), rows4_f(mloc, 1)), fmaxf(rows4_f(mloc, 2), rows4_f(mloc, 3)));
  const float m_new = fmaxf(st.m, mloc);           // finite: nvalid >= 1
  const float alpha = exp2_nonpos(st.m - m_new);         // 0 on the first fold (st.m = -inf)
  st.l *= alpha;
#pragma unroll
  for (int k = 0; k < 8; ++k) st.acc[k] *= alpha;
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    const float p = exp2_nonpos(z[u] - m_new);          // 0 for padded rows
    st.l += p;
    float f[8];
    unpack8(vv[u], f);
#pragma unroll
    for (int k = 0; k < 8; ++k) st.acc[k] = fmaf(p, f[k], st.acc[k]);
  }
  st.m = m_new;
}

}  // namespace dsk
