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

// Fold 4*NS already-loaded token rows (K rows kv, V rows vv; row 4u+g in kv[u] of lane group g)
// into the state.  Rows >= nvalid are padding (their loads were redirected to a real row).
template <int NS>
__device__ __forceinline__ void fold_loaded(WaveState& st, const float (&qf)[8], const uint4 (&kv)[NS],
                                            const uint4 (&vv)[NS], int nvalid, int g, float scale_log2) {
  float z[NS];
  float mloc = -__builtin_inff();
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    float f[8];
    unpack8(kv[u], f);
    float d = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) d = fmaf(qf[k], f[k], d);
    d = group16_sum(d) * scale_log2;
    z[u] = (4 * u + g < nvalid) ? d : -__builtin_inff();
    mloc = fmaxf(mloc, z[u]);
  }
  mloc = fmaxf(fmaxf(rows4_f(mloc, 0), rows4_f(mloc, 1)), fmaxf(rows4_f(mloc, 2), rows4_f(mloc, 3)));
  const float m_new = fmaxf(st.m, mloc);           // finite: nvalid >= 1
  const float alpha = exp2f(st.m - m_new);         // 0 on the first fold (st.m = -inf)
  st.l *= alpha;
#pragma unroll
  for (int k = 0; k < 8; ++k) st.acc[k] *= alpha;
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    const float p = exp2f(z[u] - m_new);           // 0 for padded rows
    st.l += p;
    float f[8];
    unpack8(vv[u], f);
#pragma unroll
    for (int k = 0; k < 8; ++k) st.acc[k] = fmaf(p, f[k], st.acc[k]);
  }
  st.m = m_new;
}

}  // namespace dsk
