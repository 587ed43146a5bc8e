// Minimal host program on the C ABI alone (HIP runtime + include/dsk.h, no Python, no torch):
// builds a synthetic cache, runs the compression pass (candidates, DD-Select, slot map, K
// summaries), one decode step (dsk_select_topk + dsk_sparse_decode_attn), and checks the
// attention output of every head against a plain double-precision softmax over the tokens the
// library selected.  Exit status 0 and a line "dsk_example: ok ..." on success.
//
//   hipcc --offload-arch=gfx950 -I include examples/dsk_example.cpp -L. -ldsk -o dsk_example
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "dsk.h"

#define HIP_OK(x)                                                                              \
  do {                                                                                         \
    hipError_t e_ = (x);                                                                       \
    if (e_ != hipSuccess) {                                                                    \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                      \
      return 2;                                                                                \
    }                                                                                          \
  } while (0)
#define DSK_OK_(x)                                                                             \
  do {                                                                                         \
    dsk_status s_ = (x);                                                                       \
    if (s_ != DSK_OK) {                                                                        \
      std::fprintf(stderr, "%s failed: %s\n", #x, dsk_strerror(s_));                           \
      return 3;                                                                                \
    }                                                                                          \
  } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
static float rnd_normal() {   // sum of 12 uniforms: close enough to N(0,1) for a synthetic cache
  float s = 0.0f;
  for (int i = 0; i < 12; ++i) s += (float)(rnd() & 0xFFFF) / 65536.0f;
  return s - 6.0f;
}
static uint16_t to_bf16(float x) {   // round to nearest even
  uint32_t u;
  std::memcpy(&u, &x, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
static double from_bf16(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return (double)f;
}

template <class T>
static T* dev_alloc(size_t n) {
  void* p = nullptr;
  if (hipMalloc(&p, n * sizeof(T) + 256) != hipSuccess) { std::fprintf(stderr, "hipMalloc failed\n"); std::exit(2); }
  return static_cast<T*>(p);
}

int main() {
  const int L = 20000, Hq = 8, Hkv = 2, D = DSK_HEAD_DIM, b = 16, budget = 512, n_class = 4;
  const int C = 30, delta = 15, k = budget / b, G = Hq / Hkv;
  int n_dev = 0;
  HIP_OK(hipGetDeviceCount(&n_dev));
  if (n_dev < 1) { std::fprintf(stderr, "no GPU\n"); return 2; }
  HIP_OK(hipSetDevice(0));

  // ---- synthetic inputs ---------------------------------------------------------------------
  std::vector<int32_t> tok(L), delim = {11, 222, 3333, 44444}, cu = {0, L};
  for (int t = 0; t < L; ++t) tok[t] = 50000 + (int)(rnd() % 1000);
  for (int t = (int)(rnd() % 30); t < L; t += 1 + (int)(rnd() % 60)) tok[t] = delim[rnd() % n_class];
  std::vector<uint8_t> wq = {10, 5, 8, 6};   // class weights in tenths
  std::vector<uint16_t> K((size_t)Hkv * L * D), V(K.size()), q((size_t)Hq * D);
  for (auto& x : K) x = to_bf16(rnd_normal());
  for (auto& x : V) x = to_bf16(rnd_normal());
  for (auto& x : q) x = to_bf16(rnd_normal());

  int32_t *d_tok = dev_alloc<int32_t>(L), *d_delim = dev_alloc<int32_t>(n_class), *d_cu = dev_alloc<int32_t>(2);
  uint8_t* d_wq = dev_alloc<uint8_t>(n_class);
  uint16_t *d_K = dev_alloc<uint16_t>(K.size()), *d_V = dev_alloc<uint16_t>(V.size()), *d_q = dev_alloc<uint16_t>(q.size());
  HIP_OK(hipMemcpy(d_tok, tok.data(), L * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_delim, delim.data(), n_class * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_cu, cu.data(), 8, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_wq, wq.data(), n_class, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_K, K.data(), K.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_V, V.data(), V.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_q, q.data(), q.size() * 2, hipMemcpyHostToDevice));

  // ---- compression pass ---------------------------------------------------------------------
  const int cap = (int)dsk_block_capacity(L, 1, C - delta);
  int32_t *d_bs = dev_alloc<int32_t>(cap + 4), *d_sb = dev_alloc<int32_t>(cap + 4), *d_cub = dev_alloc<int32_t>(2);
  int32_t* d_status = dev_alloc<int32_t>(1);
  uint16_t* d_ksum = dev_alloc<uint16_t>((size_t)Hkv * cap * 2 * D);
  HIP_OK(hipMemset(d_bs, 0, (cap + 4) * 4));
  HIP_OK(hipMemset(d_sb, 0, (cap + 4) * 4));
  HIP_OK(hipMemset(d_status, 0, 4));

  dsk_compress_args ca;
  std::memset(&ca, 0, sizeof ca);
  ca.struct_size = sizeof ca;
  ca.stages = DSK_STAGE_CANDIDATES | DSK_STAGE_SEGMENT | DSK_STAGE_SUMMARIES;
  ca.B = 1; ca.Hq = Hq; ca.Hkv = Hkv; ca.D = D;
  ca.total_tokens = L; ca.max_seqlen = L; ca.cu_seqlens = d_cu;
  ca.K = d_K; ca.k_stride_tok = D; ca.k_stride_head = (int64_t)L * D;
  ca.token_ids = d_tok; ca.delim_ids = d_delim; ca.n_class = n_class;
  ca.max_cand_total = 0;                       // weights come from a table: no candidate list needed
  ca.class_weight_q = d_wq;
  ca.C = C; ca.delta = delta; ca.alpha_num = 5; ca.alpha_den = 10; ca.b = b;
  ca.max_blocks_total = cap; ca.block_start = d_bs; ca.cu_blocks = d_cub; ca.slot_base = d_sb;
  ca.ksum = d_ksum; ca.summary_mode = DSK_SUMMARY_MINMAX; ca.dev_status = d_status;
  ca.workspace_bytes = dsk_compress_workspace_bytes(&ca);
  ca.workspace = dev_alloc<unsigned char>(ca.workspace_bytes);
  DSK_OK_(dsk_compress(&ca, nullptr));

  // ---- one decode step ----------------------------------------------------------------------
  int32_t *d_slot = dev_alloc<int32_t>((size_t)Hq * k), *d_start = dev_alloc<int32_t>((size_t)Hq * k);
  int32_t *d_len = dev_alloc<int32_t>((size_t)Hq * k), *d_cnt = dev_alloc<int32_t>(Hq);
  dsk_select_args sa;
  std::memset(&sa, 0, sizeof sa);
  sa.struct_size = sizeof sa;
  sa.B = 1; sa.Hq = Hq; sa.Hkv = Hkv; sa.D = D;
  sa.max_blocks_total = cap; sa.cu_blocks = d_cub; sa.block_start = d_bs; sa.slot_base = d_sb;
  sa.ksum = d_ksum; sa.q = d_q; sa.b = b; sa.budget = budget;
  sa.sel_slot = d_slot; sa.sel_start = d_start; sa.sel_len = d_len; sa.sel_count = d_cnt;
  sa.workspace_bytes = dsk_select_workspace_bytes(&sa);
  sa.workspace = dev_alloc<unsigned char>(sa.workspace_bytes);
  DSK_OK_(dsk_select_topk(&sa, nullptr));

  float *d_out = dev_alloc<float>((size_t)Hq * D), *d_lse = dev_alloc<float>(Hq);
  dsk_attn_args aa;
  std::memset(&aa, 0, sizeof aa);
  aa.struct_size = sizeof aa;
  aa.B = 1; aa.Hq = Hq; aa.Hkv = Hkv; aa.D = D;
  aa.q = d_q; aa.K = d_K; aa.V = d_V;
  aa.k_stride_tok = aa.v_stride_tok = D; aa.k_stride_head = aa.v_stride_head = (int64_t)L * D;
  aa.total_tokens = L; aa.k = k; aa.b = b;
  aa.sel_start = d_start; aa.sel_len = d_len; aa.sel_count = d_cnt;
  aa.out = d_out; aa.lse = d_lse;
  aa.workspace_bytes = dsk_attn_workspace_bytes(&aa);
  aa.workspace = dev_alloc<unsigned char>(aa.workspace_bytes);
  DSK_OK_(dsk_sparse_decode_attn(&aa, nullptr));
  HIP_OK(hipDeviceSynchronize());

  // ---- read back and check ------------------------------------------------------------------
  int32_t status = 0, cub[2] = {0, 0};
  std::vector<int32_t> start((size_t)Hq * k), len((size_t)Hq * k), cnt(Hq);
  std::vector<float> out((size_t)Hq * D), lse(Hq);
  HIP_OK(hipMemcpy(&status, d_status, 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(cub, d_cub, 8, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(start.data(), d_start, start.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(len.data(), d_len, len.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(cnt.data(), d_cnt, cnt.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(out.data(), d_out, out.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(lse.data(), d_lse, lse.size() * 4, hipMemcpyDeviceToHost));
  if (status != 0) { std::fprintf(stderr, "device status %d: %s\n", status, dsk_strerror((dsk_status)status)); return 4; }

  const double scale = 1.0 / std::sqrt((double)D);
  double worst = 0.0;
  long tokens = 0;
  for (int h = 0; h < Hq; ++h) {
    const int hk = h / G;
    std::vector<int> toks;
    for (int j = 0; j < cnt[h]; ++j)
      for (int t = 0; t < len[(size_t)h * k + j]; ++t) toks.push_back(start[(size_t)h * k + j] + t);
    tokens += (long)toks.size();
    std::vector<double> z(toks.size());
    double zmax = -1e300;
    for (size_t i = 0; i < toks.size(); ++i) {
      double s = 0.0;
      for (int d = 0; d < D; ++d) s += from_bf16(q[(size_t)h * D + d]) * from_bf16(K[((size_t)hk * L + toks[i]) * D + d]);
      z[i] = s * scale;
      if (z[i] > zmax) zmax = z[i];
    }
    double den = 0.0;
    for (double& x : z) { x = std::exp(x - zmax); den += x; }
    double omax = 0.0, emax = 0.0;
    for (int d = 0; d < D; ++d) {
      double o = 0.0;
      for (size_t i = 0; i < toks.size(); ++i) o += z[i] / den * from_bf16(V[((size_t)hk * L + toks[i]) * D + d]);
      omax = std::fmax(omax, std::fabs(o));
      emax = std::fmax(emax, std::fabs(o - (double)out[(size_t)h * D + d]));
    }
    worst = std::fmax(worst, emax / std::fmax(omax, 1e-30));
    if (std::fabs((double)lse[h] - (zmax + std::log(den))) > 1e-3) { std::fprintf(stderr, "lse mismatch on head %d\n", h); return 5; }
  }
  if (!(worst <= 2e-3)) { std::fprintf(stderr, "attention mismatch: rel err %.3e\n", worst); return 5; }
  std::printf("dsk_example: ok  blocks=%d  selected tokens per head=%ld  worst attention rel err=%.2e\n", cub[1],
              tokens / Hq, worst);
  return 0;
}
