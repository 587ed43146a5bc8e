// Sparse decode attention over the K/V rows of the selected slots (App. B.2 Steps 2-3):
// a split-K flash-decode.  The gather is HBM-bound (512 B of K+V per token, ~2 flop/B), so
// there is no MFMA here: a 256-byte bf16 row is spread over 16 lanes x 16 B and a wavefront
// reads 4 token rows per load instruction.  A wavefront owns SPW slots of at most 4*NS rows; it
// issues every K and V load of a slot (16 x 16 B per lane, 16 KB per wavefront for 32 rows)
// before it touches the data, then folds the slot into an online-softmax state (m, l, acc).
// The wavefronts of a workgroup (8 for slots of up to 32 rows, 2 slots each) merge through LDS
// into one partial per (sequence, head, chunk of 16 slots); a second small kernel merges the
// partials of a head in a fixed order.  (Merging inside this kernel -- the workgroup of a head that
// finishes last, found with an arrival counter, folds the head's partials -- was built three ways:
// write-through partials with a device-scope counter, ordinary stores with a device-scope counter,
// ordinary stores with a counter that stays in the XCD's L2.  At 128K / 32 heads the attention call
// took 9.8 / 9.6 / 9.3 us against 9.3 us with the merge launch, whose cost in a graph is that of an
// empty kernel, about 1.5 us: the store-acknowledge, counter and reload round trips of the last
// workgroup cost as much.  Not kept.)
// The launch is a 1-D grid in which workgroup id = 8 * j + x runs on XCD x: all chunks of all
// query heads of a (sequence, KV head) group are given the same x, so that rows selected by
// several heads of the group are fetched into one L2 once (9.3 instead of 10.5 us for the call at
// 128K / 32 heads against a grid that spread a head's chunks over the XCDs).
#include "dsk_attn_fold.hpp"
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kMergeBigThreads = 1024;

// slots per workgroup for a slot length bound b
__host__ __device__ constexpr int attn_slots_per_wg(int b) { return b <= 32 ? 16 : 8; }
// Launches of many workgroups (a batch) run better on workgroups of 4 wavefronts x 2 slots: the last
// round of workgroups on the CUs is finer (8 ragged sequences, b = 16: gather 28.2 -> 26.0 us, step
// 48.6 -> 47.0 us), while small launches lose to the doubled number of partials (one sequence of
// 32K or 128K tokens: step +0.2 us), so the shape follows the workgroup count.
constexpr int64_t kAttnSmallWgFrom = 1536;   // workgroups of 16 slots from which 8-slot workgroups are launched

// Shared selection: the tiled kernel (attn_shared_kernel, WAVES x SPW slots per workgroup) takes
// group widths 2, 4, 8 and slots of at most 32 rows.  It reads every selected row once, where
// attn_kernel run per query head reads it once per head with all but the first read served by
// L2; that is as fast while the launch is small (config 3, 1024 selected slots per step:
// 5.9 us either way, and 8 instead of 16 partials to merge), and slower from a few thousand
// slots on (8 sequences of config 5, 8192 slots: 15.3 against 18.6 us), so the tiled kernel is
// used from 4096 slots per step.  Measured against 4 x 1, 8 x 1 and 8 x 2.
constexpr int kSharedWaves = 4;
constexpr int kSharedSpw = 2;
constexpr int64_t kSharedTiledMinSlots = 4096;
static bool attn_shared_tiled(const dsk_attn_args& a) {
  const int G = a.Hq / a.Hkv;
  return (a.flags & DSK_ATTN_SHARED_SELECTION) && (G == 2 || G == 4 || G == 8) && a.b <= 32 &&
         (int64_t)a.B * a.Hkv * a.k >= kSharedTiledMinSlots;
}

// ordinary (compiler-scheduled) loads; used for slots longer than 32 rows
template <int NS>
__device__ __forceinline__ void fold_rows(WaveState& st, const QRow& qf, const uint16_t* __restrict__ kbase,
                                          const uint16_t* __restrict__ vbase, int64_t kst, int64_t vst,
                                          int nvalid, int g, float scale_log2) {
  uint4 kv[NS], vv[NS];
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    int r = 4 * u + g;
    r = r < nvalid ? r : nvalid - 1;
    kv[u] = *reinterpret_cast<const uint4*>(kbase + (int64_t)r * kst);
  }
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    int r = 4 * u + g;
    r = r < nvalid ? r : nvalid - 1;
    vv[u] = *reinterpret_cast<const uint4*>(vbase + (int64_t)r * vst);
  }
  fold_loaded<NS>(st, qf, kv, vv, nvalid, g, scale_log2);
}

// compile-time loop over the slots of a wave: wait for slot S's K and V, fold, recurse
template <int NS, int SPW, int S>
struct FoldSlots {
  static __device__ __forceinline__ void run(WaveState& st, const QRow& qf, uint4 (&kd)[SPW][NS],
                                             uint4 (&vd)[SPW][NS], const int (&nv)[SPW], int g,
                                             float scale_log2) {
    // loads were issued slot by slot, K rows then V rows; pinning slot S here keeps the loads of
    // the later slots in flight while this one is folded
#pragma unroll
    for (int u = 0; u < NS; ++u) pin_loaded(kd[S][u]);
#pragma unroll
    for (int u = 0; u < NS; ++u) pin_loaded(vd[S][u]);
    if (nv[S] > 0) fold_loaded<NS>(st, qf, kd[S], vd[S], nv[S], g, scale_log2);
    if constexpr (S + 1 < SPW) FoldSlots<NS, SPW, S + 1>::run(st, qf, kd, vd, nv, g, scale_log2);
  }
};

// One workgroup of WAVES wavefronts per (chunk of WAVES*SPW slots, head, sequence); writes one partial, or the
// final result when the head has a single chunk.  NS = 0 selects the generic path for slots
// longer than 32 rows (2 slots per wave, rows folded 32 at a time).
template <int NS, int SPW, int WAVES, bool STAGED = false>
__global__ __launch_bounds__(WAVES * DSK_WAVE) void attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    int64_t kst, int64_t ksh, int64_t vst, int64_t vsh, int Hq, int G, int n_groups, int k, int b, int total_tokens,
    const int32_t* __restrict__ sel_start, const int32_t* __restrict__ sel_len,
    const int32_t* __restrict__ sel_count, int sel_div, float scale_log2, int nchunks,
    float2* __restrict__ part_ml, float* __restrict__ part_acc, float* __restrict__ out,
    uint16_t* __restrict__ out_bf16, float* __restrict__ lse) {
  constexpr int kAttnWaves = WAVES;
  __shared__ float sm_m[kAttnWaves];
  __shared__ float sm_l[kAttnWaves];
  __shared__ float sm_acc[kAttnWaves][DSK_HEAD_DIM];
  constexpr int kSlotsPerWg = kAttnWaves * SPW;

  // workgroup id = 8 * j + x lands on XCD x.  Group gi = s * Hkv + hk takes x = gi % 8; its
  // G * nchunks workgroups are consecutive in j.
  // Without grouped heads there is nothing to share: the chunks of a head are dealt out over the
  // XCDs in plain order (measured 2 % faster at 40 heads than keeping a head on one XCD).
  int s, hk, h, chunk;
  if (G == 1) {
    chunk = blockIdx.x % nchunks;
    const int sh_lin = blockIdx.x / nchunks;
    s = sh_lin / Hq;
    h = hk = sh_lin - s * Hq;
  } else {
    const int Hkv = Hq / G;
    const int per_group = G * nchunks;
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;
    const int gl = j / per_group;
    const int r = j - gl * per_group;
    const int gi = gl * 8 + xcd;
    if (gi >= n_groups) return;                  // padding of the last round of groups
    s = gi / Hkv;
    hk = gi - s * Hkv;
    const int gq = r / nchunks;
    chunk = r - gq * nchunks;
    h = hk * G + gq;
  }
  const int64_t sh = (int64_t)s * Hq + h;
  // row of the selection arrays: the head's own, or its KV head's when sel_div = Hq/Hkv heads share one
  const int64_t sr = sel_div == 1 ? sh : (int64_t)s * (Hq / sel_div) + h / sel_div;   // no division on the per-head path
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int slot0 = chunk * kSlotsPerWg;

  // the wave's slots: slot0 + wave + kAttnWaves * r; their spans are fetched together with the count
  int count = sel_count[sr];
  int st_[SPW], ln_[SPW];
#pragma unroll
  for (int r = 0; r < SPW; ++r) {
    const int j = slot0 + wave + kAttnWaves * r;
    st_[r] = j < k ? sel_start[sr * k + j] : 0;
    ln_[r] = j < k ? sel_len[sr * k + j] : 0;
  }
  if (count > k) count = k;
  if (total_tokens <= 0) count = 0;   // no K/V row exists: not even the redirected loads of skipped slots may run
  if (count <= 0) {   // nothing selected: chunk 0 writes the defined empty result
    if (chunk == 0 && threadIdx.x < DSK_HEAD_DIM) {
      store_attn_out(out, out_bf16, sh * DSK_HEAD_DIM + threadIdx.x, 0.0f);
      if (threadIdx.x == 0 && lse) lse[sh] = -__builtin_inff();
    }
    return;
  }
  if (slot0 >= count) return;   // uniform over the workgroup; not counted in `used` below
  const int used = (count + kSlotsPerWg - 1) / kSlotsPerWg;

  const int g = lane >> 4;
  const int c = lane & 15;
  const QRow qf = make_qrow(*reinterpret_cast<const uint4*>(q + sh * DSK_HEAD_DIM + c * 8));
  const uint16_t* Kh = K + (int64_t)hk * ksh + c * 8;
  const uint16_t* Vh = V + (int64_t)hk * vsh + c * 8;

  WaveState st;
  st.m = -__builtin_inff();
  st.l = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) st.acc[i] = 0.0f;

  if constexpr (NS > 0) {
    // every slot has at most 4*NS rows: all K/V loads of the wave's SPW slots go out now
    uint4 kd[SPW][NS], vd[SPW][NS];
    int nv[SPW];
#pragma unroll
    for (int r = 0; r < SPW; ++r) {
      const int j = slot0 + wave + kAttnWaves * r;
      int start = st_[r];
      int len = ln_[r] < b ? ln_[r] : b;
      len = len < 4 * NS ? len : 4 * NS;
      const bool ok = j < count && start >= 0 && len > 0 && start <= total_tokens - len;   // never read outside K/V
      nv[r] = ok ? len : 0;
      start = ok ? start : 0;            // a skipped slot reads row 0 (harmless) so that the loads
      len = ok ? len : 1;                // below stay unconditional
#pragma unroll
      for (int u = 0; u < NS; ++u) {
        int row = 4 * u + g;
        row = row < len ? row : len - 1;
        kd[r][u] = *reinterpret_cast<const uint4*>(Kh + (int64_t)(start + row) * kst);
      }
#pragma unroll
      for (int u = 0; u < NS; ++u) {
        int row = 4 * u + g;
        row = row < len ? row : len - 1;
        vd[r][u] = *reinterpret_cast<const uint4*>(Vh + (int64_t)(start + row) * vst);
      }
      if constexpr (STAGED) {
#pragma unroll
        for (int u = 0; u < NS; ++u) pin_loaded(kd[r][u]);
#pragma unroll
        for (int u = 0; u < NS; ++u) pin_loaded(vd[r][u]);
        if (nv[r] > 0) fold_loaded<NS>(st, qf, kd[r], vd[r], nv[r], g, scale_log2);
      }
    }
    if constexpr (!STAGED) FoldSlots<NS, SPW, 0>::run(st, qf, kd, vd, nv, g, scale_log2);
  } else {
#pragma unroll
    for (int r = 0; r < SPW; ++r) {
      const int j = slot0 + wave + kAttnWaves * r;
      const int start = st_[r];
      int len = ln_[r];
      if (len > b) len = b;
      if (j >= count || start < 0 || len <= 0 || start > total_tokens - len) continue;   // never read outside K/V
      for (int r0 = 0; r0 < len; r0 += 32) {
        const int nvr = len - r0;
        const uint16_t* kb = Kh + (int64_t)(start + r0) * kst;
        const uint16_t* vb = Vh + (int64_t)(start + r0) * vst;
        if (nvr > 16) fold_rows<8>(st, qf, kb, vb, kst, vst, nvr < 32 ? nvr : 32, g, scale_log2);
        else fold_rows<4>(st, qf, kb, vb, kst, vst, nvr, g, scale_log2);
      }
    }
  }

  // lane groups -> wave
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    st.acc[i] += shfl_xor_f(st.acc[i], 16);
    st.acc[i] += shfl_xor_f(st.acc[i], 32);
  }
  st.l += shfl_xor_f(st.l, 16);
  st.l += shfl_xor_f(st.l, 32);
  if (lane == 0) { sm_m[wave] = st.m; sm_l[wave] = st.l; }
  if (g == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) sm_acc[wave][c * 8 + i] = st.acc[i];
  }
  __syncthreads();

  // waves -> workgroup partial, fixed order
  const int d = threadIdx.x;
  if (d >= DSK_HEAD_DIM) return;
  float M = sm_m[0];
#pragma unroll
  for (int w = 1; w < kAttnWaves; ++w) M = fmaxf(M, sm_m[w]);
  float l = 0.0f, a = 0.0f;
#pragma unroll
  for (int w = 0; w < kAttnWaves; ++w) {
    const float f = sm_m[w] == -__builtin_inff() ? 0.0f : exp2f(sm_m[w] - M);   // idle wave
    l = fmaf(sm_l[w], f, l);
    a = fmaf(sm_acc[w][d], f, a);
  }
  if (used == 1) {   // the only chunk of this head: finish here
    store_attn_out(out, out_bf16, sh * DSK_HEAD_DIM + d, l > 0.0f ? a / l : 0.0f);
    if (d == 0 && lse) lse[sh] = l > 0.0f ? (M + log2f(l)) * kLn2 : -__builtin_inff();
    return;
  }
  const int64_t pbase = sh * nchunks;
  part_acc[(pbase + chunk) * DSK_HEAD_DIM + d] = a;
  if (d == 0) part_ml[pbase + chunk] = make_float2(M, l);
}

// Shared selection (one slot list per KV head, used by all its query heads): a workgroup per
// (chunk of WAVES*SPW slots, KV head x tile of GT query heads, sequence).  Every K/V row a
// wavefront loads is folded into the GT heads' states, so the group's rows are read once instead
// of once per query head.  Same partial layout as attn_kernel (one partial per query head and
// chunk), merged by attn_merge_kernel.
template <int NS, int SPW, int WAVES, int GT>
__global__ __launch_bounds__(WAVES * DSK_WAVE) void attn_shared_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    int64_t kst, int64_t ksh, int64_t vst, int64_t vsh, int Hq, int G, int k, int b, int total_tokens,
    const int32_t* __restrict__ sel_start, const int32_t* __restrict__ sel_len,
    const int32_t* __restrict__ sel_count, float scale_log2, int nchunks,
    float2* __restrict__ part_ml, float* __restrict__ part_acc, float* __restrict__ out,
    uint16_t* __restrict__ out_bf16, float* __restrict__ lse) {
  static_assert(NS > 0, "slots of at most 4*NS rows");
  __shared__ float sm_m[WAVES][GT];
  __shared__ float sm_l[WAVES][GT];
  __shared__ float sm_acc[WAVES][GT][DSK_HEAD_DIM];
  constexpr int kSlotsPerWg = WAVES * SPW;

  const int chunk = blockIdx.x;
  const int tiles_g = G / GT;
  const int hk = blockIdx.y / tiles_g;
  const int h0 = hk * G + (blockIdx.y % tiles_g) * GT;     // first query head of this tile
  const int s = blockIdx.z;
  const int64_t sr = (int64_t)s * (Hq / G) + hk;            // row of the selection arrays
  const int64_t sh0 = (int64_t)s * Hq + h0;
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int slot0 = chunk * kSlotsPerWg;

  int count = sel_count[sr];
  int st_[SPW], ln_[SPW];
#pragma unroll
  for (int r = 0; r < SPW; ++r) {
    const int j = slot0 + wave + WAVES * r;
    st_[r] = j < k ? sel_start[sr * k + j] : 0;
    ln_[r] = j < k ? sel_len[sr * k + j] : 0;
  }
  if (count > k) count = k;
  if (total_tokens <= 0) count = 0;   // no K/V row exists: not even the redirected loads of skipped slots may run
  if (count <= 0) {   // nothing selected: chunk 0 writes the defined empty result of the tile's heads
    if (chunk == 0 && threadIdx.x < DSK_HEAD_DIM) {
#pragma unroll
      for (int j = 0; j < GT; ++j) {
        store_attn_out(out, out_bf16, (sh0 + j) * DSK_HEAD_DIM + threadIdx.x, 0.0f);
        if (threadIdx.x == 0 && lse) lse[sh0 + j] = -__builtin_inff();
      }
    }
    return;
  }
  if (slot0 >= count) return;
  const int used = (count + kSlotsPerWg - 1) / kSlotsPerWg;

  const int g = lane >> 4;
  const int c = lane & 15;
  QRow qf[GT];
#pragma unroll
  for (int j = 0; j < GT; ++j) qf[j] = make_qrow(*reinterpret_cast<const uint4*>(q + (sh0 + j) * DSK_HEAD_DIM + c * 8));
  const uint16_t* Kh = K + (int64_t)hk * ksh + c * 8;
  const uint16_t* Vh = V + (int64_t)hk * vsh + c * 8;

  WaveState st[GT];
#pragma unroll
  for (int j = 0; j < GT; ++j) {
    st[j].m = -__builtin_inff();
    st[j].l = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) st[j].acc[i] = 0.0f;
  }

  uint4 kd[SPW][NS], vd[SPW][NS];
  int nv[SPW];
#pragma unroll
  for (int r = 0; r < SPW; ++r) {
    const int j = slot0 + wave + WAVES * r;
    int start = st_[r];
    int len = ln_[r] < b ? ln_[r] : b;
    len = len < 4 * NS ? len : 4 * NS;
    const bool ok = j < count && start >= 0 && len > 0 && start <= total_tokens - len;   // never read outside K/V
    nv[r] = ok ? len : 0;
    start = ok ? start : 0;
    len = ok ? len : 1;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      int row = 4 * u + g;
      row = row < len ? row : len - 1;
      kd[r][u] = *reinterpret_cast<const uint4*>(Kh + (int64_t)(start + row) * kst);
    }
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      int row = 4 * u + g;
      row = row < len ? row : len - 1;
      vd[r][u] = *reinterpret_cast<const uint4*>(Vh + (int64_t)(start + row) * vst);
    }
  }
#pragma unroll
  for (int r = 0; r < SPW; ++r) {
#pragma unroll
    for (int u = 0; u < NS; ++u) pin_loaded(kd[r][u]);
#pragma unroll
    for (int u = 0; u < NS; ++u) pin_loaded(vd[r][u]);
    if (nv[r] > 0) {
#pragma unroll
      for (int j = 0; j < GT; ++j) fold_loaded<NS>(st[j], qf[j], kd[r], vd[r], nv[r], g, scale_log2);
    }
  }

#pragma unroll
  for (int j = 0; j < GT; ++j) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      st[j].acc[i] += shfl_xor_f(st[j].acc[i], 16);
      st[j].acc[i] += shfl_xor_f(st[j].acc[i], 32);
    }
    st[j].l += shfl_xor_f(st[j].l, 16);
    st[j].l += shfl_xor_f(st[j].l, 32);
    if (lane == 0) { sm_m[wave][j] = st[j].m; sm_l[wave][j] = st[j].l; }
    if (g == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) sm_acc[wave][j][c * 8 + i] = st[j].acc[i];
    }
  }
  __syncthreads();

  // waves -> one partial per head of the tile, fixed order
  for (int idx = threadIdx.x; idx < GT * DSK_HEAD_DIM; idx += WAVES * DSK_WAVE) {
    const int j = idx / DSK_HEAD_DIM;
    const int d = idx % DSK_HEAD_DIM;
    float M = sm_m[0][j];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) M = fmaxf(M, sm_m[w][j]);
    float l = 0.0f, a = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float f = sm_m[w][j] == -__builtin_inff() ? 0.0f : exp2f(sm_m[w][j] - M);   // idle wave
      l = fmaf(sm_l[w][j], f, l);
      a = fmaf(sm_acc[w][j][d], f, a);
    }
    const int64_t sh = sh0 + j;
    if (used == 1) {
      store_attn_out(out, out_bf16, sh * DSK_HEAD_DIM + d, l > 0.0f ? a / l : 0.0f);
      if (d == 0 && lse) lse[sh] = l > 0.0f ? (M + log2f(l)) * kLn2 : -__builtin_inff();
    } else {
      part_acc[(sh * nchunks + chunk) * DSK_HEAD_DIM + d] = a;
      if (d == 0) part_ml[sh * nchunks + chunk] = make_float2(M, l);
    }
  }
}

// Merge of the partials of one (sequence, head) in a fixed order: 16 lane groups each fold the
// chunks ch = group, group+16, ... (all loads of a round are independent), then one pass over
// the 16 group states in LDS.  Heads with a single chunk were finished by attn_kernel.
template <int kMergeThreads>
__global__ __launch_bounds__(kMergeThreads) void attn_merge_kernel(
    const float2* __restrict__ part_ml, const float* __restrict__ part_acc,
    const int32_t* __restrict__ sel_count, const int32_t* __restrict__ cu_seqlens, int Hq, int sel_div, int k,
    int nchunks, int slots_per_wg, float* __restrict__ out, uint16_t* __restrict__ out_bf16,
    float* __restrict__ lse) {
  constexpr int kMergeGroups = kMergeThreads / 16;
  __shared__ float sm_m[kMergeGroups];
  __shared__ float sm_l[kMergeGroups];
  __shared__ float sm_acc[kMergeGroups][DSK_HEAD_DIM];
  const int64_t sh = blockIdx.x;
  const int grp = threadIdx.x >> 4;
  const int c = threadIdx.x & 15;
  const float2* ml = part_ml + sh * nchunks;
  const float* acc = part_acc + sh * nchunks * DSK_HEAD_DIM + c * 8;
  // first round of partials is fetched together with the count (the workspace always holds
  // nchunks entries per head; stale ones are discarded below by index)
  float2 v0 = make_float2(0.0f, 0.0f);
  float4 x00 = make_float4(0.f, 0.f, 0.f, 0.f), x01 = x00;
  if (grp < nchunks) {
    v0 = ml[grp];
    x00 = *reinterpret_cast<const float4*>(acc + (int64_t)grp * DSK_HEAD_DIM);
    x01 = *reinterpret_cast<const float4*>(acc + (int64_t)grp * DSK_HEAD_DIM + 4);
  }
  // units folded per head: selected slots, or (full attention) the tokens of the sequence
  int count;
  if (cu_seqlens != nullptr) {
    const int s = (int)(sh / Hq);
    count = cu_seqlens[s + 1] - cu_seqlens[s];
  } else {
    if (sel_div == 1) {
      count = sel_count[sh];
    } else {
      const int s = (int)(sh / Hq), h = (int)(sh % Hq);
      count = sel_count[(int64_t)s * (Hq / sel_div) + h / sel_div];
    }
  }
  if (count > k) count = k;
  int used = (int)(((int64_t)count + slots_per_wg - 1) / slots_per_wg);
  if (used > nchunks) used = nchunks;   // never past the partials this head owns
  if (used <= 1) return;   // empty or single-chunk heads are complete already
  float m = -__builtin_inff(), l = 0.0f, a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = 0.0f;
  for (int ch = grp; ch < used; ch += kMergeGroups) {
    float2 v;
    float4 x0, x1;
    if (ch == grp) { v = v0; x0 = x00; x1 = x01; }
    else {
      v = ml[ch];
      x0 = *reinterpret_cast<const float4*>(acc + (int64_t)ch * DSK_HEAD_DIM);
      x1 = *reinterpret_cast<const float4*>(acc + (int64_t)ch * DSK_HEAD_DIM + 4);
    }
    if (v.x == -__builtin_inff()) continue;
    const float mn = fmaxf(m, v.x);
    const float fo = exp2f(m - mn), fn = exp2f(v.x - mn);   // m = -inf -> fo = 0
    l = l * fo + v.y * fn;
    a[0] = a[0] * fo + x0.x * fn; a[1] = a[1] * fo + x0.y * fn; a[2] = a[2] * fo + x0.z * fn; a[3] = a[3] * fo + x0.w * fn;
    a[4] = a[4] * fo + x1.x * fn; a[5] = a[5] * fo + x1.y * fn; a[6] = a[6] * fo + x1.z * fn; a[7] = a[7] * fo + x1.w * fn;
    m = mn;
  }
  if (c == 0) { sm_m[grp] = m; sm_l[grp] = l; }
#pragma unroll
  for (int i = 0; i < 8; ++i) sm_acc[grp][c * 8 + i] = a[i];
  __syncthreads();
  const int d = threadIdx.x;
  if (d < DSK_HEAD_DIM) {
    float M = sm_m[0];
#pragma unroll
    for (int g2 = 1; g2 < kMergeGroups; ++g2) M = fmaxf(M, sm_m[g2]);
    float L = 0.0f, A = 0.0f;
#pragma unroll
    for (int g2 = 0; g2 < kMergeGroups; ++g2) {
      const float f = sm_m[g2] == -__builtin_inff() ? 0.0f : exp2f(sm_m[g2] - M);
      L = fmaf(sm_l[g2], f, L);
      A = fmaf(sm_acc[g2][d], f, A);
    }
    store_attn_out(out, out_bf16, sh * DSK_HEAD_DIM + d, L > 0.0f ? A / L : 0.0f);
    if (d == 0 && lse) lse[sh] = L > 0.0f ? (M + log2f(L)) * kLn2 : -__builtin_inff();
  }
}

AttnWs attn_ws_layout(const dsk_attn_args& a) {
  AttnWs ws;
  ws.slots_per_wg = attn_shared_tiled(a) ? kSharedWaves * kSharedSpw : attn_slots_per_wg(a.b);
  if (!attn_shared_tiled(a) && a.b <= 16 &&
      (int64_t)a.B * a.Hq * ((a.k + ws.slots_per_wg - 1) / ws.slots_per_wg) >= kAttnSmallWgFrom)
    ws.slots_per_wg = 8;
  ws.nchunks = (a.k + ws.slots_per_wg - 1) / ws.slots_per_wg;
  const size_t n = (size_t)a.B * a.Hq * ws.nchunks;
  ws.part_ml = 0;
  ws.part_acc = align_up(n * sizeof(float2));
  ws.total = ws.part_acc + align_up(n * DSK_HEAD_DIM * sizeof(float));
  return ws;
}

hipError_t launch_attn(const dsk_attn_args& a, const AttnWs& ws, hipStream_t st) {
  unsigned char* w = static_cast<unsigned char*>(a.workspace);
  float2* part_ml = reinterpret_cast<float2*>(w + ws.part_ml);
  float* part_acc = reinterpret_cast<float*>(w + ws.part_acc);
  const float scale = a.scale != 0.0f ? a.scale : 0.08838834764831845f;   // 128^-1/2
  const int n_groups = a.B * a.Hkv;
  const dim3 grid(a.Hq == a.Hkv ? (unsigned)(n_groups * ws.nchunks)
                                : (unsigned)(8 * ((n_groups + 7) / 8) * (a.Hq / a.Hkv) * ws.nchunks));

  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  const uint16_t* K = static_cast<const uint16_t*>(a.K);
  const uint16_t* V = static_cast<const uint16_t*>(a.V);
  // heads that read one row of the selection arrays; the workgroups of a group's heads gather the
  // same rows on one XCD, so only one of them misses in L2
  const int sel_div = (a.flags & DSK_ATTN_SHARED_SELECTION) ? a.Hq / a.Hkv : 1;
  if (attn_shared_tiled(a)) {
    const int G = a.Hq / a.Hkv;
    const int GT = G == 2 ? 2 : 4;
    const dim3 sgrid((unsigned)ws.nchunks, (unsigned)(a.Hkv * (G / GT)), (unsigned)a.B);
    const dim3 sblock(kSharedWaves * DSK_WAVE);
#define DSK_SHARED_ARGS                                                                                        \
  q, K, V, a.k_stride_tok, a.k_stride_head, a.v_stride_tok, a.v_stride_head, a.Hq, G, a.k, a.b, a.total_tokens, \
      a.sel_start, a.sel_len, a.sel_count, scale * kLog2e, ws.nchunks, part_ml, part_acc, a.out,                \
      static_cast<uint16_t*>(a.out_bf16), a.lse
    if (GT == 2) {
      if (a.b <= 16) attn_shared_kernel<4, kSharedSpw, kSharedWaves, 2><<<sgrid, sblock, 0, st>>>(DSK_SHARED_ARGS);
      else attn_shared_kernel<8, kSharedSpw, kSharedWaves, 2><<<sgrid, sblock, 0, st>>>(DSK_SHARED_ARGS);
    } else {
      if (a.b <= 16) attn_shared_kernel<4, kSharedSpw, kSharedWaves, 4><<<sgrid, sblock, 0, st>>>(DSK_SHARED_ARGS);
      else attn_shared_kernel<8, kSharedSpw, kSharedWaves, 4><<<sgrid, sblock, 0, st>>>(DSK_SHARED_ARGS);
    }
#undef DSK_SHARED_ARGS
    hipError_t serr = hipGetLastError();
    if (serr != hipSuccess || ws.nchunks <= 1 || (a.flags & DSK_ATTN_PARTIALS_ONLY) || a.total_tokens <= 0) return serr;
    return launch_attn_merge(part_ml, part_acc, a.sel_count, nullptr, a.B, a.Hq, sel_div, a.k, ws.nchunks,
                             ws.slots_per_wg, a.out, static_cast<uint16_t*>(a.out_bf16), a.lse, st);
  }
#define DSK_ATTN_ARGS                                                                                          \
  q, K, V, a.k_stride_tok, a.k_stride_head, a.v_stride_tok, a.v_stride_head, a.Hq, a.Hq / a.Hkv, n_groups, a.k, a.b, \
      a.total_tokens, a.sel_start, a.sel_len, a.sel_count, sel_div, scale * kLog2e, ws.nchunks, part_ml, part_acc, a.out, \
      static_cast<uint16_t*>(a.out_bf16), a.lse
  // Slots of at most 32 rows: workgroups of 8 wavefronts, 2 slots each (16 slots per workgroup).
  // Measured against 4 wavefronts x 2 or 4 slots, 8 x 1 or 4, 16 x 1 or 2 on all configurations:
  // the gather takes 7.3 instead of 8.6 us at 128K / b = 32, and 4.6 instead of 5.6 us at
  // 32K / b = 16 (half as many workgroups to dispatch and half as many partials to merge).
  if (a.b <= 16 && ws.slots_per_wg == 8) attn_kernel<4, 2, 4, false><<<grid, dim3(256), 0, st>>>(DSK_ATTN_ARGS);
  else if (a.b <= 16) attn_kernel<4, 2, 8, false><<<grid, dim3(512), 0, st>>>(DSK_ATTN_ARGS);
  else if (a.b <= 32) attn_kernel<8, 2, 8, true><<<grid, dim3(512), 0, st>>>(DSK_ATTN_ARGS);
  else attn_kernel<0, 2, 4><<<grid, dim3(256), 0, st>>>(DSK_ATTN_ARGS);
#undef DSK_ATTN_ARGS
  hipError_t err = hipGetLastError();
  // a cache without tokens: every head already holds the defined empty result, no partial exists
  if (err != hipSuccess || ws.nchunks <= 1 || (a.flags & DSK_ATTN_PARTIALS_ONLY) || a.total_tokens <= 0) return err;
  return launch_attn_merge(part_ml, part_acc, a.sel_count, nullptr, a.B, a.Hq, sel_div, a.k, ws.nchunks,
                           ws.slots_per_wg, a.out, static_cast<uint16_t*>(a.out_bf16), a.lse, st);
}

hipError_t launch_attn_merge(const float2* part_ml, const float* part_acc, const int32_t* counts,
                             const int32_t* cu_seqlens, int B, int Hq, int sel_div, int k, int nchunks, int per_chunk,
                             float* out, uint16_t* out_bf16, float* lse, hipStream_t st) {
  // one lane group of 16 per partial when there are few, several partials per group otherwise
  const dim3 grid((unsigned)(B * Hq));
  if (nchunks <= 8)
    attn_merge_kernel<128><<<grid, dim3(128), 0, st>>>(part_ml, part_acc, counts, cu_seqlens, Hq, sel_div, k, nchunks,
                                                       per_chunk, out, out_bf16, lse);
  else if (nchunks <= 32)
    attn_merge_kernel<256><<<grid, dim3(256), 0, st>>>(part_ml, part_acc, counts, cu_seqlens, Hq, sel_div, k, nchunks,
                                                       per_chunk, out, out_bf16, lse);
  else
    attn_merge_kernel<kMergeBigThreads><<<grid, dim3(kMergeBigThreads), 0, st>>>(
        part_ml, part_acc, counts, cu_seqlens, Hq, sel_div, k, nchunks, per_chunk, out, out_bf16, lse);
  return hipGetLastError();
}

}  // namespace dsk
