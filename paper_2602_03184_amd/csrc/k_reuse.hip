// KV reuse over fixed-size slots (App. B.2, "KVCache Reuse with V2F").
//
// Every (sequence, query head) owns a resident buffer of k positions of b rows.  A step's
// selection is compared with what the buffer holds: slots held and selected again stay where
// they are (cut, for all heads of the sequence, to the smallest such count r), the others are
// copied from the K/V source into the positions that are not kept.
//
// Three kernels, one wavefront per (sequence, head) in the first two:
//   reuse_count_kernel  reusable entries of each head                      (Step 1, first half)
//   reuse_plan_kernel   r = min over the heads; kept / free positions; load list; the buffer's
//                       description as a selection                         (Steps 1-3)
//   reuse_load_kernel   one wavefront per load copies the slot's K and V rows   (Step 3)
// The wavefronts of a workgroup never talk to each other: each owns a quarter of the LDS arrays
// and orders its own LDS traffic with wave-level fences, so there is no workgroup barrier.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

namespace {

constexpr int kReuseWaves = 4;   // heads per workgroup in the count / plan kernels
constexpr int kReuseMaxK = DSK_REUSE_MAX_K;

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ int popc_below(uint64_t mask, int lane) {
  return __popcll(mask & ((1ull << lane) - 1ull));
}

// copies the head's selection (first n entries) into the wave's LDS row
__device__ __forceinline__ void stage_selection(int* sel, const int32_t* __restrict__ sel_slot, int n, int lane) {
  for (int j = lane; j < n; j += DSK_WAVE) sel[j] = sel_slot[j];
  wave_lds_fence();
}

// index of slot x in the ascending row sel[0..n), or -1
__device__ __forceinline__ int find_slot(const int* sel, int n, int x) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (sel[mid] < x) lo = mid + 1;
    else hi = mid;
  }
  return (lo < n && sel[lo] == x) ? lo : -1;
}

// index in the selection of the slot held at position p, or -1 when the position is empty, the
// slot is not selected again, or it lies in the stale tail
__device__ __forceinline__ int match_position(const int* sel, int n, const int32_t* __restrict__ res_slot, int p, int k,
                                              int stale) {
  if (p >= k) return -1;
  const int x = res_slot[p];
  if (x < 0 || x >= stale) return -1;
  return find_slot(sel, n, x);
}

__global__ __launch_bounds__(kReuseWaves * DSK_WAVE) void reuse_count_kernel(
    const int32_t* __restrict__ sel_slot, const int32_t* __restrict__ sel_count,
    const int32_t* __restrict__ stale_from, const int32_t* __restrict__ res_slot, int Hq, int k,
    int32_t* __restrict__ cnt) {
  __shared__ int sm_sel[kReuseWaves][kReuseMaxK];
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int h = blockIdx.x * kReuseWaves + wave;
  const int s = blockIdx.y;
  if (h >= Hq) return;
  const int64_t sh = (int64_t)s * Hq + h;
  int n = sel_count[sh];
  n = n < 0 ? 0 : (n > k ? k : n);
  const int stale = stale_from ? stale_from[s] : 0x7FFFFFFF;
  int* sel = sm_sel[wave];
  stage_selection(sel, sel_slot + sh * k, n, lane);
  int total = 0;
  for (int p0 = 0; p0 < k; p0 += DSK_WAVE) {
    const int m = match_position(sel, n, res_slot + sh * k, p0 + lane, k, stale);
    total += __popcll(__ballot(m >= 0));
  }
  if (lane == 0) cnt[sh] = total;
}

__global__ __launch_bounds__(kReuseWaves * DSK_WAVE) void reuse_plan_kernel(
    const int32_t* __restrict__ sel_slot, const int32_t* __restrict__ sel_start,
    const int32_t* __restrict__ sel_len, const int32_t* __restrict__ sel_count,
    const int32_t* __restrict__ stale_from, const int32_t* __restrict__ cnt, int Hq, int k, int b,
    int32_t* __restrict__ res_slot, int32_t* __restrict__ res_len, int32_t* __restrict__ res_start,
    int32_t* __restrict__ res_count, int32_t* __restrict__ load_pos, int32_t* __restrict__ load_slot,
    int32_t* __restrict__ load_start, int32_t* __restrict__ load_len, int32_t* __restrict__ load_count,
    int32_t* __restrict__ reuse_count) {
  __shared__ int sm_sel[kReuseWaves][kReuseMaxK];
  __shared__ uint16_t sm_free[kReuseWaves][kReuseMaxK];
  __shared__ uint8_t sm_kept[kReuseWaves][kReuseMaxK];
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int h = blockIdx.x * kReuseWaves + wave;
  const int s = blockIdx.y;
  if (h >= Hq) return;
  const int64_t sh = (int64_t)s * Hq + h;
  const int64_t base = sh * k;
  int n = sel_count[sh];
  n = n < 0 ? 0 : (n > k ? k : n);
  const int stale = stale_from ? stale_from[s] : 0x7FFFFFFF;

  // Step 1: r = the smallest reusable count over the heads of this sequence
  uint32_t rmin = 0xFFFFFFFFu;
  for (int hh = lane; hh < Hq; hh += DSK_WAVE) {
    const uint32_t c = (uint32_t)cnt[(int64_t)s * Hq + hh];
    rmin = c < rmin ? c : rmin;
  }
  const int r = (int)wave_min_u(rmin);
  if (h == 0 && lane == 0) reuse_count[s] = r;

  int* sel = sm_sel[wave];
  uint16_t* freepos = sm_free[wave];
  uint8_t* kept_sel = sm_kept[wave];
  for (int j = lane; j < n; j += DSK_WAVE) kept_sel[j] = 0;
  stage_selection(sel, sel_slot + base, n, lane);

  // positions: the first r reusable ones stay; the others are free, in ascending order
  int run = 0, nfree = 0, last = -1;
  for (int p0 = 0; p0 < k; p0 += DSK_WAVE) {
    const int p = p0 + lane;
    const int m = match_position(sel, n, res_slot + base, p, k, stale);
    const uint64_t reusable = __ballot(m >= 0);
    const bool kept = m >= 0 && run + popc_below(reusable, lane) < r;
    const uint64_t is_free = __ballot(p < k && !kept);
    if (kept) {
      kept_sel[m] = 1;
      last = p;
    } else if (p < k) {
      freepos[nfree + popc_below(is_free, lane)] = (uint16_t)p;
    }
    if (p < k) res_start[base + p] = (int32_t)(((int64_t)s * k + p) * b);
    run += __popcll(reusable);
    nfree += __popcll(is_free);
  }
  wave_lds_fence();

  // Steps 2-3: the selected slots that are not kept, in selection order, into the free positions
  int nload = 0;
  for (int j0 = 0; j0 < n; j0 += DSK_WAVE) {
    const int j = j0 + lane;
    const bool need = j < n && kept_sel[j] == 0;
    const uint64_t needs = __ballot(need);
    const int i = nload + popc_below(needs, lane);
    if (need && i < nfree) {
      const int pos = freepos[i];
      int len = sel_len[base + j];
      len = len < 0 ? 0 : (len > b ? b : len);
      load_pos[base + i] = pos;
      load_slot[base + i] = sel[j];
      load_start[base + i] = sel_start[base + j];
      load_len[base + i] = len;
      res_slot[base + pos] = sel[j];
      res_len[base + pos] = len;
      last = pos > last ? pos : last;
    }
    nload += __popcll(needs);
  }
  nload = nload < nfree ? nload : nfree;
  // unused load entries and left-over positions
  for (int i = nload + lane; i < k; i += DSK_WAVE) {
    load_pos[base + i] = -1;
    load_slot[base + i] = -1;
    load_start[base + i] = 0;
    load_len[base + i] = 0;
    if (i < nfree) {
      const int pos = freepos[i];
      res_slot[base + pos] = -1;
      res_len[base + pos] = 0;
    }
  }
  const int top = (int)wave_max_u((uint32_t)(last + 1));
  if (lane == 0) {
    res_count[sh] = top;
    load_count[sh] = nload;
  }
}

// One wavefront per load: rows of 16 lanes x 16 bytes, four rows per instruction, up to 32 rows
// in flight for K and for V before the stores.
__global__ __launch_bounds__(kReuseWaves * DSK_WAVE) void reuse_load_kernel(
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, int64_t kst, int64_t ksh, int64_t vst,
    int64_t vsh, int total_tokens, int Hq, int G, int k, int b, const int32_t* __restrict__ load_pos,
    const int32_t* __restrict__ load_start, const int32_t* __restrict__ load_len,
    const int32_t* __restrict__ load_count, uint16_t* __restrict__ Kres, uint16_t* __restrict__ Vres,
    int64_t res_head_stride) {
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int i = blockIdx.x * kReuseWaves + wave;
  const int h = blockIdx.y;
  const int s = blockIdx.z;
  const int64_t sh = (int64_t)s * Hq + h;
  int n = load_count[sh];
  n = n > k ? k : n;
  if (i >= n) return;
  const int pos = load_pos[sh * k + i];
  const int start = load_start[sh * k + i];
  int len = load_len[sh * k + i];
  if (pos < 0 || pos >= k) return;
  len = len < 0 ? 0 : (len > b ? b : len);
  if (start < 0 || start > total_tokens - len) len = 0;   // never read outside K/V: the position is zero-filled

  const int g = lane >> 4;
  const int c = lane & 15;
  const int hk = h / G;
  const uint16_t* Ks = K + (int64_t)hk * ksh + c * 8;
  const uint16_t* Vs = V + (int64_t)hk * vsh + c * 8;
  const int64_t row0 = ((int64_t)s * k + pos) * b;
  uint16_t* Kd = Kres + (int64_t)h * res_head_stride + row0 * DSK_HEAD_DIM + c * 8;
  uint16_t* Vd = Vres + (int64_t)h * res_head_stride + row0 * DSK_HEAD_DIM + c * 8;
  for (int r0 = 0; r0 < b; r0 += 32) {
    uint4 kd[8], vd[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = r0 + 4 * u + g;
      kd[u] = make_uint4(0u, 0u, 0u, 0u);
      if (row < len) kd[u] = *reinterpret_cast<const uint4*>(Ks + (int64_t)(start + row) * kst);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = r0 + 4 * u + g;
      vd[u] = make_uint4(0u, 0u, 0u, 0u);
      if (row < len) vd[u] = *reinterpret_cast<const uint4*>(Vs + (int64_t)(start + row) * vst);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = r0 + 4 * u + g;
      if (row < b) {
        *reinterpret_cast<uint4*>(Kd + (int64_t)row * DSK_HEAD_DIM) = kd[u];
        *reinterpret_cast<uint4*>(Vd + (int64_t)row * DSK_HEAD_DIM) = vd[u];
      }
    }
  }
}

}  // namespace

size_t reuse_ws_bytes(const dsk_reuse_args& a) { return align_up((size_t)a.B * a.Hq * sizeof(int32_t)); }

hipError_t launch_reuse(const dsk_reuse_args& a, hipStream_t st) {
  int32_t* cnt = static_cast<int32_t*>(a.workspace);
  const dim3 grid_heads((unsigned)((a.Hq + kReuseWaves - 1) / kReuseWaves), (unsigned)a.B);
  const dim3 block(kReuseWaves * DSK_WAVE);
  reuse_count_kernel<<<grid_heads, block, 0, st>>>(a.sel_slot, a.sel_count, a.stale_from, a.res_slot, a.Hq, a.k, cnt);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  reuse_plan_kernel<<<grid_heads, block, 0, st>>>(a.sel_slot, a.sel_start, a.sel_len, a.sel_count, a.stale_from, cnt,
                                                  a.Hq, a.k, a.b, a.res_slot, a.res_len, a.res_start, a.res_count,
                                                  a.load_pos, a.load_slot, a.load_start, a.load_len, a.load_count,
                                                  a.reuse_count);
  err = hipGetLastError();
  if (err != hipSuccess || (a.flags & DSK_REUSE_PLAN_ONLY)) return err;
  const dim3 grid_load((unsigned)((a.k + kReuseWaves - 1) / kReuseWaves), (unsigned)a.Hq, (unsigned)a.B);
  reuse_load_kernel<<<grid_load, block, 0, st>>>(
      static_cast<const uint16_t*>(a.K), static_cast<const uint16_t*>(a.V), a.k_stride_tok, a.k_stride_head,
      a.v_stride_tok, a.v_stride_head, a.total_tokens, a.Hq, a.Hq / a.Hkv, a.k, a.b, a.load_pos, a.load_start,
      a.load_len, a.load_count, static_cast<uint16_t*>(a.Kres), static_cast<uint16_t*>(a.Vres),
      (int64_t)a.B * a.k * a.b * DSK_HEAD_DIM);
  return hipGetLastError();
}

}  // namespace dsk
