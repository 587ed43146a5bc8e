// Candidate delimiter positions (input set D of Alg. 1; semantic boundary tokens of Sec. 4.1)
// and the per-class samples Alg. 1 is evaluated on.
//   classify: token id -> class byte (index in delim_ids, 255 = not a delimiter), per-tile counts
//   scan:     exclusive scan of the tile counts, candidate range of every sequence
//   scatter:  stream compaction into cand_pos / cand_class (ascending by construction)
//   sample:   per (sequence, class) the first M candidates with R <= t <= L-1-W
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kCandThreads = 256;
constexpr int kCandWaves = kCandThreads / DSK_WAVE;
static_assert(kCandTile == kCandThreads * 4, "one thread classifies 4 consecutive tokens");

__device__ __forceinline__ int wg_excl_scan_small(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int incl = wave_incl_scan_i(v, lane);
  __syncthreads();
  if (lane == DSK_WAVE - 1) wave_tot[wave] = incl;
  __syncthreads();
  int off = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < kCandWaves; ++w) {
    const int t = wave_tot[w];
    if (w < wave) off += t;
    total += t;
  }
  return off + incl - v;
}

__global__ __launch_bounds__(kCandThreads) void cand_classify_kernel(
    const int32_t* __restrict__ token_ids, int total_tokens, const int32_t* __restrict__ delim_ids,
    int n_class, uint8_t* __restrict__ cls_at, int32_t* __restrict__ tile_count) {
  __shared__ int32_t ids[DSK_MAX_CLASSES];
  __shared__ int wave_tot[kCandWaves];
  if ((int)threadIdx.x < n_class) ids[threadIdx.x] = delim_ids[threadIdx.x];
  __syncthreads();
  const int t0 = blockIdx.x * kCandTile + threadIdx.x * 4;
  int cnt = 0;
  uint8_t cls[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    cls[u] = 255;
    const int t = t0 + u;
    if (t < total_tokens) {
      const int tok = token_ids[t];
      for (int c = n_class - 1; c >= 0; --c) if (tok == ids[c]) cls[u] = (uint8_t)c;
      if (cls[u] != 255) ++cnt;
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) if (t0 + u < total_tokens) cls_at[t0 + u] = cls[u];
  int total;
  wg_excl_scan_small(cnt, wave_tot, total);
  if (threadIdx.x == 0) tile_count[blockIdx.x] = total;
}

__global__ __launch_bounds__(kCandThreads) void cand_scan_kernel(
    int32_t* __restrict__ tile_count, int n_tiles, const uint8_t* __restrict__ cls_at,
    const int32_t* __restrict__ cu_seqlens, int B, int total_tokens, int max_cand,
    int32_t* __restrict__ cand_cu, int32_t* dev_status) {
  __shared__ int wave_tot[kCandWaves];
  __shared__ int carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_tiles; base += kCandThreads) {
    const int i = base + threadIdx.x;
    const int v = i < n_tiles ? tile_count[i] : 0;
    int total;
    const int excl = wg_excl_scan_small(v, wave_tot, total);
    if (i < n_tiles) tile_count[i] = carry + excl;
    __syncthreads();
    if (threadIdx.x == 0) carry += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    tile_count[n_tiles] = carry;
    if (carry > max_cand) set_status(dev_status, DSK_ERR_CAPACITY);
  }
  __syncthreads();
  // candidate range of every sequence: exclusive count at its first token.  One wavefront per
  // boundary; the partial tile in front of it is counted with all loads in flight.
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  for (int s = wave; s <= B; s += kCandWaves) {
    const int p = cu_seqlens[s];
    int c;
    if (p >= total_tokens || p < 0) {
      c = p < 0 ? 0 : carry;
    } else {
      const int tile = p / kCandTile;
      const int t0 = tile * kCandTile;
      int part = 0;
#pragma unroll
      for (int u = 0; u < kCandTile / DSK_WAVE; ++u) {
        const int t = t0 + u * DSK_WAVE + lane;
        const uint8_t cl = cls_at[t < p ? t : t0];           // t0 <= p < total_tokens: in bounds
        part += (t < p && cl != 255) ? 1 : 0;
      }
      c = tile_count[tile] + wave_sum_i(part);
    }
    if (lane == 0) cand_cu[s] = c;
  }
}

__global__ __launch_bounds__(kCandThreads) void cand_scatter_kernel(
    const uint8_t* __restrict__ cls_at, int total_tokens, const int32_t* __restrict__ tile_base,
    int max_cand, int32_t* __restrict__ cand_pos, uint8_t* __restrict__ cand_class) {
  __shared__ int wave_tot[kCandWaves];
  const int t0 = blockIdx.x * kCandTile + threadIdx.x * 4;
  uint8_t cls[4];
  int cnt = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    cls[u] = (t0 + u < total_tokens) ? cls_at[t0 + u] : (uint8_t)255;
    cnt += (cls[u] != 255);
  }
  int total;
  int o = tile_base[blockIdx.x] + wg_excl_scan_small(cnt, wave_tot, total);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (cls[u] != 255) {
      if (o < max_cand) { cand_pos[o] = t0 + u; cand_class[o] = cls[u]; }
      ++o;
    }
  }
}

// one wavefront per (class, sequence)
__global__ __launch_bounds__(DSK_WAVE) void cand_sample_kernel(
    const int32_t* __restrict__ cand_pos, const uint8_t* __restrict__ cand_class,
    const int32_t* __restrict__ cand_cu, const int32_t* __restrict__ cu_seqlens, int n_class, int M,
    int R, int W, int max_cand, int32_t* __restrict__ samp_pos) {
  const int c = blockIdx.x;
  const int s = blockIdx.y;
  const int lane = threadIdx.x;
  const int seq0 = cu_seqlens[s];
  const int L = cu_seqlens[s + 1] - seq0;
  int j0 = cand_cu[s];
  int j1 = cand_cu[s + 1];
  if (j1 > max_cand) j1 = max_cand;
  int32_t* out = samp_pos + ((int64_t)s * n_class + c) * M;
  int found = 0;
  for (int base = j0; base < j1 && found < M; base += DSK_WAVE) {
    const int j = base + lane;
    bool hit = false;
    int t = 0;
    if (j < j1) {
      t = cand_pos[j];
      const int tl = t - seq0;
      hit = (cand_class[j] == c) && tl >= R && tl <= L - 1 - W;
    }
    const unsigned long long bal = __ballot(hit);
    const int rank = found + __popcll(bal & ((1ull << lane) - 1ull));
    if (hit && rank < M) out[rank] = t;
    found += __popcll(bal);
  }
  if (found > M) found = M;
  for (int m = found + lane; m < M; m += DSK_WAVE) out[m] = -1;
}

hipError_t launch_candidates(const dsk_compress_args& a, const CompressWs& ws, hipStream_t st) {
  unsigned char* w = static_cast<unsigned char*>(a.workspace);
  uint8_t* cls_at = w + ws.cls_at;
  int32_t* tile_count = reinterpret_cast<int32_t*>(w + ws.tile_count);
  hipError_t err;
  if (ws.n_cand_tiles > 0) {
    cand_classify_kernel<<<dim3((unsigned)ws.n_cand_tiles), dim3(kCandThreads), 0, st>>>(
        a.token_ids, a.total_tokens, a.delim_ids, a.n_class, cls_at, tile_count);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  cand_scan_kernel<<<dim3(1), dim3(kCandThreads), 0, st>>>(tile_count, ws.n_cand_tiles, cls_at, a.cu_seqlens, a.B,
                                                           a.total_tokens, a.max_cand_total, a.cand_cu,
                                                           a.dev_status);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (ws.n_cand_tiles > 0) {
    cand_scatter_kernel<<<dim3((unsigned)ws.n_cand_tiles), dim3(kCandThreads), 0, st>>>(
        cls_at, a.total_tokens, tile_count, a.max_cand_total, a.cand_pos, a.cand_class);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  return launch_cand_sample(a, st);
}

hipError_t launch_cand_sample(const dsk_compress_args& a, hipStream_t st) {
  if (a.samp_pos != nullptr && a.M > 0) {
    cand_sample_kernel<<<dim3((unsigned)a.n_class, (unsigned)a.B), dim3(DSK_WAVE), 0, st>>>(
        a.cand_pos, a.cand_class, a.cand_cu, a.cu_seqlens, a.n_class, a.M, a.R, a.W, a.max_cand_total,
        a.samp_pos);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace dsk
