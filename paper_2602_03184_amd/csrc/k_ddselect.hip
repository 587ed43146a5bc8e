// DD-Select segmentation (Sec. 4.1, Dynamic Segmentation Procedure) and the variable-to-
// fixed slot map (Sec. 4.2), integer-exact.
//
// The procedure is a chain s_c -> e*(s_c) whose successor depends only on s_c and static
// data, and it only moves forward by at most C + delta.  It is parallelised by cutting every
// sequence into tiles of kSegTile positions:
//   1. mark:   dense byte array  boundary position e -> weight tenths of the delimiter at
//              e-1 (255 = no delimiter offers e).
//   2. maps:   per tile, the successor of every position in LDS, then for every possible
//              entry offset (< C + delta) a walk to the tile's end: (exit position, blocks,
//              slots) of that entry.
//   3. chain:  per sequence, hop through the tile maps (staged in LDS) to fix each tile's
//              real entry and its block / slot offsets.
//   4. scan:   block and slot bases of the sequences of the batch, capacity check.
//   5. emit:   per tile, walk from the real entry and write block_start / slot_base.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kSegThreads = 256;
constexpr int kChainLdsEntries = 6144;   // uint2 entries staged per chunk in the chain kernel (48 KB)

struct SegParams {
  const int32_t* cu_seqlens;
  const int32_t* C_per_seq;
  const int32_t* delta_per_seq;
  int C, delta, a_num, a_den, b;
  int map_row, tiles_per_seq;
  int max_seqlen, total_tokens;
};

// cu_seqlens must agree with the host copies the launch geometry and buffers were sized on
__device__ __forceinline__ bool seq_ok(const SegParams& p, int seq0, int L) {
  return seq0 >= 0 && L >= 0 && L <= p.max_seqlen && seq0 + L <= p.total_tokens;
}

__device__ __forceinline__ void seq_params(const SegParams& p, int s, int& C, int& delta, int32_t* dev_status) {
  C = p.C_per_seq ? p.C_per_seq[s] : p.C;
  delta = p.delta_per_seq ? p.delta_per_seq[s] : p.delta;
  if (C < 1 || C > p.C || delta < 0 || delta >= C || delta > p.delta) {
    // out-of-contract per-sequence values: clamp into the validated envelope so that the
    // LDS tiles sized on the host stay large enough and every chunk stays non-empty
    if (threadIdx.x == 0) set_status(dev_status, DSK_ERR_PARAM);
    C = C < 1 ? 1 : (C > p.C ? p.C : C);
    int dmax = p.delta < C - 1 ? p.delta : C - 1;
    delta = delta < 0 ? 0 : (delta > dmax ? dmax : delta);
  }
}

// ---- 1. markers -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void seg_fill_kernel(uint8_t* __restrict__ marker, int n) {
  // n bytes, n padded to a multiple of 16 by the workspace layout
  uint4* m = reinterpret_cast<uint4*>(marker);
  const int n16 = (n + 15) / 16;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += gridDim.x * blockDim.x)
    m[i] = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
}

__global__ __launch_bounds__(256) void seg_scatter_kernel(
    const int32_t* __restrict__ cand_pos, const uint8_t* __restrict__ cand_class,
    const int32_t* __restrict__ cand_cu, const int32_t* __restrict__ cu_seqlens, int B, int n_class,
    int max_cand, const uint8_t* __restrict__ class_weight_q, uint8_t* __restrict__ marker,
    int32_t* dev_status) {
  int n = cand_cu[B];
  if (n > max_cand) n = max_cand;
  for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
    // sequence of candidate j: last s with cand_cu[s] <= j
    int lo = 0, hi = B;   // invariant cand_cu[lo] <= j < cand_cu[hi]
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (cand_cu[mid] <= j) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int t = cand_pos[j];
    const int cls = cand_class[j];
    if (t < cu_seqlens[s] || t >= cu_seqlens[s + 1] || cls >= n_class) {
      set_status(dev_status, DSK_ERR_SHAPE);
      continue;
    }
    int w = class_weight_q[s * n_class + cls];
    if (w > 10) { set_status(dev_status, DSK_ERR_PARAM); w = 10; }
    marker[t + 1] = (uint8_t)w;
  }
}

// ---- 2 / 5. tile kernel ---------------------------------------------------------------------
// LDS: nxt[kSegTile] u16 (successor - position), ns[kSegTile] u16 (slots of that chunk),
//      mk[kSegTile + 2*delta_max + 1] u8 (markers of the boundaries the tile's windows touch)
template <int MODE>
__global__ __launch_bounds__(kSegThreads) void seg_tile_kernel(
    SegParams p, const uint8_t* __restrict__ marker, uint2* __restrict__ tile_map,
    int4* __restrict__ tile_info, const int4* __restrict__ seq_info, int32_t* __restrict__ block_start,
    int32_t* __restrict__ slot_base, int cap, int32_t* dev_status) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* nxt = reinterpret_cast<uint16_t*>(smem);
  uint16_t* ns = nxt + kSegTile;
  uint8_t* mk = reinterpret_cast<uint8_t*>(ns + kSegTile);

  const int s = blockIdx.y;
  const int j = blockIdx.x;
  const int seq0 = p.cu_seqlens[s];
  const int L = p.cu_seqlens[s + 1] - seq0;
  if (!seq_ok(p, seq0, L)) {
    if (threadIdx.x == 0) set_status(dev_status, DSK_ERR_SHAPE);
    return;
  }
  const int p0 = j * kSegTile;
  if (p0 >= L) return;
  const int p1 = (p0 + kSegTile < L) ? p0 + kSegTile : L;
  int C, delta;
  seq_params(p, s, C, delta, dev_status);
  const int dd = delta > 1 ? delta : 1;
  const int tid = threadIdx.x;

  // boundaries any window of this tile can touch: [p0 + C - delta, min(L, p1 - 1 + C + delta)]
  const int mlo = p0 + C - delta;
  int mhi = p1 - 1 + C + delta;
  if (mhi > L) mhi = L;
  for (int e = mlo + tid; e <= mhi; e += kSegThreads) mk[e - mlo] = marker[seq0 + e];
  __syncthreads();

  for (int q = p0 + tid; q < p1; q += kSegThreads) {
    const int s_e = q + C;
    int n;
    if (s_e >= L) {
      n = L;
    } else {
      const int lo = s_e - delta;
      const int hi = (s_e + delta < L) ? s_e + delta : L;
      int best = -1, best_e = s_e;
      for (int e = lo; e <= hi; ++e) {
        const int w = mk[e - mlo];
        if (w != 255) {
          const int dist = e > s_e ? e - s_e : s_e - e;
          const int sc = p.a_num * w * dd + (p.a_den - p.a_num) * 10 * (dd - dist);
          if (sc > best) { best = sc; best_e = e; }   // strict: ties keep the smaller e
        }
      }
      n = best_e;
    }
    const int len = n - q;
    nxt[q - p0] = (uint16_t)len;
    ns[q - p0] = (uint16_t)((len + p.b - 1) / p.b);
  }
  __syncthreads();

  const int tile = s * p.tiles_per_seq + j;
  if (MODE == 0) {
    const int tlen = p1 - p0;
    uint2* row = tile_map + (int64_t)tile * p.map_row;
    for (int ent = tid; ent < p.map_row; ent += kSegThreads) {
      uint2 r = make_uint2(0u, 0u);
      if (ent < tlen) {
        int q = p0 + ent, cnt = 0, slots = 0;
        while (q < p1) {
          slots += ns[q - p0];
          q += nxt[q - p0];
          ++cnt;
        }
        r = make_uint2((uint32_t)(q - p1) | ((uint32_t)cnt << 16), (uint32_t)slots);
      }
      row[ent] = r;
    }
  } else {
    if (tid == 0) {
      const int4 info = tile_info[tile];
      const int4 sq = seq_info[s];
      int q = info.x;
      int gb = sq.z + info.y;
      int gs = sq.w + info.z;
      while (q < p1) {
        if (gb < cap) {
          block_start[gb] = seq0 + q;
          slot_base[gb] = gs;
        }
        gs += ns[q - p0];
        q += nxt[q - p0];
        ++gb;
      }
    }
  }
}

// ---- 3. chain -------------------------------------------------------------------------------
__global__ __launch_bounds__(kSegThreads) void seg_chain_kernel(
    SegParams p, const uint2* __restrict__ tile_map, int4* __restrict__ tile_info,
    int4* __restrict__ seq_info) {
  __shared__ uint2 rows[kChainLdsEntries];
  __shared__ int carry[3];
  const int s = blockIdx.x;
  int L = p.cu_seqlens[s + 1] - p.cu_seqlens[s];
  if (!seq_ok(p, p.cu_seqlens[s], L)) L = 0;   // flagged by the tile kernel; emit nothing
  const int n_tiles = (L + kSegTile - 1) / kSegTile;
  const int tiles_per_chunk = kChainLdsEntries / p.map_row;   // map_row <= kSegTile <= entries
  if (threadIdx.x == 0) { carry[0] = 0; carry[1] = 0; carry[2] = 0; }
  for (int j0 = 0; j0 < n_tiles; j0 += tiles_per_chunk) {
    const int jn = (n_tiles - j0 < tiles_per_chunk) ? n_tiles - j0 : tiles_per_chunk;
    const uint2* src = tile_map + ((int64_t)s * p.tiles_per_seq + j0) * p.map_row;
    __syncthreads();
    for (int i = threadIdx.x; i < jn * p.map_row; i += kSegThreads) rows[i] = src[i];
    __syncthreads();
    if (threadIdx.x == 0) {
      int entry = carry[0], blk = carry[1], slots = carry[2];
      for (int jj = 0; jj < jn; ++jj) {
        const int j = j0 + jj;
        const int t0 = j * kSegTile;
        const int t1 = (t0 + kSegTile < L) ? t0 + kSegTile : L;
        tile_info[s * p.tiles_per_seq + j] = make_int4(entry, blk, slots, 0);
        if (entry < t1) {   // entry >= t1: a chunk longer than a tile jumps over it
          const uint2 r = rows[jj * p.map_row + (entry - t0)];
          blk += (int)(r.x >> 16);
          slots += (int)r.y;
          entry = t1 + (int)(r.x & 0xFFFFu);
        }
      }
      carry[0] = entry; carry[1] = blk; carry[2] = slots;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) seq_info[s] = make_int4(carry[1], carry[2], 0, 0);
}

// ---- 4. scan over the sequences of the batch ------------------------------------------------
__global__ __launch_bounds__(64) void seg_seqscan_kernel(
    int4* __restrict__ seq_info, int B, int cap, int total_tokens, int32_t* __restrict__ cu_blocks,
    int32_t* __restrict__ block_start, int32_t* __restrict__ slot_base, int32_t* dev_status) {
  if (threadIdx.x != 0) return;
  int blk = 0, slots = 0;
  for (int s = 0; s < B; ++s) {
    int4 v = seq_info[s];
    cu_blocks[s] = blk;
    v.z = blk;
    v.w = slots;
    seq_info[s] = v;
    blk += v.x;
    slots += v.y;
  }
  cu_blocks[B] = blk;
  if (blk > cap) {
    set_status(dev_status, DSK_ERR_CAPACITY);
    // keep the tables self-consistent for the truncated prefix
    return;
  }
  block_start[blk] = total_tokens;
  slot_base[blk] = slots;
}

// ---- host -----------------------------------------------------------------------------------
static size_t seg_tile_lds_bytes(const dsk_compress_args& a) {
  return (size_t)kSegTile * 4 + (size_t)kSegTile + 2 * (size_t)a.delta + 16;
}

hipError_t launch_segment(const dsk_compress_args& a, const CompressWs& ws, hipStream_t st) {
  unsigned char* w = static_cast<unsigned char*>(a.workspace);
  uint8_t* marker = w + ws.marker;
  uint2* tile_map = reinterpret_cast<uint2*>(w + ws.tile_map);
  int4* tile_info = reinterpret_cast<int4*>(w + ws.tile_info);
  int4* seq_info = reinterpret_cast<int4*>(w + ws.seq_info);

  SegParams p;
  p.cu_seqlens = a.cu_seqlens;
  p.C_per_seq = a.C_per_seq;
  p.delta_per_seq = a.delta_per_seq;
  p.C = a.C; p.delta = a.delta; p.a_num = a.alpha_num; p.a_den = a.alpha_den; p.b = a.b;
  p.map_row = ws.map_row; p.tiles_per_seq = ws.tiles_per_seq;
  p.max_seqlen = a.max_seqlen; p.total_tokens = a.total_tokens;

  hipError_t err;
  const int nmark = a.total_tokens + 1;
  {
    int n16 = (nmark + 15) / 16;
    int wgs = (n16 + 255) / 256;
    if (wgs > 1024) wgs = 1024;
    seg_fill_kernel<<<dim3(wgs), dim3(256), 0, st>>>(marker, nmark);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (a.max_cand_total > 0) {
    int wgs = (a.max_cand_total + 255) / 256;
    if (wgs > 1024) wgs = 1024;
    seg_scatter_kernel<<<dim3(wgs), dim3(256), 0, st>>>(a.cand_pos, a.cand_class, a.cand_cu, a.cu_seqlens,
                                                         a.B, a.n_class, a.max_cand_total, a.class_weight_q,
                                                         marker, a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  const size_t lds = seg_tile_lds_bytes(a);
  if (ws.tiles_per_seq > 0) {
    const dim3 grid((unsigned)ws.tiles_per_seq, (unsigned)a.B);
    seg_tile_kernel<0><<<grid, dim3(kSegThreads), lds, st>>>(p, marker, tile_map, tile_info, seq_info,
                                                             a.block_start, a.slot_base, a.max_blocks_total,
                                                             a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  seg_chain_kernel<<<dim3((unsigned)a.B), dim3(kSegThreads), 0, st>>>(p, tile_map, tile_info, seq_info);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  seg_seqscan_kernel<<<dim3(1), dim3(64), 0, st>>>(seq_info, a.B, a.max_blocks_total, a.total_tokens,
                                                   a.cu_blocks, a.block_start, a.slot_base, a.dev_status);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (ws.tiles_per_seq > 0) {
    const dim3 grid((unsigned)ws.tiles_per_seq, (unsigned)a.B);
    seg_tile_kernel<1><<<grid, dim3(kSegThreads), lds, st>>>(p, marker, tile_map, tile_info, seq_info,
                                                             a.block_start, a.slot_base, a.max_blocks_total,
                                                             a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  return hipSuccess;
}

}  // namespace dsk
