// DD-Select segmentation (Sec. 4.1, Dynamic Segmentation Procedure) and the variable-to-
// fixed slot map (Sec. 4.2), integer-exact.
//
// The procedure is a chain s_c -> e*(s_c) whose successor depends only on s_c and static
// data, and it only moves forward by at most C + delta.  It is parallelised by cutting every
// sequence into tiles of kSegTile positions; input is a dense per-token class byte (255 = not a
// delimiter) produced by the candidate stage, or scattered from the caller's candidate lists.
//   tile<0>: successor of every position of the tile.  Instead of scanning the 2*delta+1
//            boundaries of every position's search range, every delimiter in reach "votes" its
//            packed (score, smaller-e-wins) key into the 2*delta+1 start positions whose range
//            contains it (64-bit LDS atomic max): work is proportional to delimiters, not
//            positions.  Then pointer jumping (successor of successor, log2 rounds) gives, for
//            every position at once, where the chain leaves the tile and how many blocks / slots
//            it lays down on the way; the first C+delta of these form the tile's entry map.
//   chain:   per sequence, hop through the entry maps (staged in LDS) to fix each tile's real
//            entry and its block / slot offsets; for a single-sequence batch also the totals.
//   scan:    block and slot bases of the sequences of a batch (B > 1), capacity check.
//   tile<1>: same successor table; the positions reachable from the real entry are marked
//            with the same doubling scheme, ranked by a workgroup scan and written out.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kSegThreads = 256;
constexpr int kSegPerThread = kSegTile / kSegThreads;   // consecutive positions owned by a thread
constexpr int kSegWaves = kSegThreads / DSK_WAVE;
constexpr int kChainLdsEntries = 6144;   // uint2 entries staged per chunk in the chain kernel (48 KB)

struct SegParams {
  const int32_t* cu_seqlens;
  const int32_t* C_per_seq;
  const int32_t* delta_per_seq;
  const uint8_t* class_weight_q;   // [B, n_class]
  int n_class;
  int C, delta, a_num, a_den, b;
  int map_row, tiles_per_seq;
  int max_seqlen, total_tokens;
  int B, cap;
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

// ---- dense class bytes from caller-provided candidate lists -----------------------------------
__global__ __launch_bounds__(256) void seg_fill_kernel(uint8_t* __restrict__ cls_at, int n) {
  // n bytes, padded to a multiple of 16 by the workspace layout
  uint4* m = reinterpret_cast<uint4*>(cls_at);
  const int n16 = (n + 15) / 16;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += gridDim.x * blockDim.x)
    m[i] = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
}

__global__ __launch_bounds__(256) void seg_scatter_kernel(
    const int32_t* __restrict__ cand_pos, const uint8_t* __restrict__ cand_class,
    const int32_t* __restrict__ cand_cu, const int32_t* __restrict__ cu_seqlens, int B, int n_class,
    int max_cand, uint8_t* __restrict__ cls_at, int32_t* dev_status) {
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
    cls_at[t] = (uint8_t)cls;
  }
}

// ---- tile kernel -----------------------------------------------------------------------------
// dynamic LDS layout (bytes):
//   best  u64 [kSegTile]                      votes; dead after the successor table is built,
//   pos/cb/cs u16 [2][kSegTile] each          ... so the pointer-jumping arrays overlay it
//   nxt   u16 [kSegTile]   successor - position
//   ns    u16 [kSegTile]   slots of the chunk starting here
//   mark  u8  [kSegTile]   (emit mode) reachable from the tile's entry
//   wq    u8  [64]         class -> weight tenths of this sequence
//   red   i32 [2*kSegWaves + 2]
__host__ __device__ constexpr size_t seg_tile_lds_bytes() {
  return (size_t)kSegTile * 12      // jump arrays (the vote array, 8 bytes per position, overlays them)
         + (size_t)kSegTile * 4     // nxt, ns
         + (size_t)kSegTile         // mark
         + 64 + 64;                 // wq, red
}
static_assert((2 * kSegWaves + 2) * 4 <= 64, "red fits its slot");

template <int MODE>
__global__ __launch_bounds__(kSegThreads) void seg_tile_kernel(
    SegParams p, const uint8_t* __restrict__ cls_at, uint2* __restrict__ tile_map,
    const int4* __restrict__ tile_info, const int4* __restrict__ seq_info, int32_t* __restrict__ block_start,
    int32_t* __restrict__ slot_base, int32_t* dev_status) {
  extern __shared__ __align__(16) unsigned char smem[];
  // jump arrays (12 * kSegTile bytes) share storage with the vote array (8 * kSegTile bytes)
  unsigned long long* best = reinterpret_cast<unsigned long long*>(smem);
  uint16_t* jpos = reinterpret_cast<uint16_t*>(smem);            // [2][kSegTile] position - p0, or exit
  uint16_t* jcb = jpos + 2 * kSegTile;                            // [2][kSegTile] blocks laid down
  uint16_t* jcs = jcb + 2 * kSegTile;                             // [2][kSegTile] slots laid down
  uint16_t* nxt = jcs + 2 * kSegTile;
  uint16_t* ns = nxt + kSegTile;
  uint8_t* mark = reinterpret_cast<uint8_t*>(ns + kSegTile);
  uint8_t* wq = mark + kSegTile;
  int* red = reinterpret_cast<int*>(wq + 64);

  const int s = blockIdx.y;
  const int j = blockIdx.x;
  const int tid = threadIdx.x;
  const int seq0 = p.cu_seqlens[s];
  const int L = p.cu_seqlens[s + 1] - seq0;
  if (!seq_ok(p, seq0, L)) {
    if (tid == 0) set_status(dev_status, DSK_ERR_SHAPE);
    return;
  }
  const int p0 = j * kSegTile;
  if (p0 >= L) return;
  const int p1 = (p0 + kSegTile < L) ? p0 + kSegTile : L;
  const int tlen = p1 - p0;
  const int tile = s * p.tiles_per_seq + j;
  int4 info = make_int4(0, 0, 0, 0), sq = make_int4(0, 0, 0, 0);
  if (MODE == 1) {   // issued early; needed only for the output
    info = tile_info[tile];
    sq = seq_info[s];
  }
  int C, delta;
  seq_params(p, s, C, delta, dev_status);
  const int dd = delta > 1 ? delta : 1;

  if (tid < 64) {
    int w = tid < p.n_class ? p.class_weight_q[s * p.n_class + tid] : 0;
    if (w > 10) { set_status(dev_status, DSK_ERR_PARAM); w = 10; }
    wq[tid] = (uint8_t)w;
  }
  for (int i = tid; i < kSegTile; i += kSegThreads) { best[i] = 0ull; mark[i] = 0; }
  __syncthreads();

  // votes: boundary e (offered by a delimiter at e-1) can end a chunk that starts at q with
  // s_e = q + C in [e - delta, e + delta] and s_e < L.  key = score << 16 | (0xFFFF - (e - q)):
  // highest score wins, then the smallest e; 0 = no vote.
  {
    const int e_lo = p0 + C - delta > 1 ? p0 + C - delta : 1;
    int e_hi = p1 - 1 + C + delta;
    if (e_hi > L) e_hi = L;
    for (int e = e_lo + tid; e <= e_hi; e += kSegThreads) {
      const int cls = cls_at[seq0 + e - 1];
      if (cls == 255) continue;
      const int w = cls < 64 ? wq[cls] : 0;
      int q_lo = e - C - delta, q_hi = e - C + delta;
      if (q_lo < p0) q_lo = p0;
      if (q_hi > p1 - 1) q_hi = p1 - 1;
      if (q_hi > L - C - 1) q_hi = L - C - 1;      // s_e = q + C must stay below L
      for (int q = q_lo; q <= q_hi; ++q) {
        const int s_e = q + C;
        const int dist = e > s_e ? e - s_e : s_e - e;
        const unsigned long long sc = (unsigned long long)(p.a_num * w * dd + (p.a_den - p.a_num) * 10 * (dd - dist));
        const unsigned long long key = ((sc + 1ull) << 16) | (unsigned long long)(0xFFFF - (e - q));
        atomicMax(&best[q - p0], key);
      }
    }
  }
  __syncthreads();
  // successor table (registers first: `best` is about to be overlaid)
  int my_len[kSegPerThread];
#pragma unroll
  for (int r = 0; r < kSegPerThread; ++r) {
    const int i = tid * kSegPerThread + r;
    const int q = p0 + i;
    int len = 0;
    if (i < tlen) {
      const int s_e = q + C;
      if (s_e >= L) len = L - q;
      else {
        const unsigned long long key = best[i];
        len = key ? 0xFFFF - (int)(key & 0xFFFFull) : C;
      }
    }
    my_len[r] = len;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kSegPerThread; ++r) {
    const int i = tid * kSegPerThread + r;
    const int len = my_len[r];
    const int nslot = (len + p.b - 1) / p.b;
    nxt[i] = (uint16_t)len;
    ns[i] = (uint16_t)nslot;
    // level-0 jump: one chunk
    jpos[i] = (uint16_t)(i + len);          // >= tlen means "left the tile" (i + len <= tlen + C + delta)
    jcb[i] = (uint16_t)(i < tlen ? 1 : 0);
    jcs[i] = (uint16_t)nslot;
  }
  if (MODE == 1 && tid == 0 && info.x >= p0 && info.x < p1) mark[info.x - p0] = 1;
  __syncthreads();

  // pointer jumping: level r holds 2^r chunks per hop; positions that left the tile are fixed points
  int cur = 0;
  for (int round = 0; round < 16; ++round) {
    int active = 0;
    uint16_t* ps = jpos + cur * kSegTile; uint16_t* pd = jpos + (cur ^ 1) * kSegTile;
    uint16_t* bs_ = jcb + cur * kSegTile; uint16_t* bd = jcb + (cur ^ 1) * kSegTile;
    uint16_t* ss = jcs + cur * kSegTile;  uint16_t* sd = jcs + (cur ^ 1) * kSegTile;
#pragma unroll
    for (int r = 0; r < kSegPerThread; ++r) {
      const int i = tid * kSegPerThread + r;
      const int t = ps[i];
      int np = t, nb = bs_[i], nsl = ss[i];
      if (i < tlen && t < tlen) {
        if (MODE == 1 && mark[i]) mark[t] = 1;   // reachable set doubles with the hop length
        np = ps[t];
        nb += bs_[t];
        nsl += ss[t];
        active = 1;
      }
      pd[i] = (uint16_t)np; bd[i] = (uint16_t)nb; sd[i] = (uint16_t)nsl;
    }
    cur ^= 1;
    if (!__syncthreads_or(active)) break;
  }
  const uint16_t* fpos = jpos + cur * kSegTile;
  const uint16_t* fcb = jcb + cur * kSegTile;
  const uint16_t* fcs = jcs + cur * kSegTile;

  if (MODE == 0) {
    uint2* row = tile_map + (int64_t)tile * p.map_row;
    for (int ent = tid; ent < p.map_row; ent += kSegThreads) {
      uint2 rv = make_uint2(0u, 0u);
      if (ent < tlen) rv = make_uint2((uint32_t)(fpos[ent] - tlen) | ((uint32_t)fcb[ent] << 16), (uint32_t)fcs[ent]);
      row[ent] = rv;
    }
    return;
  }

  // emit: rank the marked positions of the tile (thread order = position order)
  int nb_local = 0, ns_local = 0;
#pragma unroll
  for (int r = 0; r < kSegPerThread; ++r) {
    const int i = tid * kSegPerThread + r;
    if (i < tlen && mark[i]) { ++nb_local; ns_local += ns[i]; }
  }
  const int lane = tid & (DSK_WAVE - 1), wave = tid / DSK_WAVE;
  const int ib = wave_incl_scan_i(nb_local, lane);
  const int is = wave_incl_scan_i(ns_local, lane);
  if (lane == DSK_WAVE - 1) { red[2 * wave] = ib; red[2 * wave + 1] = is; }
  __syncthreads();
  int ob = 0, os = 0;
#pragma unroll
  for (int w = 0; w < kSegWaves; ++w)
    if (w < wave) { ob += red[2 * w]; os += red[2 * w + 1]; }
  int gb = sq.z + info.y + ob + ib - nb_local;
  int gs = sq.w + info.z + os + is - ns_local;
#pragma unroll
  for (int r = 0; r < kSegPerThread; ++r) {
    const int i = tid * kSegPerThread + r;
    if (i < tlen && mark[i]) {
      if (gb < p.cap) {
        block_start[gb] = seq0 + p0 + i;
        slot_base[gb] = gs;
      }
      ++gb;
      gs += ns[i];
    }
  }
  (void)fpos; (void)fcb; (void)fcs;
}

// ---- chain ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kSegThreads) void seg_chain_kernel(
    SegParams p, const uint2* __restrict__ tile_map, int4* __restrict__ tile_info,
    int4* __restrict__ seq_info, int32_t* __restrict__ cu_blocks, int32_t* __restrict__ block_start,
    int32_t* __restrict__ slot_base, int32_t* dev_status) {
  __shared__ uint2 rows[kChainLdsEntries];
  __shared__ int carry[3];
  const int s = blockIdx.x;
  int L = p.cu_seqlens[s + 1] - p.cu_seqlens[s];
  if (!seq_ok(p, p.cu_seqlens[s], L)) L = 0;   // flagged by the tile kernel; emit nothing
  int n_tiles = (L + kSegTile - 1) / kSegTile;
  if (n_tiles > p.tiles_per_seq) n_tiles = p.tiles_per_seq;
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
  if (threadIdx.x == 0) {
    seq_info[s] = make_int4(carry[1], carry[2], 0, 0);
    if (p.B == 1) {   // single sequence: the batch scan is trivial, finish here
      cu_blocks[0] = 0;
      cu_blocks[1] = carry[1];
      if (carry[1] > p.cap) set_status(dev_status, DSK_ERR_CAPACITY);
      else { block_start[carry[1]] = p.total_tokens; slot_base[carry[1]] = carry[2]; }
    }
  }
}

// ---- scan over the sequences of the batch (B > 1) ----------------------------------------------
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
    return;   // the tables stay self-consistent for the truncated prefix
  }
  block_start[blk] = total_tokens;
  slot_base[blk] = slots;
}

// ---- host -----------------------------------------------------------------------------------
hipError_t launch_segment(const dsk_compress_args& a, const CompressWs& ws, bool have_cls_at, hipStream_t st) {
  unsigned char* w = static_cast<unsigned char*>(a.workspace);
  uint8_t* cls_at = w + ws.cls_at;
  uint2* tile_map = reinterpret_cast<uint2*>(w + ws.tile_map);
  int4* tile_info = reinterpret_cast<int4*>(w + ws.tile_info);
  int4* seq_info = reinterpret_cast<int4*>(w + ws.seq_info);

  SegParams p;
  p.cu_seqlens = a.cu_seqlens;
  p.C_per_seq = a.C_per_seq;
  p.delta_per_seq = a.delta_per_seq;
  p.class_weight_q = a.class_weight_q;
  p.n_class = a.n_class;
  p.C = a.C; p.delta = a.delta; p.a_num = a.alpha_num; p.a_den = a.alpha_den; p.b = a.b;
  p.map_row = ws.map_row; p.tiles_per_seq = ws.tiles_per_seq;
  p.max_seqlen = a.max_seqlen; p.total_tokens = a.total_tokens;
  p.B = a.B; p.cap = a.max_blocks_total;

  hipError_t err;
  if (!have_cls_at) {   // candidates came from the caller: scatter them into the dense class array
    const int n = a.total_tokens;
    int n16 = (n + 15) / 16;
    int wgs = (n16 + 255) / 256;
    if (wgs > 1024) wgs = 1024;
    if (wgs > 0) {
      seg_fill_kernel<<<dim3(wgs), dim3(256), 0, st>>>(cls_at, n);
      if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (a.max_cand_total > 0) {
      wgs = (a.max_cand_total + 255) / 256;
      if (wgs > 1024) wgs = 1024;
      seg_scatter_kernel<<<dim3(wgs), dim3(256), 0, st>>>(a.cand_pos, a.cand_class, a.cand_cu, a.cu_seqlens,
                                                           a.B, a.n_class, a.max_cand_total, cls_at, a.dev_status);
      if ((err = hipGetLastError()) != hipSuccess) return err;
    }
  }
  const size_t lds = seg_tile_lds_bytes();
  if (ws.tiles_per_seq > 0) {
    const dim3 grid((unsigned)ws.tiles_per_seq, (unsigned)a.B);
    seg_tile_kernel<0><<<grid, dim3(kSegThreads), lds, st>>>(p, cls_at, tile_map, tile_info, seq_info,
                                                             a.block_start, a.slot_base, a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  seg_chain_kernel<<<dim3((unsigned)a.B), dim3(kSegThreads), 0, st>>>(p, tile_map, tile_info, seq_info, a.cu_blocks,
                                                                      a.block_start, a.slot_base, a.dev_status);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (a.B > 1) {
    seg_seqscan_kernel<<<dim3(1), dim3(64), 0, st>>>(seq_info, a.B, a.max_blocks_total, a.total_tokens,
                                                     a.cu_blocks, a.block_start, a.slot_base, a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (ws.tiles_per_seq > 0) {
    const dim3 grid((unsigned)ws.tiles_per_seq, (unsigned)a.B);
    seg_tile_kernel<1><<<grid, dim3(kSegThreads), lds, st>>>(p, cls_at, tile_map, tile_info, seq_info,
                                                             a.block_start, a.slot_base, a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  return hipSuccess;
}

}  // namespace dsk
