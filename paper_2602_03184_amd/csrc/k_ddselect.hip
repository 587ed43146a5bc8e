// DD-Select segmentation (Sec. 4.1, Dynamic Segmentation Procedure) and the variable-to-
// fixed slot map (Sec. 4.2), integer-exact.
//
// The procedure is a chain s_c -> e*(s_c) whose successor depends only on s_c and static
// data, and it only moves forward by at most C + delta.  It is parallelised by cutting every
// sequence into tiles of kSegTile positions.  The delimiter class of a token comes from a dense
// per-token class byte (255 = not a delimiter) -- written by the candidate stage, or scattered from
// the caller's candidate lists -- or, when the candidate stage runs in the same call and nothing
// waits for its lists, from token_ids / delim_ids inside the first tile pass, which then also counts
// the candidates so that the later passes can write the lists on their way.
//   tile<0>: successor of every position of the tile.  Instead of scanning the 2*delta+1
//            boundaries of every position's search range, every delimiter in reach "votes" its
//            packed (score, smaller-e-wins) key into the 2*delta+1 start positions whose range
//            contains it (64-bit LDS atomic max): work is proportional to delimiters, not
//            positions.  Then pointer jumping (successor of successor, log2 rounds) gives, for
//            every position at once, where the chain leaves the tile and how many blocks / slots
//            it lays down on the way; the first C+delta of these form the tile's entry map.  The
//            chunk length and the hop-2, -4, -8 .. targets of every position are kept for the emit pass.
//   chain:   per sequence, hop through the entry maps (staged in LDS) to fix each tile's real
//            entry and its block / slot offsets; for a single-sequence batch also the totals.
//   scan:    block and slot bases of the sequences of a batch (B > 1), capacity check.
//   tile<1>: the chunks the chain lays down in the tile are the positions 0, 1, 2 .. hops behind the
//            tile's real entry; each is found through the hop-2^l tables the first pass kept, ranked
//            by a workgroup scan and written out.
//   tile<2>: tile<1> for a single sequence of few tiles, which also chains the tiles in front of
//            its own by itself: no chain launch.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kTileThreads = 1024;                      // workgroup of the tile kernel: the tiles are few (one per
                                                        // 2048 positions) and their phases barrier-bound, so
                                                        // wide workgroups shorten them (256 / 512 / 1024
                                                        // threads: 95 / 88 / 86.5 us for the pass at 128K)
constexpr int kSegPerThread = kSegTile / kTileThreads;  // positions owned by a thread of the tile kernel
constexpr int kTileWaves = kTileThreads / DSK_WAVE;
constexpr int kChainLdsEntries = 6144;   // uint2 entries staged per chunk in the chain kernel (48 KB)

struct SegParams {
  const int32_t* cu_seqlens;
  const int32_t* C_per_seq;
  const int32_t* delta_per_seq;
  const uint8_t* class_weight_q;   // [B, n_class]
  int n_class;
  int C, delta, a_num, a_den, b;
  uint32_t b_inv;          // floor(2^32 / b) + 1 for 1 < b < 2^15, else 0: division by b as a multiply
  int map_row, tiles_per_seq;
  int max_seqlen, total_tokens;
  int B, cap;
  uint16_t* seg_jump;      // [max_levels][jump_stride] per token: position in its tile 2^(level+1) chunks on
  int max_levels;          // levels the buffer holds: one less than the doubling rounds of any sequence
  int jump_stride;
};

constexpr int kMaxJumpLevels = 10;   // kept levels: hops of 2 .. 2^10 chunks; with the chunk itself, 2^11 >= kSegTile
static_assert((1 << (kMaxJumpLevels + 1)) >= kSegTile, "levels cover a tile of one-position chunks");
__host__ __device__ inline int jump_rounds(int tlen, int min_len) {
  const int hops = (tlen + min_len - 1) / min_len;
  int rounds = 0;
  while ((1 << rounds) < hops) ++rounds;
  return rounds;
}

// Candidate lists produced by the segmentation kernels themselves (stage CANDIDATES and stage
// SEGMENT in one call, weights from a table): the first tile pass classifies and counts the
// positions of its tile, the chain kernel turns the counts into list offsets, the emit pass
// writes the lists.  tile_count == nullptr: no lists are produced here.
struct SegCand {
  uint8_t* own_cls;        // [total_tokens] class byte of every token (workspace)
  int32_t* tile_count;     // [B * tiles_per_seq] candidates of a tile (workspace)
  int32_t* tile_base;      // [B * tiles_per_seq] candidates of the sequence in front of a tile (workspace)
  int32_t* cand_cu;        // [B + 1] output
  int32_t* cand_pos;       // [max_cand] output
  uint8_t* cand_class;     // [max_cand] output
  int max_cand;
};

// first token and length of sequence s.  A batch of one sequence is [0, total_tokens) by the
// host's copy of cu_seqlens, which saves every kernel of the chain a dependent memory round trip.
__device__ __forceinline__ void seq_range(const SegParams& p, int s, int& seq0, int& L) {
  if (p.B == 1) { seq0 = 0; L = p.total_tokens; return; }
  seq0 = p.cu_seqlens[s];
  L = p.cu_seqlens[s + 1] - seq0;
}

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
    // the lists are ascending within a sequence by contract; the dense class bytes do not depend
    // on the order, so the segmentation still runs, but the caller is told
    if (j > cand_cu[s] && cand_pos[j - 1] >= t) set_status(dev_status, DSK_ERR_ORDER);
    cls_at[t] = (uint8_t)cls;
  }
}

// ---- chain: shared by the chain kernel and the emit pass that does its own chaining -----------------
// Entry maps are functions (entry offset into a tile) -> (entry offset into the next tile, chunks
// and slots laid down on the way), so the walk from tile to tile is a prefix "sum" under function
// composition and runs as a doubling scan: after round r, row j holds the composite of tiles
// j - 2^r + 1 .. j.  Rows are staged in LDS, kChainLdsEntries / 2 entries per buffer; longer
// sequences are cut into runs of tiles that pass a carry.  An LDS entry packs (offset: 16 bits,
// chunks: 24 bits, slots: 24 bits): a run is at most kChainLdsEntries / 2 tiles, each with at most
// 2048 chunks or slots.  Search ranges wider than kChainFastSpan take the plain walk, one lookup
// per tile.
constexpr int kChainThreads = 1024;
constexpr int kChainFastSpan = 512;                      // C + delta up to here: >= 6 tiles per run
static_assert((kChainLdsEntries / 2) * kSegTile < (1 << 24), "packed counts of a run");

__device__ __forceinline__ int chain_off(uint2 v) { return (int)(v.x & 0xFFFFu); }
__device__ __forceinline__ int chain_blocks(uint2 v) { return (int)((v.x >> 16) | ((v.y >> 24) << 16)); }
__device__ __forceinline__ int chain_slots(uint2 v) { return (int)(v.y & 0xFFFFFFu); }
__device__ __forceinline__ uint2 chain_pack(int off, int blocks, int slots) {
  return make_uint2((uint32_t)off | ((uint32_t)(blocks & 0xFFFF) << 16),
                    (uint32_t)slots | ((uint32_t)(blocks >> 16) << 24));
}


// The doubling scan over the entry maps of tiles j0 .. j0 + T - 1 of a sequence of L positions, in
// two steps so that a caller can have the loads in flight with its other loads: chain_load fetches
// the rows (registers), chain_scan stages them in `cur` and runs the rounds; on return row j of the
// returned buffer maps an entry offset of tile j0 to the state behind tile j0 + j.
// T * map_row <= kChainLdsEntries / 2, map_row <= kChainFastSpan; all kChainThreads threads call both.
constexpr int kChainPer = (kChainLdsEntries / 2 + kChainThreads - 1) / kChainThreads;
struct ChainRows {
  uint2 ld[kChainPer];
  int jj[kChainPer], ee[kChainPer];                   // tile of the run and entry offset of element i
};

__device__ __forceinline__ void chain_load(ChainRows& r, const uint2* __restrict__ src, int T, int map_row) {
  // i / map_row without a division: inv = floor(2^32 / map_row) + 1 is exact for i * map_row < 2^32
  const uint32_t inv = 0xFFFFFFFFu / (uint32_t)map_row + 1u;
  const int n_ent = T * map_row;
#pragma unroll
  for (int u = 0; u < kChainPer; ++u) {               // the run's rows: one round trip, not kChainPer
    const int i = threadIdx.x + u * kChainThreads;
    r.ld[u] = src[i < n_ent ? i : 0];
    r.jj[u] = map_row == 1 ? i : (int)__umulhi((uint32_t)i, inv);   // inv wraps to 0 for a divisor of 1
    r.ee[u] = i - r.jj[u] * map_row;
  }
}

__device__ __forceinline__ uint2* chain_scan(const ChainRows& r, int L, int j0, int T, int map_row, uint2* cur,
                                             uint2* nxt) {
  const int n_ent = T * map_row;
#pragma unroll
  for (int u = 0; u < kChainPer; ++u) {
    const int i = threadIdx.x + u * kChainThreads;
    if (i < n_ent) {
      const int t0 = (j0 + r.jj[u]) * kSegTile;
      const int tl = (t0 + kSegTile < L) ? kSegTile : L - t0;
      cur[i] = r.ee[u] >= tl ? chain_pack(r.ee[u] - tl, 0, 0) : r.ld[u];   // beyond a short last tile: passes through
    }
  }
  __syncthreads();
  for (int d = 1; d < T; d <<= 1) {
#pragma unroll
    for (int u = 0; u < kChainPer; ++u) {
      const int i = threadIdx.x + u * kChainThreads;
      if (i < n_ent) {
        const int j = r.jj[u], e = r.ee[u];
        uint2 v = cur[i];
        if (j >= d) {                                 // tiles j-2d+1 .. j-d first, then j-d+1 .. j
          const uint2 a = cur[(j - d) * map_row + e];
          const uint2 c = cur[j * map_row + chain_off(a)];
          v = chain_pack(chain_off(c), chain_blocks(a) + chain_blocks(c), chain_slots(a) + chain_slots(c));
        }
        nxt[i] = v;
      }
    }
    __syncthreads();
    uint2* t = cur; cur = nxt; nxt = t;
  }
  return cur;
}

// State of the chain in front of tile `upto` (0 < upto <= T) when it enters tile 0 at offset 0, for a
// workgroup that needs this one prefix only: instead of the doubling scan over every row, the rows
// are combined four at a time into a tree (level k row r = tiles [r 4^k, (r+1) 4^k)), and every
// thread then walks the tree from the top, at most three steps per level.  About 4 log4(T) + 3
// log4(T) dependent LDS reads in all, against 2 log2(T) rounds over all entries.  lvl0 holds the
// staged rows of tiles 0 .. T-1 (T * map_row entries), `upper` has room for T * map_row / 3 + map_row more.
__device__ __forceinline__ void chain_prefix_tree(const ChainRows& r, int L, int T, int map_row, int upto,
                                                  uint2* lvl0, uint2* upper, int& e_out, int& blk_out, int& sl_out) {
  const int n_ent = T * map_row;
#pragma unroll
  for (int u = 0; u < kChainPer; ++u) {
    const int i = threadIdx.x + u * kChainThreads;
    if (i < n_ent) {
      const int t0 = r.jj[u] * kSegTile;
      const int tl = (t0 + kSegTile < L) ? kSegTile : L - t0;
      lvl0[i] = r.ee[u] >= tl ? chain_pack(r.ee[u] - tl, 0, 0) : r.ld[u];   // beyond a short last tile: passes through
    }
  }
  __syncthreads();
  // build the levels that a walk to `upto` can use: level k exists while 4^k <= upto; level k >= 1
  // has T >> 2k rows (full groups of four only: a walk never uses a ragged one), stored one after
  // the other in `upper`
  int n_lvl = 1;
  uint2* dst = upper;
  {
    const uint2* src = lvl0;
    const uint32_t inv = 0xFFFFFFFFu / (uint32_t)map_row + 1u;
    for (int span = 4; span <= upto; span <<= 2) {
      const int rows_dst = T >> (2 * n_lvl);
      for (int idx = threadIdx.x; idx < rows_dst * map_row; idx += kChainThreads) {
        const int row = map_row == 1 ? idx : (int)__umulhi((uint32_t)idx, inv);
        int off = idx - row * map_row, blk = 0, sl = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const uint2 v = src[(4 * row + c) * map_row + off];
          off = chain_off(v); blk += chain_blocks(v); sl += chain_slots(v);
        }
        dst[idx] = chain_pack(off, blk, sl);
      }
      __syncthreads();
      src = dst;
      dst += rows_dst * map_row;
      ++n_lvl;
    }
  }
  int pos = 0, off = 0, blk = 0, sl = 0;
  const uint2* lp = dst;                                   // end of the highest level
  for (int k = n_lvl - 1; k >= 0; --k) {
    lp = k > 0 ? lp - (T >> (2 * k)) * map_row : lvl0;
    const int span = 1 << (2 * k);
    while (pos + span <= upto) {
      const uint2 v = lp[(pos >> (2 * k)) * map_row + off];
      off = chain_off(v); blk += chain_blocks(v); sl += chain_slots(v);
      pos += span;
    }
  }
  e_out = off; blk_out = blk; sl_out = sl;
}

// class index of N token ids against the delimiter ids staged in LDS (padded to a multiple of 4
// entries); the lowest class index wins, as in the candidate stage; 255 = not a delimiter
template <int N>
__device__ __forceinline__ void classify_tokens(const int (&tok)[N], int (&cls)[N], const int32_t* ids, int n_class) {
#pragma unroll
  for (int r = 0; r < N; ++r) cls[r] = 255;
  for (int c4 = (n_class - 1) / 4 * 4; c4 >= 0; c4 -= 4) {
    const int4 id4 = *reinterpret_cast<const int4*>(ids + c4);      // LDS broadcast read
    const int idv[4] = {id4.x, id4.y, id4.z, id4.w};
#pragma unroll
    for (int cc = 3; cc >= 0; --cc) {
      const int c = c4 + cc;
      if (c < n_class) {
#pragma unroll
        for (int r = 0; r < N; ++r) cls[r] = tok[r] == idv[cc] ? c : cls[r];
      }
    }
  }
}

// ---- tile kernel -----------------------------------------------------------------------------
// dynamic LDS layout (bytes):
//   best  u64 [kSegTile]       votes; dead after the successor table is built,
//   jmp   uint2 [2][kSegTile]  ... so the pointer-jumping entries overlay it:
//                              x = (position - p0, or exit offset) | chunks << 16, y = slots
//   clist u16 [2 * kSegTile]   delimiters in reach (overlays the second jump buffer)
//   ns    u16 [kSegTile]       slots of the chunk starting here
//   wq    u8  [64]             class -> weight tenths of this sequence
//   red   i32 [40], then the delimiter ids i32 [64]
constexpr size_t kTileJumpBytes =    // jump entries; the vote array (8 bytes per position) and, in the emit pass
    (size_t)kSegTile * 16 > (size_t)kChainLdsEntries * 8 ? (size_t)kSegTile * 16     // that chains for itself, the two
                                                        : (size_t)kChainLdsEntries * 8;   // buffers of the chain scan overlay them
__host__ __device__ constexpr size_t seg_tile_lds_bytes() {
  return kTileJumpBytes
         + (size_t)kSegTile * 2     // ns
         + 64 + 448;                // wq, red (reduction words, then 64 delimiter ids)
}
static_assert(2 * kTileWaves + 3 <= 40 && (40 + 64) * 4 <= 448, "red fits its slot");
static_assert(kChainThreads == kTileThreads, "the emit pass runs the chain scan with its own workgroup");

// MODE 0 (entry maps): the successor of every position comes from the votes of the delimiters in
// reach -- read as class bytes (cls_at), or, when cls_at is NULL, classified here from token_ids /
// delim_ids -- and the chunk lengths found are kept in seg_len for MODE 1 (emit), which starts from
// them and casts no vote.  MODE 2 is the emit pass of a single sequence whose entry maps fit one run of
// the chain scan: every workgroup chains the tiles in front of its own by itself, so the chain
// kernel is not launched; the workgroup of the last tile also writes the totals.
template <int MODE>
__global__ __launch_bounds__(kTileThreads) void seg_tile_kernel(
    SegParams p, SegCand cand, const uint8_t* __restrict__ cls_at, const int32_t* __restrict__ token_ids,
    const int32_t* __restrict__ delim_ids, uint16_t* __restrict__ seg_len, uint2* __restrict__ tile_map,
    const int4* __restrict__ tile_info, const int4* __restrict__ seq_info, int32_t* __restrict__ cu_blocks,
    int32_t* __restrict__ cu_slots, int32_t* __restrict__ block_start, int32_t* __restrict__ slot_base,
    int32_t* dev_status) {
  extern __shared__ __align__(16) unsigned char smem[];
  // jump entries (16 * kSegTile bytes) share storage with the vote array (8 * kSegTile bytes)
  unsigned long long* best = reinterpret_cast<unsigned long long*>(smem);
  uint2* jmp = reinterpret_cast<uint2*>(smem);                    // [2][kSegTile]
  uint16_t* ns = reinterpret_cast<uint16_t*>(smem + kTileJumpBytes); // [kSegTile] slots of the chunk starting here
  uint8_t* wq = reinterpret_cast<uint8_t*>(ns + kSegTile);
  int* red = reinterpret_cast<int*>(wq + 64);

  const int s = blockIdx.y;
  const int j = blockIdx.x;
  const int tid = threadIdx.x;
  int seq0, L;
  seq_range(p, s, seq0, L);
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
  // MODE 2: one sequence, so its block and slot bases (sq) are zero, and info comes from the scan
  // below, whose rows (the entry maps of the tiles in front, and of this one in the last tile) are
  // requested here, with everything else the kernel reads first
  ChainRows cr;
  const int chain_T = MODE == 2 ? (p0 + kSegTile >= L ? j + 1 : j) : 0;
  if (MODE == 2 && chain_T > 0) chain_load(cr, tile_map + (int64_t)s * p.tiles_per_seq * p.map_row, chain_T, p.map_row);
  int C, delta;
  seq_params(p, s, C, delta, dev_status);
  const int dd = delta > 1 ? delta : 1;

  int my_len[kSegPerThread];
  int oc1[kSegPerThread];            // (emit, candidate lists) class bytes of the tile's positions
  int cand_o = 0;                    // list offset of the tile's first candidate
  if (MODE != 0 && cand.tile_count != nullptr) {
#pragma unroll
    for (int r = 0; r < kSegPerThread; ++r) {
      const int i = r * kTileThreads + tid;
      oc1[r] = cand.own_cls[seq0 + p0 + (i < tlen ? i : 0)];
    }
    if (MODE == 1) cand_o = cand.tile_base[tile] + (p.B == 1 ? 0 : cand.cand_cu[s]);
    else cand_o = tid < j ? cand.tile_count[tile - j + tid] : 0;     // summed below; j < kTileThreads
  }
  // (emit) where the chain is 2, 4, 8 .. chunks after each of the thread's positions, as the first
  // pass left it; every level the buffer holds is requested (the count in use depends on the
  // sequence's C and delta, which may still be on their way)
  uint16_t lv[kMaxJumpLevels][kSegPerThread];
  if (MODE != 0) {
#pragma unroll
    for (int l = 0; l < kMaxJumpLevels; ++l) {
#pragma unroll
      for (int r = 0; r < kSegPerThread; ++r) {
        const int i = r * kTileThreads + tid;
        lv[l][r] = l < p.max_levels ? p.seg_jump[(int64_t)l * p.jump_stride + seq0 + p0 + (i < tlen ? i : 0)] : (uint16_t)0xFFFF;
      }
    }
  }
  if (MODE == 0) {
    // the class bytes (or token ids) of the first kVoteChunk boundaries in reach go out before
    // anything is waited for: they travel with the weight and delimiter-id loads below
    constexpr int kVoteChunk = 2 * kSegTile;                                        // 4 positions per thread
    constexpr int kPerThread = kVoteChunk / kTileThreads;
    const int e_lo = p0 + C - delta > 1 ? p0 + C - delta : 1;
    int e_hi = p1 - 1 + C + delta;
    if (e_hi > L) e_hi = L;
    int first[kPerThread];
#pragma unroll
    for (int r = 0; r < kPerThread; ++r) {
      int e = e_lo + r * kTileThreads + tid;
      e = e <= e_hi ? e : e_hi;
      e = e >= 1 ? e : 1;                              // e_hi >= 1 whenever the tile has a position
      first[r] = cls_at != nullptr ? (int)cls_at[seq0 + e - 1] : token_ids[seq0 + e - 1];
    }
    // candidate lists from this pass: the tile's own positions are classified as well (the
    // boundaries above start C - delta positions further on)
    const bool own = cand.tile_count != nullptr;
    int own_tok[kSegPerThread];
    if (own) {
#pragma unroll
      for (int r = 0; r < kSegPerThread; ++r) {
        const int i = r * kTileThreads + tid;
        own_tok[r] = token_ids[seq0 + p0 + (i < tlen ? i : 0)];
      }
    }
    if (tid < 64) {
      int w = tid < p.n_class ? p.class_weight_q[s * p.n_class + tid] : 0;
      if (w > 10) { set_status(dev_status, DSK_ERR_PARAM); w = 10; }
      wq[tid] = (uint8_t)w;
    }
    for (int i = tid; i < kSegTile; i += kTileThreads) best[i] = 0ull;
    int* n_list = red;
    if (tid == 0) *n_list = 0;
    // delimiter ids for the in-kernel classification; the entries past n_class repeat id 0 and are
    // never compared
    int32_t* ids = red + 40;                                          // 64 ints behind the reduction words
    if (cls_at == nullptr && tid < 64) ids[tid] = delim_ids[tid < p.n_class ? tid : 0];
    __syncthreads();

    if (own) {
      int oc[kSegPerThread];
      classify_tokens<kSegPerThread>(own_tok, oc, ids, p.n_class);
      int n_wave = 0;
#pragma unroll
      for (int r = 0; r < kSegPerThread; ++r) {
        const int i = r * kTileThreads + tid;
        if (i < tlen) cand.own_cls[seq0 + p0 + i] = (uint8_t)oc[r];
        n_wave += __popcll(__ballot(i < tlen && oc[r] != 255));
      }
      if ((tid & (DSK_WAVE - 1)) == 0) red[4 + tid / DSK_WAVE] = n_wave;   // summed once the barriers below have passed
    }

    // votes: boundary e (offered by a delimiter at e-1) can end a chunk that starts at q with
    // s_e = q + C in [e - delta, e + delta] and s_e < L.  key = score << 16 | (0xFFFF - (e - q)):
    // highest score wins, then the smallest e; 0 = no vote.  The boundaries in reach are scanned
    // kVoteChunk at a time (normally once); the delimiters found are first compacted into an LDS
    // list (one reservation per wavefront, ballots inside it) so that the vote loops run on threads
    // that all have one (a dense scan would leave 1 lane in 30 busy).
    {
      uint16_t* clist = reinterpret_cast<uint16_t*>(smem + (size_t)kSegTile * 8);     // free until the jump arrays are built
      const int lane = tid & (DSK_WAVE - 1);
      for (int e0 = e_lo; e0 <= e_hi; e0 += kVoteChunk) {
        int cb_[kPerThread];
        if (cls_at != nullptr) {
#pragma unroll
          for (int r = 0; r < kPerThread; ++r) {       // independent byte loads: one round trip
            int e = e0 + r * kTileThreads + tid;
            e = e <= e_hi ? e : e_hi;
            cb_[r] = e0 == e_lo ? first[r] : (int)cls_at[seq0 + e - 1];
          }
        } else {
          int tok[kPerThread];
#pragma unroll
          for (int r = 0; r < kPerThread; ++r) {
            int e = e0 + r * kTileThreads + tid;
            e = e <= e_hi ? e : e_hi;
            tok[r] = e0 == e_lo ? first[r] : token_ids[seq0 + e - 1];
          }
          classify_tokens<kPerThread>(tok, cb_, ids, p.n_class);
        }
        // compaction: position of each delimiter inside its wavefront from ballots, one LDS
        // reservation per wavefront
        unsigned long long bal[kPerThread];
        int n_wave = 0;
#pragma unroll
        for (int r = 0; r < kPerThread; ++r) {
          const int eo = r * kTileThreads + tid;
          bal[r] = __ballot(e0 + eo <= e_hi && cb_[r] != 255);
          n_wave += __popcll(bal[r]);
        }
        int base = 0;
        if (lane == 0 && n_wave > 0) base = atomicAdd(n_list, n_wave);
        base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
        for (int r = 0; r < kPerThread; ++r) {
          const int eo = r * kTileThreads + tid;        // e - e0 < 4096: 12 bits, weight 0..10: 4 bits
          if ((bal[r] >> lane) & 1ull) {
            const int w = cb_[r] < 64 ? wq[cb_[r]] : 0;
            clist[base + __popcll(bal[r] & ((1ull << lane) - 1ull))] = (uint16_t)((eo << 4) | w);   // at most kVoteChunk entries = 8 KB
          }
          base += __popcll(bal[r]);
        }
        __syncthreads();
        // one thread per (delimiter, start position in its reach): n * (2 delta + 1) votes spread
        // over the workgroup.  Pair number tid + j * threads -> (delimiter ci, offset kk) without a
        // division per pair: the first pair of a thread by a reciprocal multiply (exact, since
        // tid * span < 2^32), the following ones by adding the quotient and remainder of threads / span.
        const int n = *n_list;
        const int span = 2 * delta + 1;
        const uint32_t span_inv = 0xFFFFFFFFu / (uint32_t)span + 1u;   // wraps to 0 for span == 1
        const int step_q = span == 1 ? kTileThreads : (int)__umulhi((uint32_t)kTileThreads, span_inv);
        const int step_r = kTileThreads - step_q * span;
        int ci = span == 1 ? tid : (int)__umulhi((uint32_t)tid, span_inv);
        int kk = tid - ci * span;
        while (ci < n) {
          const int ent = clist[ci];
          const int e = e0 + (ent >> 4);
          const int w = ent & 15;
          const int q = e - C - delta + kk;
          if (q >= p0 && q <= p1 - 1 && q <= L - C - 1) {   // s_e = q + C must stay below L
            const int s_e = q + C;
            const int dist = e > s_e ? e - s_e : s_e - e;
            const unsigned long long sc = (unsigned long long)(p.a_num * w * dd + (p.a_den - p.a_num) * 10 * (dd - dist));
            const unsigned long long key = ((sc + 1ull) << 16) | (unsigned long long)(0xFFFF - (e - q));
            atomicMax(&best[q - p0], key);
          }
          ci += step_q;
          kk += step_r;
          if (kk >= span) { kk -= span; ++ci; }
        }
        __syncthreads();
        if (e0 + kVoteChunk <= e_hi) {                 // another chunk of boundaries follows (rare)
          if (tid == 0) *n_list = 0;
          __syncthreads();
        }
      }
    }
    // successor table (registers first: `best` is about to be overlaid).  Lane-interleaved
    // ownership (i = r*threads + tid) keeps these LDS accesses free of bank conflicts.
#pragma unroll
    for (int r = 0; r < kSegPerThread; ++r) {
      const int i = r * kTileThreads + tid;
      const int q = p0 + i;
      int len = 0;
      if (i < tlen) {
        const int s_e = q + C;
        if (s_e >= L) len = L - q;
        else {
          const unsigned long long key = best[i];
          len = key ? 0xFFFF - (int)(key & 0xFFFFull) : C;
        }
        seg_len[seq0 + q] = (uint16_t)len;             // chunk lengths stay below 2^16 (C + delta <= 8192)
      }
      my_len[r] = len;
    }
  } else {
#pragma unroll
    for (int r = 0; r < kSegPerThread; ++r) {
      const int i = r * kTileThreads + tid;
      my_len[r] = i < tlen ? (int)seg_len[seq0 + p0 + i] : 0;
    }
    if (cand.tile_count != nullptr) {
      // rank of every candidate of the tile: positions are owned interleaved (i = r * threads +
      // tid), so the order is row r, then wavefront, then lane
      const int lane = tid & (DSK_WAVE - 1), wave = tid / DSK_WAVE;
      int* cnt = red + 40;                                 // [kSegPerThread][kTileWaves]; the id slots are free in this mode
      unsigned long long bal[kSegPerThread];
#pragma unroll
      for (int r = 0; r < kSegPerThread; ++r) {
        const int i = r * kTileThreads + tid;
        bal[r] = __ballot(i < tlen && oc1[r] != 255);
        if (lane == 0) cnt[r * kTileWaves + wave] = __popcll(bal[r]);
      }
      if (MODE == 2) {                                     // candidates of the tiles in front of this one
        const int part = wave_sum_i(cand_o);
        if (lane == 0) cnt[kSegPerThread * kTileWaves + wave] = part;
      }
      __syncthreads();
      if (MODE == 2) {
        cand_o = 0;
#pragma unroll
        for (int w = 0; w < kTileWaves; ++w) cand_o += cnt[kSegPerThread * kTileWaves + w];
      }
      static_assert(kSegPerThread * kTileWaves <= DSK_WAVE && (kSegPerThread + 1) * kTileWaves <= 64,
                    "one lane per (row, wavefront) count; the counts fit the id slots");
      const int c = lane < kSegPerThread * kTileWaves ? cnt[lane] : 0;
      const int ex = wave_incl_scan_i(c, lane) - c;
      if (MODE == 2 && tid == DSK_WAVE - 1 && p0 + kSegTile >= L) {   // last tile: ex + c is the tile's count
        cand.cand_cu[0] = 0;
        cand.cand_cu[1] = cand_o + ex + c;
        if (cand_o + ex + c > cand.max_cand) set_status(dev_status, DSK_ERR_CAPACITY);
      }
#pragma unroll
      for (int r = 0; r < kSegPerThread; ++r) {
        const int o = cand_o + __builtin_amdgcn_readlane(ex, r * kTileWaves + wave) +
                      __popcll(bal[r] & ((1ull << lane) - 1ull));
        if (((bal[r] >> lane) & 1ull) && o < cand.max_cand) {
          cand.cand_pos[o] = seq0 + p0 + r * kTileThreads + tid;
          cand.cand_class[o] = (uint8_t)oc1[r];
        }
      }
    }
  }
  __syncthreads();
  if (MODE == 2) {
    // the tiles in front of this one, chained here: the scan buffers lie where the jump entries
    // are built afterwards
    const bool last = p0 + kSegTile >= L;
    uint2* rows = reinterpret_cast<uint2*>(smem);
    int e = 0, blk = 0, sl = 0;
    if (j > 0)
      chain_prefix_tree(cr, L, chain_T, p.map_row, j, rows, rows + kChainLdsEntries / 2, e, blk, sl);
    info = make_int4(p0 + e, blk, sl, 0);
    if (last && tid == 0) {
      // the sequence's totals: one more step, through this tile's own map (staged as row j; for a
      // single tile nothing was staged and its row is read from memory)
      const uint2 c = j > 0 ? rows[j * p.map_row + e] : tile_map[(int64_t)tile * p.map_row];
      const int nb = blk + chain_blocks(c), nsl = sl + chain_slots(c);
      cu_blocks[0] = 0;
      cu_blocks[1] = nb;
      if (cu_slots) { cu_slots[0] = 0; cu_slots[1] = nsl; }
      if (nb > p.cap) set_status(dev_status, DSK_ERR_CAPACITY);
      else { block_start[nb] = p.total_tokens; slot_base[nb] = nsl; }
    }
    __syncthreads();
  }
  uint2 own[kSegPerThread];                            // the thread's own jump entries stay in registers between the rounds
#pragma unroll
  for (int r = 0; r < kSegPerThread; ++r) {
    const int i = r * kTileThreads + tid;
    const int len = my_len[r];
    // ceil(len / b): len + b - 1 < 2^16 and b < 2^15 on the multiply path, so the reciprocal is exact
    const int nslot = p.b_inv ? (int)__umulhi((uint32_t)(len + p.b - 1), p.b_inv) : (len + p.b - 1) / p.b;
    ns[i] = (uint16_t)nslot;
    // level-0 jump: one chunk.  position >= tlen means "left the tile" (i + len <= tlen + C + delta)
    own[r] = make_uint2((uint32_t)(i + len) | ((i < tlen ? 1u : 0u) << 16), (uint32_t)nslot);
    if (MODE == 0) jmp[i] = own[r];
  }
  // pointer jumping: level r holds 2^r chunks per hop; positions that left the tile are fixed
  // points.  Every chunk that does not end the sequence has at least C - delta positions, so the
  // chain crosses the tile in at most ceil(tlen / (C - delta)) hops and as many doublings as cover
  // that number finish every position: a fixed round count, no termination vote.  The first pass
  // keeps the target positions of every level (2 bytes per position and level) for the emit pass.
  const int rounds = jump_rounds(tlen, C - delta);       // C - delta >= 1
  if (rounds - 1 > p.max_levels) {                       // cannot happen for a buffer sized by the host's rule
    if (tid == 0) set_status(dev_status, DSK_ERR_WORKSPACE);
    return;
  }
  if (MODE == 0) {
    __syncthreads();
    int cur = 0;
    for (int round = 0; round < rounds; ++round) {
      const uint2* js = jmp + cur * kSegTile;
      uint2* jd = jmp + (cur ^ 1) * kSegTile;
#pragma unroll
      for (int r = 0; r < kSegPerThread; ++r) {
        const int i = r * kTileThreads + tid;
        uint2 v = own[r];
        const int t = (int)(v.x & 0xFFFFu);
        if (i < tlen && t < tlen) {
          const uint2 v2 = js[t];
          v = make_uint2((v2.x & 0xFFFFu) | ((v.x & 0xFFFF0000u) + (v2.x & 0xFFFF0000u)), v.y + v2.y);
        }
        jd[i] = v;
        own[r] = v;
        if (i < tlen && round < rounds - 1)              // the last level is not hopped from again
          p.seg_jump[(int64_t)round * p.jump_stride + seq0 + p0 + i] = (uint16_t)(v.x & 0xFFFFu);
      }
      cur ^= 1;
      __syncthreads();
    }
    const uint2* fj = jmp + cur * kSegTile;
    if (cand.tile_count != nullptr && tid == 0) {
      int n = 0;
#pragma unroll
      for (int w = 0; w < kTileWaves; ++w) n += red[4 + w];
      cand.tile_count[tile] = n;
    }
    uint2* row = tile_map + (int64_t)tile * p.map_row;
    for (int ent = tid; ent < p.map_row; ent += kTileThreads) {
      uint2 rv = make_uint2(0u, 0u);
      if (ent < tlen) {
        const uint2 v = fj[ent];
        rv = make_uint2(((v.x & 0xFFFFu) - (uint32_t)tlen) | (v.x & 0xFFFF0000u), v.y);
      }
      row[ent] = rv;
    }
    return;
  }

  // emit.  The chunks the chain lays down in this tile are the positions 0, 1, 2 .. hops behind the
  // tile's entry, and hop counts add up along the chain: with the hop-2^l tables of the first pass
  // in LDS (hop 1 = the chunk lengths), the thread that owns the n-th chunk finds its position by
  // one lookup per set bit of n -- no marks, no rounds, no barrier between the lookups.  A chain of
  // the tile has at most 2^rounds chunks; a thread takes two consecutive n.
  static_assert(kMaxJumpLevels + 1 <= (int)(kTileJumpBytes / (kSegTile * 2)), "hop tables fit the jump area");
  uint16_t* tab = reinterpret_cast<uint16_t*>(smem);     // [rounds][kSegTile]
#pragma unroll
  for (int r = 0; r < kSegPerThread; ++r) {
    const int i = r * kTileThreads + tid;
    tab[i] = (uint16_t)(i < tlen ? i + my_len[r] : tlen);
#pragma unroll
    for (int l = 1; l <= kMaxJumpLevels; ++l)
      if (l < rounds) tab[l * kSegTile + i] = lv[l - 1][r];
  }
  __syncthreads();
  constexpr int kPathPer = 2;
  static_assert(kPathPer * kTileThreads >= (1 << (kMaxJumpLevels + 1)), "every chunk of a tile has a thread");
  const int e_in = info.x - p0;
  int pos[kPathPer], nsv[kPathPer];
  int nb_local = 0, ns_local = 0;
#pragma unroll
  for (int r = 0; r < kPathPer; ++r) {
    const int n = tid * kPathPer + r;
    int q = (e_in >= 0 && e_in < tlen && n < (1 << rounds)) ? e_in : tlen;
#pragma unroll
    for (int l = 0; l <= kMaxJumpLevels; ++l)
      if (l < rounds && ((n >> l) & 1) && q < tlen) q = tab[l * kSegTile + q];
    pos[r] = q;
    nsv[r] = q < tlen ? (int)ns[q] : 0;
    if (q < tlen) { ++nb_local; ns_local += nsv[r]; }
  }
  const int lane = tid & (DSK_WAVE - 1), wave = tid / DSK_WAVE;
  const int ib = wave_incl_scan_i(nb_local, lane);
  const int is = wave_incl_scan_i(ns_local, lane);
  if (lane == DSK_WAVE - 1) { red[2 * wave] = ib; red[2 * wave + 1] = is; }
  __syncthreads();
  int ob = 0, os = 0;
#pragma unroll
  for (int w = 0; w < kTileWaves; ++w)
    if (w < wave) { ob += red[2 * w]; os += red[2 * w + 1]; }
  int gb = sq.z + info.y + ob + ib - nb_local;
  int gs = sq.w + info.z + os + is - ns_local;
#pragma unroll
  for (int r = 0; r < kPathPer; ++r) {
    if (pos[r] < tlen) {
      if (gb < p.cap) {
        block_start[gb] = seq0 + p0 + pos[r];
        slot_base[gb] = gs;
      }
      ++gb;
      gs += nsv[r];
    }
  }
}

__global__ __launch_bounds__(kChainThreads) void seg_chain_kernel(
    SegParams p, SegCand cand, const uint2* __restrict__ tile_map, int4* __restrict__ tile_info,
    int4* __restrict__ seq_info, int32_t* __restrict__ cu_blocks, int32_t* __restrict__ cu_slots,
    int32_t* __restrict__ block_start, int32_t* __restrict__ slot_base, int32_t* dev_status) {
  __shared__ uint2 rows[kChainLdsEntries];
  __shared__ int carry[3];
  __shared__ int cand_wave[kChainThreads / DSK_WAVE];
  const int s = blockIdx.x;
  int seq0, L;
  seq_range(p, s, seq0, L);
  if (!seq_ok(p, seq0, L)) L = 0;   // flagged by the tile kernel; emit nothing
  int n_tiles = (L + kSegTile - 1) / kSegTile;
  if (n_tiles > p.tiles_per_seq) n_tiles = p.tiles_per_seq;
  if (threadIdx.x == 0) { carry[0] = 0; carry[1] = 0; carry[2] = 0; }
  if (cand.tile_count != nullptr) {
    // candidate lists: offset of every tile's candidates inside its sequence, and the sequence's
    // total (left in cand_cu[s + 1]; the batch scan turns the totals into offsets)
    const int lane = threadIdx.x & (DSK_WAVE - 1), wave = threadIdx.x / DSK_WAVE;
    int run = 0;
    for (int j0 = 0; j0 < n_tiles; j0 += kChainThreads) {
      const int j = j0 + threadIdx.x;
      const int v = j < n_tiles ? cand.tile_count[s * p.tiles_per_seq + j] : 0;
      const int incl = wave_incl_scan_i(v, lane);
      if (lane == DSK_WAVE - 1) cand_wave[wave] = incl;
      __syncthreads();
      int off = 0, total = 0;
#pragma unroll
      for (int w = 0; w < kChainThreads / DSK_WAVE; ++w) {
        const int t = cand_wave[w];
        if (w < wave) off += t;
        total += t;
      }
      if (j < n_tiles) cand.tile_base[s * p.tiles_per_seq + j] = run + off + incl - v;
      run += total;
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      if (p.B == 1) {
        cand.cand_cu[0] = 0;
        cand.cand_cu[1] = run;
        if (run > cand.max_cand) set_status(dev_status, DSK_ERR_CAPACITY);
      } else {
        cand.cand_cu[s + 1] = run;
      }
    }
  }
  if (p.map_row <= kChainFastSpan) {
    // carry[0] is the entry offset into the first tile of the run
    const int run = (kChainLdsEntries / 2) / p.map_row;
    for (int j0 = 0; j0 < n_tiles; j0 += run) {
      const int T = (n_tiles - j0 < run) ? n_tiles - j0 : run;
      const uint2* src = tile_map + ((int64_t)s * p.tiles_per_seq + j0) * p.map_row;
      __syncthreads();
      ChainRows cr;
      chain_load(cr, src, T, p.map_row);
      const uint2* cur = chain_scan(cr, L, j0, T, p.map_row, rows, rows + kChainLdsEntries / 2);
      // row j now maps an entry of the run's first tile to the state behind tile j0 + j
      const int e0 = carry[0], blk0 = carry[1], slots0 = carry[2];
      for (int j = threadIdx.x; j < T; j += kChainThreads) {
        int e = e0, blk = blk0, sl = slots0;
        if (j > 0) {
          const uint2 c = cur[(j - 1) * p.map_row + e0];
          e = chain_off(c); blk += chain_blocks(c); sl += chain_slots(c);
        }
        tile_info[s * p.tiles_per_seq + j0 + j] = make_int4((j0 + j) * kSegTile + e, blk, sl, 0);
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        const uint2 c = cur[(T - 1) * p.map_row + e0];
        carry[0] = chain_off(c); carry[1] = blk0 + chain_blocks(c); carry[2] = slots0 + chain_slots(c);
      }
    }
  } else {
    const int tiles_per_chunk = kChainLdsEntries / p.map_row;   // map_row <= kSegTile <= entries
    for (int j0 = 0; j0 < n_tiles; j0 += tiles_per_chunk) {
      const int jn = (n_tiles - j0 < tiles_per_chunk) ? n_tiles - j0 : tiles_per_chunk;
      const uint2* src = tile_map + ((int64_t)s * p.tiles_per_seq + j0) * p.map_row;
      __syncthreads();
      for (int i = threadIdx.x; i < jn * p.map_row; i += kChainThreads) rows[i] = src[i];
      __syncthreads();
      if (threadIdx.x == 0) {
        int entry = carry[0], blk = carry[1], slots = carry[2];   // here carry[0] is an absolute position
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
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    seq_info[s] = make_int4(carry[1], carry[2], 0, 0);
    if (p.B == 1) {   // single sequence: the batch scan is trivial, finish here
      cu_blocks[0] = 0;
      cu_blocks[1] = carry[1];
      if (cu_slots) { cu_slots[0] = 0; cu_slots[1] = carry[2]; }
      if (carry[1] > p.cap) set_status(dev_status, DSK_ERR_CAPACITY);
      else { block_start[carry[1]] = p.total_tokens; slot_base[carry[1]] = carry[2]; }
    }
  }
}

// ---- scan over the sequences of the batch (B > 1) ----------------------------------------------
__global__ __launch_bounds__(64) void seg_seqscan_kernel(
    int4* __restrict__ seq_info, int B, int cap, int total_tokens, int32_t* __restrict__ cu_blocks,
    int32_t* __restrict__ cu_slots, int32_t* __restrict__ block_start, int32_t* __restrict__ slot_base,
    int32_t* cand_cu, int max_cand, int32_t* dev_status) {
  if (threadIdx.x != 0) return;
  if (cand_cu != nullptr) {   // per-sequence candidate totals (behind each sequence's entry) -> offsets
    int run = 0;
    cand_cu[0] = 0;
    for (int s = 0; s < B; ++s) {
      run += cand_cu[s + 1];
      cand_cu[s + 1] = run;
    }
    if (run > max_cand) set_status(dev_status, DSK_ERR_CAPACITY);
  }
  int blk = 0, slots = 0;
  for (int s = 0; s < B; ++s) {
    int4 v = seq_info[s];
    cu_blocks[s] = blk;
    if (cu_slots) cu_slots[s] = slots;
    v.z = blk;
    v.w = slots;
    seq_info[s] = v;
    blk += v.x;
    slots += v.y;
  }
  cu_blocks[B] = blk;
  if (cu_slots) cu_slots[B] = slots;
  if (blk > cap) {
    set_status(dev_status, DSK_ERR_CAPACITY);
    return;   // the tables stay self-consistent for the truncated prefix
  }
  block_start[blk] = total_tokens;
  slot_base[blk] = slots;
}

// ---- host -----------------------------------------------------------------------------------
hipError_t launch_segment(const dsk_compress_args& a, const CompressWs& ws, SegClassSource src, hipStream_t st) {
  unsigned char* w = static_cast<unsigned char*>(a.workspace);
  SegCand cand = {};
  if (src == SegClassSource::kTokenIdsWithLists) {
    cand.own_cls = w + ws.cls_at;
    cand.tile_count = reinterpret_cast<int32_t*>(w + ws.seg_cand);
    cand.tile_base = cand.tile_count + (size_t)a.B * ws.tiles_per_seq;
    cand.cand_cu = a.cand_cu;
    cand.cand_pos = a.cand_pos;
    cand.cand_class = a.cand_class;
    cand.max_cand = a.max_cand_total;
  }
  const bool classify_here = src == SegClassSource::kTokenIds || src == SegClassSource::kTokenIdsWithLists;
  uint8_t* cls_at = w + ws.cls_at;
  uint16_t* seg_len = reinterpret_cast<uint16_t*>(w + ws.seg_len);
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
  p.b_inv = (a.b > 1 && a.b < 32768) ? 0xFFFFFFFFu / (uint32_t)a.b + 1u : 0u;
  p.map_row = ws.map_row; p.tiles_per_seq = ws.tiles_per_seq;
  p.max_seqlen = a.max_seqlen; p.total_tokens = a.total_tokens;
  p.B = a.B; p.cap = a.max_blocks_total;
  p.seg_jump = reinterpret_cast<uint16_t*>(w + ws.seg_jump);
  p.max_levels = ws.jump_levels;
  p.jump_stride = ws.jump_stride;

  hipError_t err;
  if (src == SegClassSource::kCallerLists) {   // scatter the caller's candidates into the dense class array
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
    // kTokenIds: no class bytes exist; the tile kernel classifies the tokens of its reach itself
    seg_tile_kernel<0><<<grid, dim3(kTileThreads), lds, st>>>(
        p, cand, classify_here ? nullptr : cls_at, a.token_ids, a.delim_ids, seg_len, tile_map,
        tile_info, seq_info, a.cu_blocks, a.cu_slots, a.block_start, a.slot_base, a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  // one sequence whose entry maps fit one run of the chain scan: the emit pass chains for itself
  const bool self_chain = a.B == 1 && a.max_seqlen == a.total_tokens && ws.tiles_per_seq >= 1 &&
                          ws.tiles_per_seq < kTileThreads &&
                          ws.map_row <= kChainFastSpan &&
                          (int64_t)ws.tiles_per_seq * ws.map_row <= kChainLdsEntries / 2;
  if (self_chain) {
    const dim3 grid((unsigned)ws.tiles_per_seq, 1u);
    seg_tile_kernel<2><<<grid, dim3(kTileThreads), lds, st>>>(p, cand, nullptr, nullptr, nullptr, seg_len, tile_map,
                                                             tile_info, seq_info, a.cu_blocks, a.cu_slots,
                                                             a.block_start, a.slot_base, a.dev_status);
    return hipGetLastError();
  }
  seg_chain_kernel<<<dim3((unsigned)a.B), dim3(kChainThreads), 0, st>>>(p, cand, tile_map, tile_info, seq_info, a.cu_blocks,
                                                                      a.cu_slots, a.block_start, a.slot_base,
                                                                      a.dev_status);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (a.B > 1) {
    seg_seqscan_kernel<<<dim3(1), dim3(64), 0, st>>>(seq_info, a.B, a.max_blocks_total, a.total_tokens,
                                                     a.cu_blocks, a.cu_slots, a.block_start, a.slot_base,
                                                     cand.tile_count ? cand.cand_cu : nullptr, cand.max_cand,
                                                     a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (ws.tiles_per_seq > 0) {
    const dim3 grid((unsigned)ws.tiles_per_seq, (unsigned)a.B);
    seg_tile_kernel<1><<<grid, dim3(kTileThreads), lds, st>>>(p, cand, nullptr, nullptr, nullptr, seg_len, tile_map,
                                                             tile_info, seq_info, a.cu_blocks, a.cu_slots,
                                                             a.block_start, a.slot_base, a.dev_status);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  return hipSuccess;
}

}  // namespace dsk
