// Host-side internals of libdsk: workspace layouts and the per-stage launchers that the
// C-ABI entry points in dsk_api.hip call.  Nothing here is exported.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/dsk.h"

namespace dsk {

constexpr int kSegTile = 2048;        // positions per DD-Select tile
constexpr int kMaxChunkSpan = 8192;   // limit on C + delta
constexpr int64_t kMaxTokenStride = 1 << 24;  // elements; keeps 32 rows of lane offsets in 32 bits
constexpr int kCandTile = 1024;       // tokens per candidate-extraction tile
constexpr int kMaxSamplesPerClass = 64;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- dsk_compress workspace ---------------------------------------------------------------
struct CompressWs {
  size_t tile_map;    // uint2 [n_tiles * map_row]   entry offset -> (exit offset | blocks<<16, slots)
  size_t tile_info;   // int4 [n_tiles]              entry position, block offset, slot offset
  size_t seq_info;    // int4 [B]                    blocks, slots, block base, slot base
  size_t cls_at;      // u8  [total_tokens]          dense class of each token, 255 = none
  size_t seg_len;     // u16 [total_tokens]          length of the chunk that would start at each position
  size_t tile_count;  // i32 [n_cand_tiles + 1]      candidates per tile, then exclusive scan
  size_t seg_cand;    // i32 [2 * n_tiles]           candidates per segmentation tile, then their offsets in the sequence
  size_t seg_jump;    // u16 [jump_levels][jump_stride]  position in the tile 2, 4, 8 .. chunks after each token
  size_t imp_part;    // f32 [B * n_class * M * Hkv] per-(sample, kv head) partial sums
  size_t total;
  int tiles_per_seq;  // ceil(max_seqlen / kSegTile)
  int map_row;        // min(C + delta, kSegTile)
  int n_cand_tiles;   // ceil(total_tokens / kCandTile)
  int jump_levels;    // doubling levels kept per token: enough for a tile of chunks of C - delta positions
  int jump_stride;    // total_tokens rounded up to 16
};
CompressWs compress_ws_layout(const dsk_compress_args& a);

hipError_t launch_candidates(const dsk_compress_args& a, const CompressWs& ws, hipStream_t st);
hipError_t launch_importance(const dsk_compress_args& a, const CompressWs& ws, hipStream_t st);
// where stage SEGMENT finds the delimiter class of a token
enum class SegClassSource {
  kClassBytes,    // dense class bytes in the workspace, just written by launch_candidates
  kCallerLists,   // the caller's candidate lists (scattered into the class bytes first)
  kTokenIds,      // token_ids / delim_ids, classified inside the tile kernel (no lists were asked for)
  kTokenIdsWithLists   // as kTokenIds, and the segmentation kernels also write the candidate lists
};
// the per-class samples of Alg. 1 from finished candidate lists
hipError_t launch_cand_sample(const dsk_compress_args& a, hipStream_t st);
hipError_t launch_segment(const dsk_compress_args& a, const CompressWs& ws, SegClassSource src, hipStream_t st);
hipError_t launch_summaries(const dsk_compress_args& a, hipStream_t st);

// ---- dsk_select_topk ----------------------------------------------------------------------
// block scores live in the workspace as rows of `stride` = round_up(max_blocks_total, 4) floats
inline int select_score_stride(const dsk_select_args& a) { return (a.max_blocks_total + 3) / 4 * 4; }
hipError_t launch_scores(const dsk_select_args& a, float* scores, int stride, hipStream_t st);
hipError_t launch_select(const dsk_select_args& a, const float* scores, int stride, hipStream_t st);

// ---- dsk_sparse_decode_attn -----------------------------------------------------------------
struct AttnWs {
  size_t part_ml;   // float2 [B*Hq*nchunks]  (running max in log2 units, denominator)
  size_t part_acc;  // f32 [B*Hq*nchunks*D]
  size_t total;
  int nchunks;
  int slots_per_wg;  // slots one attention workgroup folds into one partial (16; 8 for b > 32, and for b <= 16 in launches of many workgroups)
};
AttnWs attn_ws_layout(const dsk_attn_args& a);
hipError_t launch_attn(const dsk_attn_args& a, const AttnWs& ws, hipStream_t st);
// Fixed-order merge of nchunks partials per (sequence, head); chunk c is valid for
// c < ceil(min(count, k) / per_chunk) where count = counts[s*Hq+h], or the length of sequence s
// when cu_seqlens is given.  sel_div consecutive heads read one entry of counts ([B, Hq/sel_div]).
hipError_t launch_attn_merge(const float2* part_ml, const float* part_acc, const int32_t* counts,
                             const int32_t* cu_seqlens, int B, int Hq, int sel_div, int k, int nchunks, int per_chunk,
                             float* out, uint16_t* out_bf16, float* lse, hipStream_t st);

// ---- dsk_dense_decode_attn workspace ---------------------------------------------------------
struct DenseWs {
  size_t part_ml;        // float2 [B*Hq*nsplit]
  size_t part_acc;       // f32 [B*Hq*nsplit*D]
  size_t total;
  int nsplit;            // token ranges per sequence
  int tokens_per_split;  // multiple of 128
  int group_tile;        // query heads of a GQA group folded per pass over K/V (1, 2 or 4)
};
DenseWs dense_ws_layout(const dsk_dense_attn_args& a);
hipError_t launch_dense_attn(const dsk_dense_attn_args& a, const DenseWs& ws, hipStream_t st);

// summaries of the blocks [blk_range[0], blk_range[1]) only (device-resident range)
hipError_t launch_summaries_range(const void* X, int64_t stride_tok, int64_t stride_head, int Hkv,
                                  const int32_t* block_start, const int32_t* blk_range, int max_blocks_in_range,
                                  int cap, int total_tokens, int summary_mode, void* out, int32_t* dev_status,
                                  hipStream_t st);
// incremental update: workspace = int32 {first recomputed block, new block count}
hipError_t launch_append(const dsk_append_args& a, hipStream_t st);
// the same for a batch with one table region per sequence: workspace = int4 [B] {first rewritten
// entry, end, first K/V row, new length}
hipError_t launch_summaries_batch_ranges(const void* X, int64_t stride_tok, int64_t stride_head, int Hkv, int B,
                                         const int32_t* block_start, const void* ranges, int max_blocks_in_range,
                                         int out_rows, int summary_mode, void* out, int32_t* dev_status,
                                         hipStream_t st);
hipError_t launch_append_batch(const dsk_append_batch_args& a, hipStream_t st);

// KV reuse over resident buffers: workspace = int32 [B*Hq] reusable counts
size_t reuse_ws_bytes(const dsk_reuse_args& a);
hipError_t launch_reuse(const dsk_reuse_args& a, hipStream_t st);

}  // namespace dsk
