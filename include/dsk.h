/*
 * dsk.h -- C ABI of the DynSplit-KV hot path for AMD MI355X (gfx950).
 *
 * Three calls make up the path:
 *   dsk_compress            KV-cache compression pass: delimiter candidates, delimiter
 *                           importance (Alg. 1, Sec. 3), DD-Select segmentation (Sec. 4.1),
 *                           variable-to-fixed slot map and min/max block summaries (Sec. 4.2).
 *   dsk_select_topk         per decode step: query x block-summary scores, top-k over the
 *                           block-to-slot mapped scores (Sec. 4.2; App. B.2 Step 1).
 *   dsk_sparse_decode_attn  per decode step: attention over the K/V of the selected slots
 *                           (App. B.2 Steps 2-3).
 * and three more sit beside it:
 *   dsk_reuse_update        step-to-step reuse of the gathered K/V in per-head resident buffers of
 *                           fixed-size slots (App. B.2, "KVCache Reuse with V2F").
 *   dsk_append_tokens       incremental update of the block table and summaries while decoding
 *                           (Sec. 4.1, "Incremental Update during Decoding"), one sequence per call.
 *   dsk_append_tokens_batch the same update for every sequence of a batch in one call, on tables in
 *                           which each sequence has its own region with room to grow.
 *   dsk_dense_decode_attn   full attention over the whole cache: the full-KV baseline the method
 *                           is compared with (Sec. 5, GPU Inference analysis).
 *
 * Conventions that hold for every call
 *   - Pointers marked [dev] are device (HBM) addresses, [host] are host addresses.
 *     The caller owns every buffer; the library allocates nothing, frees nothing and
 *     keeps no pointer after the call returns.  Scratch memory comes from the
 *     caller-provided `workspace` ([dev], 256-byte aligned) whose size the matching
 *     *_workspace_bytes() query reports for the same argument struct.
 *   - All work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to
 *     void*; NULL is the default stream).  No call synchronises the device.
 *   - Argument validation is synchronous and happens before anything is enqueued: a
 *     negative dsk_status means nothing was launched.  Data-dependent problems found on
 *     the device (block capacity exceeded, bad per-sequence parameters) are written to
 *     the `dev_status` word ([dev], optional) as a dsk_status value; outputs are then
 *     truncated but every kernel still terminates.
 *   - Tokens of a ragged batch are flattened: sequence s owns global token positions
 *     cu_seqlens[s] .. cu_seqlens[s+1]-1.  Block boundaries, slot numbers and selected
 *     token spans are all expressed in these global coordinates.
 *   - K, V, q and summaries are bf16 (raw 16-bit patterns), head_dim D must be 128.
 *   - Same inputs give bit-identical outputs (fixed reduction orders, no float atomics).
 *   - Non-finite K/V/q values give unspecified results but never hang.
 *   - A batch without any token (total_tokens == 0) is valid everywhere: tables come out empty,
 *     nothing is selected, attention returns out = 0 and lse = -inf; K, V and token_ids are not
 *     read and may be NULL in that case only.
 */
#ifndef DSK_H_
#define DSK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DSK_ABI_VERSION 3u
#define DSK_HEAD_DIM 128
#define DSK_MAX_CLASSES 64

typedef enum dsk_status {
  DSK_OK = 0,
  DSK_ERR_NULL = -1,      /* a required pointer is NULL */
  DSK_ERR_SHAPE = -2,     /* B, heads, D, lengths or strides are not usable */
  DSK_ERR_PARAM = -3,     /* C, delta, alpha, b, budget, M, W, R out of range */
  DSK_ERR_ALIGN = -4,     /* K/V/q/summary/workspace pointer or stride not 16-byte aligned */
  DSK_ERR_WORKSPACE = -5, /* workspace missing or smaller than *_workspace_bytes() */
  DSK_ERR_CAPACITY = -6,  /* more blocks/candidates produced than the outputs can hold */
  DSK_ERR_ORDER = -7,     /* caller-provided candidate positions of a sequence are not strictly ascending
                             (found on the device, reported through dev_status) */
  DSK_ERR_LAUNCH = -8,    /* the HIP runtime refused a launch */
  DSK_ERR_VERSION = -9    /* struct_size does not match this library */
} dsk_status;

/* Stages of dsk_compress (bit mask).  A stage that is not run takes its inputs from the
 * buffers the earlier stage would have written. */
enum { DSK_SUMMARY_MINMAX = 0, DSK_SUMMARY_MEAN = 1 };

enum {
  DSK_STAGE_CANDIDATES = 1, /* token_ids + delim_ids -> cand_pos/cand_class/cand_cu (+ samp_pos) */
  DSK_STAGE_IMPORTANCE = 2, /* samp_pos + qwin + K -> class_weight_q (Alg. 1) */
  DSK_STAGE_SEGMENT = 4,    /* candidates + class_weight_q -> block_start/cu_blocks/slot_base */
  DSK_STAGE_SUMMARIES = 8,  /* block_start + K (+V) -> ksum (+vsum) */
  DSK_STAGE_ALL = 15
};

/* ------------------------------------------------------------------------------------------
 * dsk_compress -- the compression pass.
 *
 * Stage CANDIDATES (input set D of Alg. 1; the semantic boundary tokens of Sec. 4.1):
 *   every token whose id is in delim_ids is a candidate; its class is the index of the id
 *   in delim_ids.  Output lists are ascending in global position.  Also chooses the
 *   sampled candidates for Alg. 1: per sequence and class the first M occurrences whose
 *   sequence-local position t satisfies R <= t <= L-1-W.
 *   When only the segmentation of the same call needs the candidates (weights from a table:
 *   no sampling), the lists may be left out: cand_pos == cand_class == NULL with
 *   max_cand_total == 0 writes neither the lists nor cand_cu (which may then be NULL too); stage
 *   SEGMENT then classifies the tokens it needs itself.
 * Stage IMPORTANCE (Alg. 1 and the equation of Sec. 3, on the one layer given):
 *   for each sampled candidate t, each query head and each of the W queries following t,
 *   the causal softmax row over keys 0..q is split into the retained region
 *   {max(0,t-R+1)..t} and the discarded region {0..max(0,t-R)};
 *   s_t = mean(retained mass - alpha_imp * discarded mass).  Class means are mapped to
 *   [0,1] by (mean + alpha_imp) / (1 + alpha_imp), clamped, and rounded half-up to tenths.
 *   Classes without a sample keep the value already in class_weight_q.  One call covers one
 *   layer; samp_score_sum carries the mean over several layers from call to call.
 * Stage SEGMENT (Sec. 4.1, Dynamic Segmentation Procedure; Sec. 4.2 variable-to-fixed map):
 *   a candidate at position t offers the boundary e = t+1.  From s_c (0 at first):
 *   s_e = s_c + C; if s_e >= L the last chunk ends at L; else the offered boundary in
 *   [s_e-delta, min(L, s_e+delta)] maximising
 *       alpha_num*wq*D' + (alpha_den-alpha_num)*10*(D' - |e-s_e|),  D' = max(delta,1)
 *   (ties: smallest e) ends the chunk, or s_e if none is offered.  Integer arithmetic.
 *   Block i of the batch covers [block_start[i], block_start[i+1]); it owns the
 *   ceil(len/b) slots slot_base[i] .. slot_base[i+1]-1, each b tokens, the last one
 *   possibly shorter.
 * Stage SUMMARIES (Sec. 4.2, KVCache Compression): element-wise minimum and maximum of K
 *   (and of V when vsum != NULL) over the tokens of every block, exact in bf16.
 *   summary_mode DSK_SUMMARY_MEAN (the mean-pooling variant of App. A.2, everything else
 *   unchanged): the per-channel mean instead -- fp32 sum in a fixed order, divided by the
 *   block length, rounded to nearest-even bf16 -- written to both rows of the record, so that
 *   the score of dsk_select_topk, sum_d max(q_d*m_d, q_d*m_d), is the dot product q.m.
 * ---------------------------------------------------------------------------------------- */
typedef struct dsk_compress_args {
  uint32_t struct_size;        /* sizeof(dsk_compress_args) */
  uint32_t stages;             /* DSK_STAGE_* mask */

  /* geometry */
  int32_t B;                   /* sequences, >= 1 */
  int32_t Hq, Hkv, D;          /* query heads, KV heads (Hq % Hkv == 0), head dim (128) */
  int32_t total_tokens;        /* [host copy] cu_seqlens[B] */
  int32_t max_seqlen;          /* [host copy] max_s (cu_seqlens[s+1]-cu_seqlens[s]) */
  const int32_t* cu_seqlens;   /* [dev] [B+1], non-decreasing, cu_seqlens[0] == 0 */

  /* KV cache, bf16; element strides; dim stride is 1.  V may be NULL when vsum is NULL. */
  const void* K;               /* [dev] K[h*k_stride_head + t*k_stride_tok + d] */
  const void* V;               /* [dev] */
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head; /* multiples of 8; token strides <= 2^24 */

  /* candidates */
  const int32_t* token_ids;    /* [dev] [total_tokens]            (stage CANDIDATES in) */
  const int32_t* delim_ids;    /* [dev] [n_class] distinct ids    (stage CANDIDATES in) */
  int32_t n_class;             /* 1..DSK_MAX_CLASSES */
  int32_t max_cand_total;      /* capacity of cand_pos / cand_class */
  int32_t* cand_pos;           /* [dev] [max_cand_total] global positions, ascending (out of
                                  CANDIDATES, in of SEGMENT); NULL: see stage CANDIDATES */
  uint8_t* cand_class;         /* [dev] [max_cand_total] */
  int32_t* cand_cu;            /* [dev] [B+1] candidate range of each sequence */

  /* importance */
  int32_t M, W, R;             /* samples per class (<= 64), future window, retained size */
  float alpha_imp;             /* penalty on discarded mass (paper: 1) */
  float imp_scale;             /* logit scale; 0 -> D^-1/2 */
  int32_t* samp_pos;           /* [dev] [B, n_class, M] global position or -1 (out of
                                  CANDIDATES, in of IMPORTANCE) */
  const void* qwin;            /* [dev] bf16 [B, n_class*M, W, Hq, D]: qwin[s, c*M+m, w, h, :]
                                  is the query of head h at position samp_pos[s,c,m]+1+w */
  uint8_t* class_weight_q;     /* [dev] [B, n_class] weights in tenths, 0..10 (in/out) */
  float* class_mean;           /* [dev] [B, n_class] optional out: class mean score, NaN if
                                  the class had no sample */
  float* samp_score;           /* [dev] [B, n_class, M] optional out: s_t per sample (this layer) */
  float* samp_score_sum;       /* [dev] [B, n_class, M] optional in/out.  The expectation of Alg. 1 also runs
                                  over layers: call stage IMPORTANCE once per layer (its K and qwin) with this
                                  array -- zeroed before the first layer -- and imp_layers = 1, 2, ...; each
                                  call adds its s_t, and class_mean / class_weight_q are then taken from
                                  sum / imp_layers, i.e. after the last layer from the mean over all layers. */
  int32_t imp_layers;          /* layers in samp_score_sum including this call; read only with samp_score_sum */

  /* segmentation */
  int32_t C, delta;            /* base chunk size, max deviation: C >= 1, 0 <= delta < C,
                                  C + delta <= 8192.  With per-sequence arrays these are
                                  upper bounds of the per-sequence values. */
  const int32_t* C_per_seq;    /* [dev] [B] or NULL */
  const int32_t* delta_per_seq;/* [dev] [B] or NULL */
  int32_t alpha_num, alpha_den;/* alpha_sel = alpha_num/alpha_den in [0,1], alpha_den in 1..1000 */
  int32_t b;                   /* fixed mapped block (slot) length, 1..1024 */
  int32_t max_blocks_total;    /* capacity (in blocks) of the outputs below */
  int32_t* block_start;        /* [dev] [max_blocks_total+4] (entries 0..max_blocks_total used) */
  int32_t* cu_blocks;          /* [dev] [B+1] block range of each sequence */
  int32_t* slot_base;          /* [dev] [max_blocks_total+4] (entries 0..max_blocks_total used;
                                  dsk_select_topk reads it in 16-byte vectors) */
  int32_t* cu_slots;           /* [dev] optional out of SEGMENT, [B+1]: slot range of each sequence,
                                  cu_slots[s] = slot_base[cu_blocks[s]], cu_slots[B] = all slots */

  /* summaries: [Hkv, max_blocks_total, 2, D] bf16; [.., 0, :] = min, [.., 1, :] = max
     (DSK_SUMMARY_MEAN: both rows hold the mean) */
  void* ksum;                  /* [dev] */
  void* vsum;                  /* [dev] or NULL */
  int32_t summary_mode;        /* DSK_SUMMARY_MINMAX (0) or DSK_SUMMARY_MEAN */
  int32_t sum_stride_blocks;   /* records per head in ksum / vsum; 0 = max_blocks_total.  Larger when the
                                  call fills one sequence's region of a batch's tables (see
                                  dsk_append_tokens_batch): the table pointers then point at the region,
                                  max_blocks_total is the region's capacity */

  int32_t* dev_status;         /* [dev] optional; must be zeroed by the caller */
  void* workspace;             /* [dev] */
  size_t workspace_bytes;
} dsk_compress_args;

/* ------------------------------------------------------------------------------------------
 * dsk_select_topk -- block scores and slot top-k for one decode step.
 *
 *   score[hq, i] = sum_d max(q_d*kmax[hk,i,d], q_d*kmin[hk,i,d]),  hk = hq / (Hq/Hkv)
 *   (Sec. 4.2 "query-compressed vector product" for a (min,max) summary), fp32 accumulate.
 *   Every slot inherits its block's score (Sec. 4.2 block-to-token mapping at slot
 *   granularity; b = 1 is the token-level mapping).  Per (sequence, query head) the
 *   min(k, slots of the sequence) best slots are selected, k = budget / b, ranked by
 *   (score descending, slot index ascending), and returned in ascending slot order.
 * ---------------------------------------------------------------------------------------- */
/* dsk_select_args.flags.  DSK_SELECT_SHARED_BY_KV_GROUP is an extension that is NOT in the paper
 * (which selects per head, App. B.2 Step 1, and does not say how grouped-query models are
 * handled): the Hq/Hkv query heads of a KV head share one selection, made on the largest score
 * any of them gives a block, so that the group gathers one set of K/V rows per step. */
#define DSK_SELECT_SHARED_BY_KV_GROUP 1u

typedef struct dsk_select_args {
  uint32_t struct_size;
  int32_t B, Hq, Hkv, D;
  int32_t max_blocks_total;    /* capacity used when ksum / block tables were allocated */
  int32_t max_blocks_used;     /* [host] optional tighter upper bound on cu_blocks[B], e.g. the value
                                  read back once after dsk_compress; 0 = max_blocks_total.  Only
                                  sizes the launch and bounds speculative reads; the device value
                                  still decides what is scored. */
  int32_t max_blocks_per_seq;  /* [host] optional upper bound on the blocks of any ONE sequence (0 = the
                                  bound above).  Picks the workgroup size / register tile of the
                                  selection kernel; a sequence with more blocks is still selected
                                  correctly, through the memory-resident path. */
  const int32_t* cu_blocks;    /* [dev] [B+1] */
  const int32_t* block_start;  /* [dev] both tables: 16-byte aligned and readable up to a multiple */
  const int32_t* slot_base;    /* [dev] of 4 entries, i.e. allocate max_blocks_total + 4 ints */
  const void* ksum;            /* [dev] bf16 [Hkv, max_blocks_total, 2, D] */
  const void* q;               /* [dev] bf16 [B, Hq, D] */
  int32_t b;                   /* slot length used by dsk_compress */
  int32_t budget;              /* token budget per sequence; k = budget / b >= 1 */
  const int32_t* budget_per_seq; /* [dev] optional [B]: each sequence's own token budget (a budget that
                                  follows the sequence length, say); sequence s takes
                                  min(k, max(1, budget_per_seq[s] / b)) slots, the arrays keep k entries */
  uint32_t flags;              /* DSK_SELECT_* bits; with DSK_SELECT_SHARED_BY_KV_GROUP read Hkv for Hq in
                                  the shapes of the five outputs below */
  int32_t* sel_slot;           /* [dev] [B, Hq, k] global slot index, ascending; -1 padding */
  int32_t* sel_start;          /* [dev] [B, Hq, k] first global token of the slot */
  int32_t* sel_len;            /* [dev] [B, Hq, k] tokens in the slot (1..b); 0 padding */
  int32_t* sel_count;          /* [dev] [B, Hq] number of selected slots */
  float* scores;               /* [dev] optional out [Hq, max_blocks_total] block scores */
  /* Tables with a region per sequence (dsk_append_tokens_batch); both NULL for the packed tables of
     a batched dsk_compress.  cu_blocks then holds the region starts, and */
  const int32_t* blocks_used;  /* [dev] optional [B]: sequence s has blocks cu_blocks[s] .. +blocks_used[s]-1
                                  (what lies between them and the next region is scored but never
                                  selected) */
  const int32_t* seq_row0;     /* [dev] optional [B]: block_start of sequence s counts from the sequence's
                                  first token, which is row seq_row0[s] of K / V; added to sel_start */
  void* workspace;             /* [dev] */
  size_t workspace_bytes;
} dsk_select_args;

/* ------------------------------------------------------------------------------------------
 * dsk_sparse_decode_attn -- attention of one decode query per (sequence, head) over the
 * tokens of the selected slots (App. B.2 Steps 2-3):
 *   z_t = q.K[hk,t] * scale;  out = sum_t softmax(z)_t V[hk,t];  lse = log sum_t exp(z_t)
 * fp32 accumulation, split over slots with an online-softmax merge in a fixed order.
 * A (sequence, head) with no selected token gets out = 0 and lse = -inf.
 * ---------------------------------------------------------------------------------------- */
/* dsk_attn_args.flags: stop after the per-chunk partials (running max in log2 units, denominator,
 * unnormalised numerator) and leave them in the workspace -- for a caller that merges partials
 * itself, e.g. across devices that each hold part of a sequence.  out / lse are then final only
 * for heads whose selection fits one chunk. */
#define DSK_ATTN_PARTIALS_ONLY 1u
/* the sel_* arrays hold one selection per (sequence, KV head) -- [B, Hkv, k] and [B, Hkv], as
 * dsk_select_topk writes them with DSK_SELECT_SHARED_BY_KV_GROUP -- used by all Hq/Hkv query heads
 * of that KV head */
#define DSK_ATTN_SHARED_SELECTION 2u

typedef struct dsk_attn_args {
  uint32_t struct_size;
  int32_t B, Hq, Hkv, D;
  const void* q;               /* [dev] bf16 [B, Hq, D] */
  const void* K;               /* [dev] bf16, strides as in dsk_compress_args */
  const void* V;               /* [dev] */
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  int32_t total_tokens;        /* [host] tokens per head in K/V; spans outside it are skipped */
  int32_t k;                   /* slots per (sequence, head) in the sel_* arrays */
  int32_t b;                   /* upper bound of sel_len entries */
  const int32_t* sel_start;    /* [dev] [B, Hq, k] */
  const int32_t* sel_len;      /* [dev] [B, Hq, k] */
  const int32_t* sel_count;    /* [dev] [B, Hq] */
  float scale;                 /* 0 -> D^-1/2 */
  uint32_t flags;              /* DSK_ATTN_* bits */
  float* out;                  /* [dev] f32 [B, Hq, D] */
  void* out_bf16;              /* [dev] optional bf16 [B, Hq, D]: `out` rounded to nearest even */
  float* lse;                  /* [dev] f32 [B, Hq], natural log; may be NULL */
  void* workspace;             /* [dev] */
  size_t workspace_bytes;
} dsk_attn_args;

/* ------------------------------------------------------------------------------------------
 * dsk_dense_decode_attn -- full attention of one decode query per (sequence, head) over the
 * WHOLE cache: out = softmax(q K^T scale) V over every token of the sequence.  This is the
 * full-KV baseline the method is compared with (Sec. 5, GPU Inference analysis, Figure 8), on
 * the same device and the same K/V layout, so that a decode step of the sparse path can be set
 * against it.  The heads of a GQA group share one pass over their K/V rows (every K/V byte is
 * read once per call when Hq/Hkv is 1, 2 or 4; twice for 8; other ratios read it Hq/Hkv times).
 * bf16 inputs, fp32 accumulation, split over tokens with an online-softmax merge in a fixed
 * order.  A sequence of length 0 gets out = 0 and lse = -inf.
 * ---------------------------------------------------------------------------------------- */
typedef struct dsk_dense_attn_args {
  uint32_t struct_size;
  int32_t B, Hq, Hkv, D;
  const void* q;               /* [dev] bf16 [B, Hq, D] */
  const void* K;               /* [dev] bf16, strides as in dsk_compress_args */
  const void* V;               /* [dev] */
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  int32_t total_tokens;        /* [host] tokens per head in K/V; cu_seqlens[B] must not exceed it */
  int32_t max_seqlen;          /* [host] upper bound of the sequence lengths (sizes the split); >= 1
                                  unless total_tokens == 0 */
  const int32_t* cu_seqlens;   /* [dev] [B+1] */
  float scale;                 /* 0 -> D^-1/2 */
  uint32_t flags;              /* must be 0 */
  float* out;                  /* [dev] f32 [B, Hq, D] */
  void* out_bf16;              /* [dev] optional bf16 [B, Hq, D]: `out` rounded to nearest even */
  float* lse;                  /* [dev] f32 [B, Hq], natural log; may be NULL */
  void* workspace;             /* [dev] 256-byte aligned */
  size_t workspace_bytes;
} dsk_dense_attn_args;

/* ------------------------------------------------------------------------------------------
 * dsk_append_tokens -- incremental update during decoding (Sec. 4.1): the chunks already
 * computed are kept and only the most recent segmentation ranges are recomputed.
 *
 * One sequence per call, in the single-sequence layout of dsk_compress (block_start[0] == 0,
 * cu_blocks == {0, nblk}); a batch is updated with one call per sequence on that sequence's own
 * tables.  The sequence has grown from len_old to len_new tokens; token_ids and the K (V) rows
 * of the new tokens are already in place.  The end of the chunk that starts at s was chosen
 * among boundaries up to s + C + delta, so it is final iff s + C + delta <= len_old; the
 * procedure of stage SEGMENT is re-run from the start of the first chunk that is not final (with
 * the delimiter classes taken from token_ids / delim_ids and the weights from class_weight_q),
 * and block_start, slot_base, cu_blocks[1] and the summaries of the recomputed chunks are
 * rewritten.  The result equals a dsk_compress of the len_new tokens from scratch, bit for bit.
 * Data-dependent errors through *dev_status: DSK_ERR_SHAPE if the table on the device does not
 * end at len_old, DSK_ERR_CAPACITY if the chunks do not fit max_blocks_total (the table is
 * then truncated).  C, delta, alpha and b must be the values the table was built with.
 * ---------------------------------------------------------------------------------------- */
typedef struct dsk_append_args {
  uint32_t struct_size;
  int32_t Hkv, D;
  int32_t len_old, len_new;    /* [host] len_new >= len_old >= 0 */
  const void* K;               /* [dev] bf16, rows 0..len_new-1 valid; strides as in dsk_compress_args */
  const void* V;               /* [dev] may be NULL when vsum is NULL */
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  const int32_t* token_ids;    /* [dev] [len_new] */
  const int32_t* delim_ids;    /* [dev] [n_class] */
  int32_t n_class;
  const uint8_t* class_weight_q; /* [dev] [n_class] tenths */
  int32_t C, delta, alpha_num, alpha_den, b;
  int32_t max_blocks_total;    /* capacity of the tables below */
  int32_t* block_start;        /* [dev] in/out [max_blocks_total + 4] */
  int32_t* cu_blocks;          /* [dev] in/out [2] */
  int32_t* slot_base;          /* [dev] in/out [max_blocks_total + 4] */
  void* ksum;                  /* [dev] in/out bf16 [Hkv, max_blocks_total, 2, D] */
  void* vsum;                  /* [dev] in/out or NULL */
  int32_t summary_mode;        /* as in dsk_compress_args */
  int32_t* first_recomputed;   /* [dev] optional out: index of the first rewritten chunk */
  int32_t* first_stale_slot;   /* [dev] optional out: slot_base of that chunk -- slots from there on were
                                  re-mapped (what dsk_reuse_update takes as stale_from) */
  int32_t* dev_status;         /* [dev] optional */
  void* workspace;             /* [dev] 256-byte aligned, dsk_append_workspace_bytes() */
  size_t workspace_bytes;
} dsk_append_args;

/* ------------------------------------------------------------------------------------------
 * dsk_append_tokens_batch -- the incremental update of Sec. 4.1 for all B sequences of a batch in
 * one call (every sequence of a decoding batch grows by a token per step).
 *
 * A batch whose sequences grow cannot keep them back to back, so every sequence owns a region
 * with spare room in each table:
 *   - rows seq_row0[s] .. seq_row0[s] + len[s] - 1 of the token axis of K, V and token_ids;
 *   - entries cu_blocks[s] .. cu_blocks[s+1] - 1 of block_start / slot_base and records
 *     cu_blocks[s] .. of every head of ksum / vsum (max_blocks_total records per head), of which
 *     blocks_used[s] blocks are in use; block_start[cu_blocks[s] + blocks_used[s]] = len[s] closes
 *     the table, so a region of n entries holds at most n - 1 blocks.
 * Inside a region the tables are exactly those of a single sequence: block_start counts from the
 * sequence's first token and slot_base from 0.  A region is filled by dsk_compress with B = 1 on
 * the sequence's rows (K + seq_row0[s] * k_stride_tok ...), block_start / slot_base / ksum pointing
 * at entry cu_blocks[s], max_blocks_total = region entries - 1 and sum_stride_blocks = this
 * struct's max_blocks_total; blocks_used[s] is the cu_blocks[1] that call wrote.  dsk_select_topk
 * takes such tables through its blocks_used / seq_row0 fields.
 *
 * Per sequence the update is that of dsk_append_tokens (same finality rule, same result as a
 * from-scratch pass over len_new[s] tokens, bit for bit), with len_old[s] = seq_len[s] on entry;
 * len_new[s] == len_old[s] leaves the sequence as it is.  Data-dependent errors through *dev_status: DSK_ERR_SHAPE if a region's table
 * does not end at len_old[s] or the lengths do not fit (the sequence is then left untouched), DSK_ERR_CAPACITY if the chunks do not fit the region (that
 * sequence's table is then truncated; the others are unaffected).
 * ---------------------------------------------------------------------------------------- */
typedef struct dsk_append_batch_args {
  uint32_t struct_size;
  int32_t B, Hkv, D;
  int32_t total_rows;          /* [host] rows of the token axis of K, V, token_ids */
  int32_t max_new_tokens;      /* [host] upper bound on len_new[s] - len_old[s] (sizes the launch) */
  const int32_t* seq_row0;     /* [dev] [B] */
  int32_t* seq_len;            /* [dev] in/out [B]: the sequences' lengths before the call (len_old), replaced
                                  by the new lengths when the call has updated a sequence */
  const int32_t* len_new;      /* [dev] optional [B]: len_old[s] <= len_new[s] <= len_old[s] + max_new_tokens,
                                  seq_row0[s] + len_new[s] <= total_rows.  NULL: every sequence grows by
                                  max_new_tokens (a decoding batch in lockstep) */
  const void* K;               /* [dev] bf16; strides as in dsk_compress_args */
  const void* V;               /* [dev] may be NULL when vsum is NULL */
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  const int32_t* token_ids;    /* [dev] [total_rows] */
  const int32_t* delim_ids;    /* [dev] [n_class] */
  int32_t n_class;
  const uint8_t* class_weight_q; /* [dev] [B, n_class] tenths */
  int32_t C, delta, alpha_num, alpha_den, b;   /* C, delta: the largest of any sequence */
  const int32_t* C_per_seq;    /* [dev] optional [B] */
  const int32_t* delta_per_seq;/* [dev] optional [B] */
  int32_t max_blocks_total;    /* entries of the tables = records per head of ksum / vsum */
  const int32_t* cu_blocks;    /* [dev] [B+1] region starts, cu_blocks[0] = 0, cu_blocks[B] <= max_blocks_total */
  int32_t* blocks_used;        /* [dev] in/out [B] */
  int32_t* block_start;        /* [dev] in/out [max_blocks_total + 4] */
  int32_t* slot_base;          /* [dev] in/out [max_blocks_total + 4] */
  void* ksum;                  /* [dev] in/out bf16 [Hkv, max_blocks_total, 2, D] */
  void* vsum;                  /* [dev] in/out or NULL */
  int32_t summary_mode;
  int32_t* first_recomputed;   /* [dev] optional out [B]: first rewritten block of each sequence (index in its region) */
  int32_t* first_stale_slot;   /* [dev] optional out [B]: slot_base of that block */
  int32_t* dev_status;         /* [dev] optional */
  void* workspace;             /* [dev] 256-byte aligned, dsk_append_batch_workspace_bytes() */
  size_t workspace_bytes;
} dsk_append_batch_args;

/* ------------------------------------------------------------------------------------------
 * dsk_reuse_update -- KV reuse with the variable-to-fixed slot map (App. B.2, "KVCache Reuse
 * with V2F", Steps 1-3), for a cache whose K/V live in a slower tier (e.g. pinned host memory)
 * while every (sequence, query head) keeps the K/V of its last selection in a resident buffer of
 * k positions of b rows.  Slots being b rows at most, any selected slot fits any position.
 *
 * Per sequence, with the selection of this step (sel_*, as dsk_select_topk writes them):
 *   Step 1  a held slot is reusable when it is selected again (and its index is below
 *           stale_from[s], if given: slots from there on were re-segmented and no longer match
 *           the cache).  r = the smallest reusable count over the heads of the sequence; every
 *           head keeps its first r reusable entries in position order.
 *   Step 2  a head loads every selected slot it does not keep: sel_count - r slots, i.e. k - r
 *           for all heads with a full selection.
 *   Step 3  the loads go, in ascending slot order, to the positions that are not kept, in
 *           ascending position order; positions left over become empty.  Unless
 *           DSK_REUSE_PLAN_ONLY is set the rows are then copied: position p of head h of
 *           sequence s occupies rows (s*k + p)*b .. +b-1 of head h of Kres / Vres; rows past the
 *           slot's length are zero-filled.
 * res_slot must hold -1 (and res_len 0) in every entry before the first call and is carried by
 * the caller from step to step; held slots are distinct (the call keeps them so).  After the
 * call res_start / res_len / res_count describe the buffer as a selection, so that
 * dsk_sparse_decode_attn with K = Kres, V = Vres, Hkv = Hq, k_stride_tok = D, k_stride_head =
 * B*k*b*D, total_tokens = B*k*b, sel_start = res_start, sel_len = res_len, sel_count = res_count
 * attends over exactly the tokens of this step's selection.
 * Three launches; the workspace holds the per-head reusable counts between them.  Spans that leave [0, total_tokens) are
 * not copied (their rows are zero-filled).
 * ---------------------------------------------------------------------------------------- */
#define DSK_REUSE_PLAN_ONLY 1u
#define DSK_REUSE_MAX_K 2048

typedef struct dsk_reuse_args {
  uint32_t struct_size;
  int32_t B, Hq, Hkv, D;
  int32_t k;                   /* positions per (sequence, head) = slots per head in sel_*; <= DSK_REUSE_MAX_K */
  int32_t b;                   /* rows per position; upper bound of sel_len entries */
  uint32_t flags;              /* DSK_REUSE_* bits */
  const int32_t* sel_slot;     /* [dev] [B, Hq, k] ascending global slot indices */
  const int32_t* sel_start;    /* [dev] [B, Hq, k] first global token of the slot */
  const int32_t* sel_len;      /* [dev] [B, Hq, k] tokens in the slot */
  const int32_t* sel_count;    /* [dev] [B, Hq] */
  const int32_t* stale_from;   /* [dev] optional [B]; NULL = every held slot may be reused */
  int32_t* res_slot;           /* [dev] in/out [B, Hq, k] slot held at each position, -1 = empty */
  int32_t* res_len;            /* [dev] in/out [B, Hq, k] its token count, 0 = empty */
  int32_t* res_start;          /* [dev] out [B, Hq, k] first row of the position: (s*k + p)*b */
  int32_t* res_count;          /* [dev] out [B, Hq] 1 + the last position that is not empty */
  int32_t* load_pos;           /* [dev] out [B, Hq, k] position each load goes to; -1 padding */
  int32_t* load_slot;          /* [dev] out [B, Hq, k] slot loaded; -1 padding */
  int32_t* load_start;         /* [dev] out [B, Hq, k] its first global token */
  int32_t* load_len;           /* [dev] out [B, Hq, k] its token count; 0 padding */
  int32_t* load_count;         /* [dev] out [B, Hq] */
  int32_t* reuse_count;        /* [dev] out [B] r of each sequence */
  const void* K;               /* bf16 source, strides as in dsk_compress_args; any address the device */
  const void* V;               /*   can read (HBM or pinned host memory).  Unused with PLAN_ONLY. */
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  int32_t total_tokens;        /* [host] tokens per head in K/V */
  void* Kres;                  /* [dev] bf16 [Hq, B*k*b, D] */
  void* Vres;                  /* [dev] bf16 [Hq, B*k*b, D] */
  void* workspace;             /* [dev] 256-byte aligned, dsk_reuse_workspace_bytes() */
  size_t workspace_bytes;
} dsk_reuse_args;

/* Library / ABI version (DSK_ABI_VERSION of the build). */
uint32_t dsk_version(void);

/* Static, human-readable text for a status code. */
const char* dsk_strerror(dsk_status status);

/* Upper bound on the number of blocks DD-Select can emit for a batch of B sequences with
 * total_tokens tokens when every non-final chunk has at least min_chunk = C - delta tokens
 * (Sec. 4.1): floor(total_tokens / min_chunk) + B.  Returns -1 on bad arguments. */
int64_t dsk_block_capacity(int32_t total_tokens, int32_t B, int32_t min_chunk);

/* Workspace sizes in bytes for the given arguments (0 on invalid geometry). */
size_t dsk_compress_workspace_bytes(const dsk_compress_args* args);
size_t dsk_select_workspace_bytes(const dsk_select_args* args);
size_t dsk_attn_workspace_bytes(const dsk_attn_args* args);
size_t dsk_dense_attn_workspace_bytes(const dsk_dense_attn_args* args);
size_t dsk_append_workspace_bytes(const dsk_append_args* args);
size_t dsk_append_batch_workspace_bytes(const dsk_append_batch_args* args);
size_t dsk_reuse_workspace_bytes(const dsk_reuse_args* args);

/* Where dsk_sparse_decode_attn leaves its split-K partials in args->workspace (what a caller
 * that sets DSK_ATTN_PARTIALS_ONLY reads).  Chunk c of (sequence s, head h) covers the selected
 * slots [c*slots_per_chunk, (c+1)*slots_per_chunk) and is valid for
 * c < ceil(min(sel_count[s,h], k) / slots_per_chunk).  With p = (s*Hq + h)*nchunks + c:
 *   (m, l)  = ((const float*)(workspace + ml_offset))[2p], [2p+1]   running max of the logits in
 *             log2 units (logit * log2(e)), and sum of 2^(logit2 - m)
 *   acc[d]  = ((const float*)(workspace + acc_offset))[p*D + d]      sum of 2^(logit2 - m) * V[d]
 * The merged result is out = sum_c acc_c 2^(m_c - M) / sum_c l_c 2^(m_c - M), M = max_c m_c, and
 * lse = ln(2) * M + ln(sum_c l_c 2^(m_c - M)) (App. B.2 Step 3, online-softmax split).
 * When nchunks == 1 no partials are written: out / lse are final.  Returns DSK_ERR_SHAPE /
 * DSK_ERR_NULL / DSK_ERR_VERSION on unusable arguments (only geometry fields are read). */
typedef struct dsk_attn_partials {
  size_t ml_offset, acc_offset;    /* bytes from args->workspace */
  int32_t nchunks, slots_per_chunk;
} dsk_attn_partials;
dsk_status dsk_attn_partials_layout(const dsk_attn_args* args, dsk_attn_partials* layout);

dsk_status dsk_compress(const dsk_compress_args* args, void* stream);
dsk_status dsk_select_topk(const dsk_select_args* args, void* stream);
dsk_status dsk_sparse_decode_attn(const dsk_attn_args* args, void* stream);
dsk_status dsk_dense_decode_attn(const dsk_dense_attn_args* args, void* stream);

/* dsk_sparse_decode_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as dsk_sparse_decode_attn, except that args->workspace and
 * args->workspace_bytes are ignored: the split-K partials go to a static device array of
 * DSK_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends).
 * The call allocates and frees nothing.
 *   - Size limit: dsk_attn_workspace_bytes(args) must not exceed DSK_STATIC_SCRATCH_BYTES, i.e.
 *     about B * Hq * ceil(k / slots_per_chunk) <= 4000 partials of 520 bytes (configuration 5 of the
 *     benchmark, 8 sequences x 32 heads x 8 chunks, needs 2048); beyond it the call returns
 *     DSK_ERR_WORKSPACE and enqueues nothing.
 *   - Every call on a GPU uses that GPU's one array, and the array keeps the last call's contents.
 *     Nothing in it has to start at zero (a partial is always written before it is read within a
 *     call), so no clearing is enqueued.  Two calls that overlap on one GPU (different streams, or
 *     graphs replayed concurrently) race on the array: serialise them, or use dsk_sparse_decode_attn
 *     with a workspace per stream.
 *   - With DSK_ATTN_PARTIALS_ONLY the partials stay in the library's array, which the caller cannot
 *     address: the flag is accepted but only useful with the workspace variant.
 *   - The array's device address is looked up on the first call on each device (a host-side symbol
 *     query, no allocation); make that first call outside stream capture.  DSK_ERR_LAUNCH if the
 *     lookup or a launch fails. */
#define DSK_STATIC_SCRATCH_BYTES (2112 * 1024)
dsk_status dsk_sparse_decode_attn_static(const dsk_attn_args* args, void* stream);
dsk_status dsk_append_tokens(const dsk_append_args* args, void* stream);
dsk_status dsk_append_tokens_batch(const dsk_append_batch_args* args, void* stream);
dsk_status dsk_reuse_update(const dsk_reuse_args* args, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DSK_H_ */
