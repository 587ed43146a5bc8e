// C-ABI entry points of libdsk: synchronous argument validation, workspace layout, and the
// launch sequence of each call.  No allocation, no synchronisation, no retained pointers.
#include <hip/hip_runtime.h>

#include <mutex>

#include "dsk_internal.hpp"

namespace dsk {

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

static bool geometry_ok(int B, int Hq, int Hkv, int D) {
  return B >= 1 && Hq >= 1 && Hkv >= 1 && Hq % Hkv == 0 && D == DSK_HEAD_DIM && B <= 65535 && Hq <= 65535;
}

CompressWs compress_ws_layout(const dsk_compress_args& a) {
  CompressWs ws;
  ws.tiles_per_seq = (a.max_seqlen + kSegTile - 1) / kSegTile;
  int span = a.C + a.delta;
  if (span < 1) span = 1;
  ws.map_row = span < kSegTile ? span : kSegTile;
  ws.n_cand_tiles = (a.total_tokens + kCandTile - 1) / kCandTile;
  const size_t n_tiles = (size_t)a.B * ws.tiles_per_seq;
  size_t off = 0;
  ws.tile_map = off;   off += align_up(n_tiles * ws.map_row * sizeof(uint2));
  ws.tile_info = off;  off += align_up(n_tiles * sizeof(int4));
  ws.seq_info = off;   off += align_up((size_t)a.B * sizeof(int4));
  ws.cls_at = off;     off += align_up((size_t)a.total_tokens + 16);
  ws.seg_len = off;    off += align_up(((size_t)a.total_tokens + 16) * sizeof(uint16_t));
  ws.tile_count = off; off += align_up(((size_t)ws.n_cand_tiles + 1) * sizeof(int32_t));
  ws.seg_cand = off;   off += align_up(2 * n_tiles * sizeof(int32_t));
  // levels of the segmentation's pointer doubling kept per token: a tile of kSegTile positions in
  // chunks of at least C - delta; per-sequence C / delta may be smaller than the envelope, so then
  // the chunks may be single positions
  {
    int min_len = (a.C_per_seq != nullptr || a.delta_per_seq != nullptr) ? 1 : a.C - a.delta;
    if (min_len < 1) min_len = 1;
    int hops = (kSegTile + min_len - 1) / min_len, rounds = 0;
    while ((1 << rounds) < hops) ++rounds;
    ws.jump_levels = rounds > 0 ? rounds - 1 : 0;   // the chunk lengths are the first hop, the last level is never hopped from
    ws.jump_stride = (a.total_tokens + 15) / 16 * 16;
  }
  ws.seg_jump = off;   off += align_up((size_t)ws.jump_levels * ws.jump_stride * sizeof(uint16_t) + 32);
  const size_t n_samp = (size_t)a.B * (a.n_class > 0 ? a.n_class : 0) * (a.M > 0 ? a.M : 0);
  ws.imp_part = off;   off += align_up(n_samp * (size_t)a.Hkv * 2 * sizeof(float));
  ws.total = off;
  return ws;
}

static dsk_status validate_compress(const dsk_compress_args* a) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_compress_args)) return DSK_ERR_VERSION;
  if ((a->stages & ~(uint32_t)DSK_STAGE_ALL) != 0 || a->stages == 0) return DSK_ERR_PARAM;
  if (!geometry_ok(a->B, a->Hq, a->Hkv, a->D)) return DSK_ERR_SHAPE;
  if (a->total_tokens < 0 || a->max_seqlen < 0 || a->max_seqlen > a->total_tokens) return DSK_ERR_SHAPE;
  if (a->cu_seqlens == nullptr) return DSK_ERR_NULL;
  const bool st_cand = a->stages & DSK_STAGE_CANDIDATES, st_imp = a->stages & DSK_STAGE_IMPORTANCE;
  const bool st_seg = a->stages & DSK_STAGE_SEGMENT, st_sum = a->stages & DSK_STAGE_SUMMARIES;

  if (st_cand || st_imp || st_seg) {
    if (a->n_class < 1 || a->n_class > DSK_MAX_CLASSES) return DSK_ERR_PARAM;
  }
  // candidates for the segmentation of this call only: no lists, the class map stays in the workspace
  const bool no_lists = st_cand && st_seg && a->cand_pos == nullptr && a->cand_class == nullptr &&
                        a->max_cand_total == 0;
  if (st_cand || st_seg) {
    if (a->max_cand_total < 0) return DSK_ERR_PARAM;
    if (a->cand_cu == nullptr && !no_lists) return DSK_ERR_NULL;
    if (a->max_cand_total > 0 && (a->cand_pos == nullptr || a->cand_class == nullptr)) return DSK_ERR_NULL;
  }
  if (no_lists && (st_imp || (a->samp_pos != nullptr && a->M > 0))) return DSK_ERR_NULL;   // sampling reads the lists
  if (st_cand) {
    if ((a->token_ids == nullptr && a->total_tokens > 0) || a->delim_ids == nullptr) return DSK_ERR_NULL;
    if (a->samp_pos != nullptr && a->M > 0) {
      if (a->M > kMaxSamplesPerClass || a->W < 1 || a->R < 1) return DSK_ERR_PARAM;
    }
  }
  if (st_imp) {
    if (a->samp_pos == nullptr || a->qwin == nullptr || a->class_weight_q == nullptr || a->K == nullptr)
      return DSK_ERR_NULL;
    if (a->M < 1 || a->M > kMaxSamplesPerClass || a->W < 1 || a->W > 64 || a->R < 1) return DSK_ERR_PARAM;
    if (!(a->alpha_imp >= 0.0f) || !(a->alpha_imp <= 1.0e6f) || !(a->imp_scale >= 0.0f)) return DSK_ERR_PARAM;
    if (!aligned16(a->qwin)) return DSK_ERR_ALIGN;
    if (a->samp_score_sum != nullptr && a->imp_layers < 1) return DSK_ERR_PARAM;
  }
  if (st_seg) {
    if (a->class_weight_q == nullptr) return DSK_ERR_NULL;
    if (a->C < 1 || a->delta < 0 || a->delta >= a->C || a->C + a->delta > kMaxChunkSpan) return DSK_ERR_PARAM;
    if (a->alpha_den < 1 || a->alpha_den > 1000 || a->alpha_num < 0 || a->alpha_num > a->alpha_den)
      return DSK_ERR_PARAM;
    if (a->b < 1 || a->b > 1024) return DSK_ERR_PARAM;
  }
  if (st_seg || st_sum) {
    if (a->max_blocks_total < 1) return DSK_ERR_PARAM;
    if (a->block_start == nullptr || a->cu_blocks == nullptr) return DSK_ERR_NULL;
  }
  if (st_seg && a->slot_base == nullptr) return DSK_ERR_NULL;
  if (st_sum) {
    if (a->summary_mode != DSK_SUMMARY_MINMAX && a->summary_mode != DSK_SUMMARY_MEAN) return DSK_ERR_PARAM;
    if (a->sum_stride_blocks != 0 && a->sum_stride_blocks < a->max_blocks_total) return DSK_ERR_PARAM;
    // an empty batch (no token at all) has no K/V row to read: the pointers may then be NULL
    if ((a->K == nullptr && a->total_tokens > 0) || a->ksum == nullptr) return DSK_ERR_NULL;
    if (a->vsum != nullptr && a->V == nullptr && a->total_tokens > 0) return DSK_ERR_NULL;
    if (!aligned16(a->ksum) || (a->vsum && !aligned16(a->vsum))) return DSK_ERR_ALIGN;
  }
  if (st_sum || st_imp) {
    if (!aligned16(a->K) || a->k_stride_tok < DSK_HEAD_DIM || a->k_stride_tok % 8 || a->k_stride_head % 8 ||
        a->k_stride_head < 0)
      return a->k_stride_tok < DSK_HEAD_DIM || a->k_stride_head < 0 ? DSK_ERR_SHAPE : DSK_ERR_ALIGN;
    if (a->Hkv > 1 && a->k_stride_head == 0) return DSK_ERR_SHAPE;
    if (a->k_stride_tok > kMaxTokenStride) return DSK_ERR_SHAPE;
  }
  if (st_sum && a->vsum != nullptr) {
    if (!aligned16(a->V) || a->v_stride_tok % 8 || a->v_stride_head % 8) return DSK_ERR_ALIGN;
    if (a->v_stride_tok < DSK_HEAD_DIM || a->v_stride_head < 0 || a->v_stride_tok > kMaxTokenStride)
      return DSK_ERR_SHAPE;
  }
  const CompressWs ws = compress_ws_layout(*a);
  if (st_cand || st_imp || st_seg) {
    if (a->workspace == nullptr || a->workspace_bytes < ws.total) return DSK_ERR_WORKSPACE;
    if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  }
  return DSK_OK;
}

static dsk_status validate_select(const dsk_select_args* a) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_select_args)) return DSK_ERR_VERSION;
  if (!geometry_ok(a->B, a->Hq, a->Hkv, a->D)) return DSK_ERR_SHAPE;
  if (a->max_blocks_total < 1 || a->max_blocks_used < 0 || a->max_blocks_used > a->max_blocks_total ||
      a->max_blocks_per_seq < 0)
    return DSK_ERR_SHAPE;
  if (a->b < 1 || a->b > 1024 || a->budget < a->b) return DSK_ERR_PARAM;
  if (a->flags & ~(uint32_t)DSK_SELECT_SHARED_BY_KV_GROUP) return DSK_ERR_PARAM;
  if (!a->cu_blocks || !a->block_start || !a->slot_base || !a->ksum || !a->q || !a->sel_slot || !a->sel_start ||
      !a->sel_len || !a->sel_count)
    return DSK_ERR_NULL;
  if (!aligned16(a->ksum) || !aligned16(a->q) || !aligned16(a->slot_base) || !aligned16(a->block_start))
    return DSK_ERR_ALIGN;
  if (a->workspace == nullptr || a->workspace_bytes < dsk_select_workspace_bytes(a)) return DSK_ERR_WORKSPACE;
  if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  return DSK_OK;
}

// own_workspace: the partials go to the library's static scratch array, args->workspace is not used
static dsk_status validate_attn(const dsk_attn_args* a, bool own_workspace = false) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_attn_args)) return DSK_ERR_VERSION;
  if (!geometry_ok(a->B, a->Hq, a->Hkv, a->D)) return DSK_ERR_SHAPE;
  if (a->total_tokens < 0) return DSK_ERR_SHAPE;
  if (a->k < 1 || a->b < 1 || a->b > 1024) return DSK_ERR_PARAM;
  if (!(a->scale >= 0.0f) || (a->flags & ~(uint32_t)(DSK_ATTN_PARTIALS_ONLY | DSK_ATTN_SHARED_SELECTION)))
    return DSK_ERR_PARAM;
  if (!a->q || !a->sel_start || !a->sel_len || !a->sel_count || !a->out) return DSK_ERR_NULL;
  if ((!a->K || !a->V) && a->total_tokens > 0) return DSK_ERR_NULL;   // no token, no row to read
  if (a->k_stride_tok < DSK_HEAD_DIM || a->v_stride_tok < DSK_HEAD_DIM || a->k_stride_head < 0 ||
      a->v_stride_head < 0)
    return DSK_ERR_SHAPE;
  if (!aligned16(a->q) || !aligned16(a->K) || !aligned16(a->V) || a->k_stride_tok % 8 || a->k_stride_head % 8 ||
      a->v_stride_tok % 8 || a->v_stride_head % 8)
    return DSK_ERR_ALIGN;
  if (own_workspace) return DSK_OK;
  if (a->workspace == nullptr || a->workspace_bytes < dsk_attn_workspace_bytes(a)) return DSK_ERR_WORKSPACE;
  if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  return DSK_OK;
}

static dsk_status validate_append(const dsk_append_args* a) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_append_args)) return DSK_ERR_VERSION;
  if (a->Hkv < 1 || a->D != DSK_HEAD_DIM) return DSK_ERR_SHAPE;
  if (a->len_old < 0 || a->len_new < a->len_old) return DSK_ERR_SHAPE;
  if (a->n_class < 1 || a->n_class > DSK_MAX_CLASSES) return DSK_ERR_PARAM;
  if (a->C < 1 || a->delta < 0 || a->delta >= a->C || a->C + a->delta > kMaxChunkSpan) return DSK_ERR_PARAM;
  if (a->alpha_den < 1 || a->alpha_den > 1000 || a->alpha_num < 0 || a->alpha_num > a->alpha_den)
    return DSK_ERR_PARAM;
  if (a->b < 1 || a->b > 1024 || a->max_blocks_total < 1) return DSK_ERR_PARAM;
  if (a->summary_mode != DSK_SUMMARY_MINMAX && a->summary_mode != DSK_SUMMARY_MEAN) return DSK_ERR_PARAM;
  if (!a->K || !a->token_ids || !a->delim_ids || !a->class_weight_q || !a->block_start || !a->cu_blocks ||
      !a->slot_base || !a->ksum)
    return DSK_ERR_NULL;
  if (a->vsum != nullptr && a->V == nullptr) return DSK_ERR_NULL;
  if (a->k_stride_tok < DSK_HEAD_DIM || a->k_stride_head < 0 || a->k_stride_tok > kMaxTokenStride ||
      (a->Hkv > 1 && a->k_stride_head == 0))
    return DSK_ERR_SHAPE;
  if (!aligned16(a->K) || !aligned16(a->ksum) || a->k_stride_tok % 8 || a->k_stride_head % 8) return DSK_ERR_ALIGN;
  if (a->vsum != nullptr) {
    if (a->v_stride_tok < DSK_HEAD_DIM || a->v_stride_head < 0 || a->v_stride_tok > kMaxTokenStride)
      return DSK_ERR_SHAPE;
    if (!aligned16(a->V) || !aligned16(a->vsum) || a->v_stride_tok % 8 || a->v_stride_head % 8) return DSK_ERR_ALIGN;
  }
  if (a->workspace == nullptr || a->workspace_bytes < dsk_append_workspace_bytes(a)) return DSK_ERR_WORKSPACE;
  if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  return DSK_OK;
}

static dsk_status validate_append_batch(const dsk_append_batch_args* a) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_append_batch_args)) return DSK_ERR_VERSION;
  if (a->B < 1 || a->B > 65535 || a->Hkv < 1 || a->Hkv > 65535 * 4 || a->D != DSK_HEAD_DIM) return DSK_ERR_SHAPE;
  if (a->total_rows < 0 || a->max_new_tokens < 0) return DSK_ERR_SHAPE;
  if (a->n_class < 1 || a->n_class > DSK_MAX_CLASSES) return DSK_ERR_PARAM;
  if (a->C < 1 || a->delta < 0 || a->delta >= a->C || a->C + a->delta > kMaxChunkSpan) return DSK_ERR_PARAM;
  if (a->alpha_den < 1 || a->alpha_den > 1000 || a->alpha_num < 0 || a->alpha_num > a->alpha_den)
    return DSK_ERR_PARAM;
  if (a->b < 1 || a->b > 1024 || a->max_blocks_total < 1) return DSK_ERR_PARAM;
  if (a->summary_mode != DSK_SUMMARY_MINMAX && a->summary_mode != DSK_SUMMARY_MEAN) return DSK_ERR_PARAM;
  if (!a->seq_row0 || !a->seq_len || !a->K || !a->token_ids || !a->delim_ids || !a->class_weight_q ||
      !a->cu_blocks || !a->blocks_used || !a->block_start || !a->slot_base || !a->ksum)
    return DSK_ERR_NULL;
  if (a->vsum != nullptr && a->V == nullptr) return DSK_ERR_NULL;
  if (a->k_stride_tok < DSK_HEAD_DIM || a->k_stride_head < 0 || a->k_stride_tok > kMaxTokenStride ||
      (a->Hkv > 1 && a->k_stride_head == 0))
    return DSK_ERR_SHAPE;
  if (!aligned16(a->K) || !aligned16(a->ksum) || a->k_stride_tok % 8 || a->k_stride_head % 8) return DSK_ERR_ALIGN;
  if (a->vsum != nullptr) {
    if (a->v_stride_tok < DSK_HEAD_DIM || a->v_stride_head < 0 || a->v_stride_tok > kMaxTokenStride)
      return DSK_ERR_SHAPE;
    if (!aligned16(a->V) || !aligned16(a->vsum) || a->v_stride_tok % 8 || a->v_stride_head % 8) return DSK_ERR_ALIGN;
  }
  if (a->workspace == nullptr || a->workspace_bytes < dsk_append_batch_workspace_bytes(a)) return DSK_ERR_WORKSPACE;
  if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  return DSK_OK;
}

static dsk_status validate_dense(const dsk_dense_attn_args* a) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_dense_attn_args)) return DSK_ERR_VERSION;
  if (!geometry_ok(a->B, a->Hq, a->Hkv, a->D)) return DSK_ERR_SHAPE;
  if (a->total_tokens < 0 || a->max_seqlen < 0 || (a->max_seqlen == 0 && a->total_tokens > 0)) return DSK_ERR_SHAPE;
  if (!(a->scale >= 0.0f) || a->flags != 0) return DSK_ERR_PARAM;
  if (!a->q || !a->cu_seqlens || !a->out) return DSK_ERR_NULL;
  if ((!a->K || !a->V) && a->total_tokens > 0) return DSK_ERR_NULL;   // no token, no row to read
  if (a->k_stride_tok < DSK_HEAD_DIM || a->v_stride_tok < DSK_HEAD_DIM || a->k_stride_head < 0 ||
      a->v_stride_head < 0)
    return DSK_ERR_SHAPE;
  if (!aligned16(a->q) || !aligned16(a->K) || !aligned16(a->V) || a->k_stride_tok % 8 || a->k_stride_head % 8 ||
      a->v_stride_tok % 8 || a->v_stride_head % 8)
    return DSK_ERR_ALIGN;
  if (a->workspace == nullptr || a->workspace_bytes < dsk_dense_attn_workspace_bytes(a)) return DSK_ERR_WORKSPACE;
  if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  return DSK_OK;
}

static dsk_status validate_reuse(const dsk_reuse_args* a) {
  if (a == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_reuse_args)) return DSK_ERR_VERSION;
  if (!geometry_ok(a->B, a->Hq, a->Hkv, a->D)) return DSK_ERR_SHAPE;
  if (a->k < 1 || a->k > DSK_REUSE_MAX_K || a->b < 1 || a->total_tokens < 0) return DSK_ERR_SHAPE;
  if ((int64_t)a->B * a->k * a->b > 0x7FFFFFFF) return DSK_ERR_SHAPE;   // rows of a resident head are int32
  if (a->flags & ~DSK_REUSE_PLAN_ONLY) return DSK_ERR_PARAM;
  if (!a->sel_slot || !a->sel_start || !a->sel_len || !a->sel_count || !a->res_slot || !a->res_len ||
      !a->res_start || !a->res_count || !a->load_pos || !a->load_slot || !a->load_start || !a->load_len ||
      !a->load_count || !a->reuse_count)
    return DSK_ERR_NULL;
  if (!(a->flags & DSK_REUSE_PLAN_ONLY)) {
    if (!a->K || !a->V || !a->Kres || !a->Vres) return DSK_ERR_NULL;
    if (a->k_stride_tok < DSK_HEAD_DIM || a->v_stride_tok < DSK_HEAD_DIM || a->k_stride_head < 0 ||
        a->v_stride_head < 0)
      return DSK_ERR_SHAPE;
    if (!aligned16(a->K) || !aligned16(a->V) || !aligned16(a->Kres) || !aligned16(a->Vres) || a->k_stride_tok % 8 ||
        a->k_stride_head % 8 || a->v_stride_tok % 8 || a->v_stride_head % 8)
      return DSK_ERR_ALIGN;
  }
  if (a->workspace == nullptr || a->workspace_bytes < dsk_reuse_workspace_bytes(a)) return DSK_ERR_WORKSPACE;
  if (!aligned256(a->workspace)) return DSK_ERR_ALIGN;
  return DSK_OK;
}

// ---- scratch of dsk_sparse_decode_attn_static ------------------------------------------------
// One array per GPU the library runs on, held until the process ends.  Host code never uses the
// array's name as an address: the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[DSK_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device, or nullptr (device index out of range or
// the symbol lookup failed)
static void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace dsk

using namespace dsk;

#pragma GCC visibility push(default)
extern "C" {

uint32_t dsk_version(void) { return DSK_ABI_VERSION; }

const char* dsk_strerror(dsk_status status) {
  switch (status) {
    case DSK_OK: return "ok";
    case DSK_ERR_NULL: return "a required pointer is NULL";
    case DSK_ERR_SHAPE: return "unusable geometry (batch, heads, head_dim, lengths or strides)";
    case DSK_ERR_PARAM: return "parameter out of range";
    case DSK_ERR_ALIGN: return "pointer or stride not sufficiently aligned";
    case DSK_ERR_WORKSPACE: return "workspace missing or too small";
    case DSK_ERR_CAPACITY: return "output capacity exceeded";
    case DSK_ERR_ORDER: return "candidate positions of a sequence are not strictly ascending";
    case DSK_ERR_LAUNCH: return "HIP launch failed";
    case DSK_ERR_VERSION: return "argument struct size does not match this library";
    default: return "unknown status";
  }
}

int64_t dsk_block_capacity(int32_t total_tokens, int32_t B, int32_t min_chunk) {
  if (total_tokens < 0 || B < 1 || min_chunk < 1) return -1;
  return (int64_t)total_tokens / min_chunk + B;
}

size_t dsk_compress_workspace_bytes(const dsk_compress_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_compress_args)) return 0;
  if (a->B < 1 || a->total_tokens < 0 || a->max_seqlen < 0 || a->Hkv < 1) return 0;
  return compress_ws_layout(*a).total;
}

size_t dsk_select_workspace_bytes(const dsk_select_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_select_args)) return 0;
  if (a->Hq < 1 || a->max_blocks_total < 1) return 0;
  return align_up((size_t)a->Hq * select_score_stride(*a) * sizeof(float));
}

size_t dsk_attn_workspace_bytes(const dsk_attn_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_attn_args)) return 0;
  if (a->B < 1 || a->Hq < 1 || a->k < 1) return 0;
  return attn_ws_layout(*a).total;
}

size_t dsk_dense_attn_workspace_bytes(const dsk_dense_attn_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_dense_attn_args)) return 0;
  if (!geometry_ok(a->B, a->Hq, a->Hkv, a->D) || a->max_seqlen < 1) return 0;
  return dense_ws_layout(*a).total;
}

dsk_status dsk_dense_decode_attn(const dsk_dense_attn_args* a, void* stream) {
  const dsk_status v = validate_dense(a);
  if (v != DSK_OK) return v;
  const DenseWs ws = dense_ws_layout(*a);
  if (launch_dense_attn(*a, ws, static_cast<hipStream_t>(stream)) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

size_t dsk_append_workspace_bytes(const dsk_append_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_append_args)) return 0;
  return 256;
}

dsk_status dsk_append_tokens(const dsk_append_args* a, void* stream) {
  const dsk_status v = validate_append(a);
  if (v != DSK_OK) return v;
  if (launch_append(*a, static_cast<hipStream_t>(stream)) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

size_t dsk_append_batch_workspace_bytes(const dsk_append_batch_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_append_batch_args) || a->B < 1) return 0;
  return align_up((size_t)a->B * sizeof(int4));
}

dsk_status dsk_append_tokens_batch(const dsk_append_batch_args* a, void* stream) {
  const dsk_status v = validate_append_batch(a);
  if (v != DSK_OK) return v;
  if (launch_append_batch(*a, static_cast<hipStream_t>(stream)) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

size_t dsk_reuse_workspace_bytes(const dsk_reuse_args* a) {
  if (a == nullptr || a->struct_size != sizeof(dsk_reuse_args) || a->B < 1 || a->Hq < 1) return 0;
  return reuse_ws_bytes(*a);
}

dsk_status dsk_reuse_update(const dsk_reuse_args* a, void* stream) {
  const dsk_status v = validate_reuse(a);
  if (v != DSK_OK) return v;
  if (launch_reuse(*a, static_cast<hipStream_t>(stream)) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

dsk_status dsk_attn_partials_layout(const dsk_attn_args* a, dsk_attn_partials* out) {
  if (a == nullptr || out == nullptr) return DSK_ERR_NULL;
  if (a->struct_size != sizeof(dsk_attn_args)) return DSK_ERR_VERSION;
  if (a->B < 1 || a->Hq < 1 || a->k < 1 || a->b < 1) return DSK_ERR_SHAPE;
  const AttnWs ws = attn_ws_layout(*a);
  out->ml_offset = ws.part_ml;
  out->acc_offset = ws.part_acc;
  out->nchunks = ws.nchunks;
  out->slots_per_chunk = ws.slots_per_wg;
  return DSK_OK;
}

dsk_status dsk_compress(const dsk_compress_args* a, void* stream) {
  const dsk_status v = validate_compress(a);
  if (v != DSK_OK) return v;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const CompressWs ws = compress_ws_layout(*a);
  // candidates wanted only by the segmentation of this call (no lists): nothing to launch for them,
  // the tile kernel classifies the tokens it needs
  const bool st_cand = (a->stages & DSK_STAGE_CANDIDATES) != 0;
  const bool no_lists = st_cand && (a->stages & DSK_STAGE_SEGMENT) && a->cand_pos == nullptr &&
                        a->cand_class == nullptr && a->max_cand_total == 0;
  // lists wanted, and the segmentation of this call does not wait for weights computed from them:
  // the segmentation kernels classify, count and write the lists on their way (three launches less)
  const bool lists_by_segment = st_cand && !no_lists && (a->stages & DSK_STAGE_SEGMENT) &&
                                !(a->stages & DSK_STAGE_IMPORTANCE);
  if (st_cand && !no_lists && !lists_by_segment)
    if (launch_candidates(*a, ws, st) != hipSuccess) return DSK_ERR_LAUNCH;
  if (a->stages & DSK_STAGE_IMPORTANCE)
    if (launch_importance(*a, ws, st) != hipSuccess) return DSK_ERR_LAUNCH;
  if (a->stages & DSK_STAGE_SEGMENT) {
    const SegClassSource src = no_lists ? SegClassSource::kTokenIds
                               : lists_by_segment ? SegClassSource::kTokenIdsWithLists
                               : (st_cand ? SegClassSource::kClassBytes : SegClassSource::kCallerLists);
    if (launch_segment(*a, ws, src, st) != hipSuccess) return DSK_ERR_LAUNCH;
    if (lists_by_segment && launch_cand_sample(*a, st) != hipSuccess) return DSK_ERR_LAUNCH;
  }
  if (a->stages & DSK_STAGE_SUMMARIES)
    if (launch_summaries(*a, st) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

dsk_status dsk_select_topk(const dsk_select_args* a, void* stream) {
  const dsk_status v = validate_select(a);
  if (v != DSK_OK) return v;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* scores = static_cast<float*>(a->workspace);
  const int stride = select_score_stride(*a);
  if (launch_scores(*a, scores, stride, st) != hipSuccess) return DSK_ERR_LAUNCH;
  if (launch_select(*a, scores, stride, st) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

dsk_status dsk_sparse_decode_attn(const dsk_attn_args* a, void* stream) {
  const dsk_status v = validate_attn(a);
  if (v != DSK_OK) return v;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const AttnWs ws = attn_ws_layout(*a);
  if (launch_attn(*a, ws, st) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

dsk_status dsk_sparse_decode_attn_static(const dsk_attn_args* a, void* stream) {
  const dsk_status v = validate_attn(a, /*own_workspace=*/true);
  if (v != DSK_OK) return v;
  const AttnWs ws = attn_ws_layout(*a);
  if (ws.total > (size_t)DSK_STATIC_SCRATCH_BYTES) return DSK_ERR_WORKSPACE;   // more partials than the array holds
  void* ptr = static_scratch_ptr();
  if (ptr == nullptr) return DSK_ERR_LAUNCH;
  dsk_attn_args own = *a;
  own.workspace = ptr;
  own.workspace_bytes = DSK_STATIC_SCRATCH_BYTES;
  if (launch_attn(own, ws, static_cast<hipStream_t>(stream)) != hipSuccess) return DSK_ERR_LAUNCH;
  return DSK_OK;
}

}  // extern "C"
#pragma GCC visibility pop
