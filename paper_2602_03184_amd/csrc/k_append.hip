// Incremental update during decoding (Sec. 4.1): chunks whose end was decided on a complete
// search range are kept; DD-Select is re-run from the first open chunk over the grown
// sequence.  The open tail is a handful of chunks, so one wavefront walks it: per chunk the
// lanes score the positions of the search range (token id -> delimiter class -> integer score)
// and a wave-wide maximum of packed (score, smaller-e-wins) keys picks the boundary.  The
// summaries of the rewritten chunks are then recomputed by the summaries kernel on that range.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int m = 1; m < DSK_WAVE; m <<= 1) {
    const unsigned long long o = __shfl_xor(v, m, DSK_WAVE);
    v = o > v ? o : v;
  }
  return v;
}

// The update of one sequence by one wavefront.  token_ids, block_start and slot_base point at the
// sequence's own first entry (its tables count from its first token); *n_blocks is its block count
// (in/out); range[0..1] receives the rewritten blocks as indices into the caller's table, i.e.
// offset by blk_base.  Returns false when the table was not the one described (nothing is changed).
__device__ __forceinline__ bool append_segment_one(
    const int32_t* __restrict__ token_ids, const int32_t* __restrict__ delim_ids, int n_class,
    const uint8_t* __restrict__ class_weight_q, int len_old, int len_new, int C, int delta, int a_num,
    int a_den, int b, int cap, int32_t* __restrict__ block_start, int32_t* __restrict__ n_blocks,
    int32_t* __restrict__ slot_base, int blk_base, int32_t* __restrict__ range,
    int32_t* __restrict__ first_recomputed, int32_t* __restrict__ first_stale_slot, int32_t* dev_status) {
  __shared__ int32_t ids[DSK_MAX_CLASSES];
  __shared__ int32_t wqs[DSK_MAX_CLASSES];
  const int lane = threadIdx.x;
  if (lane < n_class) { ids[lane] = delim_ids[lane]; wqs[lane] = class_weight_q[lane]; }
  __syncthreads();

  int nblk = *n_blocks;
  if (nblk < 0) nblk = 0;
  if (nblk > cap) nblk = cap;
  const int table_end = block_start[nblk];
  if (table_end != len_old || block_start[0] != 0) {       // not the table this call was sized for
    if (lane == 0) {
      set_status(dev_status, DSK_ERR_SHAPE);
      range[0] = blk_base; range[1] = blk_base;
      if (first_recomputed) *first_recomputed = nblk;
      if (first_stale_slot) *first_stale_slot = 0;         // the table is not trusted: nothing is reusable
    }
    return false;
  }
  // open chunks form a suffix of the table: count them 64 at a time from the end
  int n_open = 0;
  for (int base = nblk - 1; base >= 0; base -= DSK_WAVE) {
    const int i = base - lane;
    const bool open = i >= 0 && block_start[i] + C + delta > len_old;
    const unsigned long long bal = __ballot(open);
    n_open += __popcll(bal);
    if (bal != ~0ull) break;                               // a final chunk was seen: all before it are final
  }
  const int i0 = nblk - n_open;
  int s_c = i0 < nblk ? block_start[i0] : len_old;
  int slot = slot_base[i0];                                // slot_base[nblk] is the slot total when i0 == nblk
  const int stale_slot = slot;
  int i = i0;
  bool overflow = false;
  const int dd = delta > 1 ? delta : 1;
  while (s_c < len_new) {
    const int s_e = s_c + C;
    int e_star;
    if (s_e >= len_new) {
      e_star = len_new;
    } else {
      const int lo = s_e - delta;                          // > s_c because delta < C
      const int hi = s_e + delta < len_new ? s_e + delta : len_new;
      unsigned long long best = 0ull;                      // 0 = nothing offered
      for (int e = lo + lane; e <= hi; e += DSK_WAVE) {
        const int tok = token_ids[e - 1];                  // the delimiter at e-1 offers the boundary e
        int cls = -1;
        for (int c = n_class - 1; c >= 0; --c) if (tok == ids[c]) cls = c;
        if (cls >= 0) {
          const int dist = e > s_e ? e - s_e : s_e - e;
          const int score = a_num * wqs[cls] * dd + (a_den - a_num) * 10 * (dd - dist);   // >= 0
          const unsigned long long key =
              ((unsigned long long)(unsigned)(score + 1) << 32) | (unsigned)(0x7FFFFFFF - e);   // ties: smaller e
          best = key > best ? key : best;
        }
      }
      best = wave_max_u64(best);
      e_star = best != 0ull ? 0x7FFFFFFF - (int)(unsigned)(best & 0xFFFFFFFFull) : s_e;
    }
    if (i >= cap) { overflow = true; break; }
    slot += (e_star - s_c + b - 1) / b;
    if (lane == 0) { block_start[i + 1] = e_star; slot_base[i + 1] = slot; }
    ++i;
    s_c = e_star;
  }
  if (lane == 0) {
    *n_blocks = i;
    range[0] = blk_base + i0;
    range[1] = blk_base + i;
    if (first_recomputed) *first_recomputed = i0;
    if (first_stale_slot) *first_stale_slot = stale_slot;
    if (overflow) set_status(dev_status, DSK_ERR_CAPACITY);
  }
  return true;
}


__global__ __launch_bounds__(DSK_WAVE) void append_segment_kernel(
    const int32_t* __restrict__ token_ids, const int32_t* __restrict__ delim_ids, int n_class,
    const uint8_t* __restrict__ class_weight_q, int len_old, int len_new, int C, int delta, int a_num,
    int a_den, int b, int cap, int32_t* __restrict__ block_start, int32_t* __restrict__ cu_blocks,
    int32_t* __restrict__ slot_base, int32_t* __restrict__ range, int32_t* __restrict__ first_recomputed,
    int32_t* __restrict__ first_stale_slot, int32_t* dev_status) {
  append_segment_one(token_ids, delim_ids, n_class, class_weight_q, len_old, len_new, C, delta, a_num, a_den, b, cap,
                     block_start, cu_blocks + 1, slot_base, 0, range, first_recomputed, first_stale_slot, dev_status);
}

// ---- all sequences of a batch, each in its own region of the tables ---------------------------
struct AppendBatchParams {
  const int32_t* seq_row0;
  int32_t* seq_len;
  const int32_t* len_new;
  const int32_t* token_ids;
  const int32_t* delim_ids;
  const uint8_t* class_weight_q;
  const int32_t* C_per_seq;
  const int32_t* delta_per_seq;
  const int32_t* cu_blocks;
  int32_t* blocks_used;
  int32_t* block_start;
  int32_t* slot_base;
  int32_t* first_recomputed;
  int32_t* first_stale_slot;
  int32_t* dev_status;
  int n_class, C, delta, a_num, a_den, b, total_rows, max_blocks_total, max_new_tokens;
};

// workspace: int4 per sequence = {first rewritten entry, end of the rewritten entries, first K/V row
// of the sequence, its new length}
__global__ __launch_bounds__(DSK_WAVE) void append_batch_segment_kernel(AppendBatchParams p, int4* __restrict__ ranges) {
  const int s = blockIdx.x;
  const int lane = threadIdx.x;
  const int row0 = p.seq_row0[s];
  const int len_old = p.seq_len[s];
  const int len_new = p.len_new != nullptr ? p.len_new[s] : len_old + p.max_new_tokens;
  const int blk0 = p.cu_blocks[s];
  const int region = p.cu_blocks[s + 1] - blk0;
  int C = p.C_per_seq ? p.C_per_seq[s] : p.C;
  int delta = p.delta_per_seq ? p.delta_per_seq[s] : p.delta;
  bool ok = row0 >= 0 && len_old >= 0 && len_new >= len_old && len_new - len_old <= p.max_new_tokens &&
            (int64_t)row0 + len_new <= p.total_rows && blk0 >= 0 && region >= 1 &&
            (int64_t)blk0 + region <= p.max_blocks_total;
  if (C < 1 || C > p.C || delta < 0 || delta >= C || delta > p.delta) {
    if (lane == 0) set_status(p.dev_status, DSK_ERR_PARAM);
    ok = false;
  } else if (!ok && lane == 0) {
    set_status(p.dev_status, DSK_ERR_SHAPE);
  }
  __shared__ int32_t range[2];
  if (!ok) {                                               // nothing of this sequence is touched
    if (lane == 0) {
      ranges[s] = make_int4(0, 0, 0, 0);
      if (p.first_recomputed) p.first_recomputed[s] = 0;
      if (p.first_stale_slot) p.first_stale_slot[s] = 0;
    }
    return;
  }
  const bool done = append_segment_one(p.token_ids + row0, p.delim_ids, p.n_class, p.class_weight_q + (int64_t)s * p.n_class, len_old,
                     len_new, C, delta, p.a_num, p.a_den, p.b, region - 1, p.block_start + blk0, p.blocks_used + s,
                     p.slot_base + blk0, blk0, range, p.first_recomputed ? p.first_recomputed + s : nullptr,
                     p.first_stale_slot ? p.first_stale_slot + s : nullptr, p.dev_status);
  __syncthreads();
  if (lane == 0) {
    ranges[s] = make_int4(range[0], range[1], row0, len_new);
    if (done) p.seq_len[s] = len_new;
  }
}

hipError_t launch_append(const dsk_append_args& a, hipStream_t st) {
  int32_t* range = static_cast<int32_t*>(a.workspace);
  append_segment_kernel<<<dim3(1), dim3(DSK_WAVE), 0, st>>>(
      a.token_ids, a.delim_ids, a.n_class, a.class_weight_q, a.len_old, a.len_new, a.C, a.delta, a.alpha_num,
      a.alpha_den, a.b, a.max_blocks_total, a.block_start, a.cu_blocks, a.slot_base, range, a.first_recomputed,
      a.first_stale_slot, a.dev_status);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  // chunks that can be rewritten: the open ones start after len_old - C - delta, and every chunk
  // but the last has at least C - delta tokens
  const int64_t span = (int64_t)(a.len_new - a.len_old) + a.C + a.delta;
  int64_t max_changed = span / (a.C - a.delta) + 2;
  if (max_changed > a.max_blocks_total) max_changed = a.max_blocks_total;
  err = launch_summaries_range(a.K, a.k_stride_tok, a.k_stride_head, a.Hkv, a.block_start, range, (int)max_changed,
                               a.max_blocks_total, a.len_new, a.summary_mode, a.ksum, a.dev_status, st);
  if (err != hipSuccess || a.vsum == nullptr) return err;
  return launch_summaries_range(a.V, a.v_stride_tok, a.v_stride_head, a.Hkv, a.block_start, range, (int)max_changed,
                                a.max_blocks_total, a.len_new, a.summary_mode, a.vsum, a.dev_status, st);
}

hipError_t launch_append_batch(const dsk_append_batch_args& a, hipStream_t st) {
  AppendBatchParams p;
  p.seq_row0 = a.seq_row0; p.seq_len = a.seq_len; p.len_new = a.len_new;
  p.token_ids = a.token_ids; p.delim_ids = a.delim_ids; p.class_weight_q = a.class_weight_q;
  p.C_per_seq = a.C_per_seq; p.delta_per_seq = a.delta_per_seq;
  p.cu_blocks = a.cu_blocks; p.blocks_used = a.blocks_used;
  p.block_start = a.block_start; p.slot_base = a.slot_base;
  p.first_recomputed = a.first_recomputed; p.first_stale_slot = a.first_stale_slot;
  p.dev_status = a.dev_status;
  p.n_class = a.n_class; p.C = a.C; p.delta = a.delta; p.a_num = a.alpha_num; p.a_den = a.alpha_den; p.b = a.b;
  p.total_rows = a.total_rows; p.max_blocks_total = a.max_blocks_total; p.max_new_tokens = a.max_new_tokens;
  int4* ranges = static_cast<int4*>(a.workspace);
  append_batch_segment_kernel<<<dim3((unsigned)a.B), dim3(DSK_WAVE), 0, st>>>(p, ranges);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  // chunks of one sequence that can be rewritten: the open ones start after len_old - C - delta,
  // and every chunk but the last has at least one token (C - delta of the sequence's own values,
  // which the host does not know when they are per sequence)
  const int min_len = (a.C_per_seq || a.delta_per_seq) ? 1 : a.C - a.delta;
  const int64_t span = (int64_t)a.max_new_tokens + a.C + a.delta;
  int64_t max_changed = span / min_len + 2;
  if (max_changed > a.max_blocks_total) max_changed = a.max_blocks_total;
  err = launch_summaries_batch_ranges(a.K, a.k_stride_tok, a.k_stride_head, a.Hkv, a.B, a.block_start, ranges,
                                      (int)max_changed, a.max_blocks_total, a.summary_mode, a.ksum, a.dev_status, st);
  if (err != hipSuccess || a.vsum == nullptr) return err;
  return launch_summaries_batch_ranges(a.V, a.v_stride_tok, a.v_stride_head, a.Hkv, a.B, a.block_start, ranges,
                                       (int)max_changed, a.max_blocks_total, a.summary_mode, a.vsum, a.dev_status, st);
}

}  // namespace dsk
