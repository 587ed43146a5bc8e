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

__global__ __launch_bounds__(DSK_WAVE) void append_segment_kernel(
    const int32_t* __restrict__ token_ids, const int32_t* __restrict__ delim_ids, int n_class,
    const uint8_t* __restrict__ class_weight_q, int len_old, int len_new, int C, int delta, int a_num,
    int a_den, int b, int cap, int32_t* __restrict__ block_start, int32_t* __restrict__ cu_blocks,
    int32_t* __restrict__ slot_base, int32_t* __restrict__ range, int32_t* __restrict__ first_recomputed,
    int32_t* __restrict__ first_stale_slot, int32_t* dev_status) {
  __shared__ int32_t ids[DSK_MAX_CLASSES];
  __shared__ int32_t wqs[DSK_MAX_CLASSES];
  const int lane = threadIdx.x;
  if (lane < n_class) { ids[lane] = delim_ids[lane]; wqs[lane] = class_weight_q[lane]; }
  __syncthreads();

  int nblk = cu_blocks[1];
  if (nblk < 0) nblk = 0;
  if (nblk > cap) nblk = cap;
  const int table_end = block_start[nblk];
  if (table_end != len_old || block_start[0] != 0) {       // not the table this call was sized for
    if (lane == 0) {
      set_status(dev_status, DSK_ERR_SHAPE);
      range[0] = 0; range[1] = 0;
      if (first_recomputed) *first_recomputed = nblk;
      if (first_stale_slot) *first_stale_slot = 0;         // the table is not trusted: nothing is reusable
    }
    return;
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
    cu_blocks[1] = i;
    range[0] = i0;
    range[1] = i;
    if (first_recomputed) *first_recomputed = i0;
    if (first_stale_slot) *first_stale_slot = stale_slot;
    if (overflow) set_status(dev_status, DSK_ERR_CAPACITY);
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

}  // namespace dsk
