// Slot top-k (Sec. 4.2, Block-to-Token Mapping; App. B.2 Step 1): one workgroup per
// (sequence, query head).
//
// Every fixed-length slot inherits the score of its semantic block, so the k best slots are
// found on the block scores with each block weighted by its slot count.  Thread t of the 256,
// 512 or 1024 (by the host's bound on the block count) owns PT (4 or 8) consecutive blocks [t*PT, t*PT+PT) of the sequence: their keys (order-preserving
// integer images of the scores) and slot counts live in registers, fetched with 16-byte loads
// that are all in flight at once.
//   1. key range and slot total (workgroup reduction);
//   2. one slot-count-weighted LDS histogram over the top 10 bits of (key - smallest key) finds the
//      bin that holds the k-th best slot; the few blocks of that bin are ranked against each
//      other by one wavefront, which gives the threshold key tau and how many slots of the
//      tau-scored blocks are still needed (8-bit radix passes over the remaining bits only when
//      more than 64 blocks share the bin);
//   3. one workgroup scan over per-thread sums (thread order = block order) resolves ties by
//      lowest slot index and gives every chosen slot its position in the ascending output
//      (block_start was fetched with the scores; the chosen blocks pass through an LDS work
//      list so that all threads write slots in parallel).
// The kernel is a chain of short serial sections (its data is 16 KB per head), so what is
// counted is instructions on that chain: values of the wavefronts are combined with one LDS read
// and a reduction or scan inside a row of 16 lanes rather than a loop over the wavefronts, and the
// bin search is done by all threads at once.  4.7 us per launch at 4076 blocks against 6.4 us for
// four radix passes of 8 bits with a single wavefront choosing each digit.
// Sequences with more blocks than the register tile holds take select_big, the same algorithm
// reading keys from memory.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kSelMaxThreads = 1024;                    // workgroups of 256, 512 or 1024 threads by block count
constexpr int kSelMaxWaves = kSelMaxThreads / DSK_WAVE;
constexpr int kSelMaxPerThread = 8;                     // blocks per thread: 4 or 8 (register tile of 4096 or 8192)
constexpr int kSelWork = 1024;                          // chosen blocks staged in LDS per emission round

// does a sequence of n blocks fit a register tile of `per_thread` blocks per thread whatever
// its alignment shift (0..3)?
__host__ __device__ constexpr bool sel_fits_tile(int n, int per_thread, int threads) {
  return n + 3 <= threads * per_thread;
}

constexpr int kSelBinBits = 10;                         // the histogram pass: 1024 bins over the key range
constexpr int kSelBins = 1 << kSelBinBits;
constexpr int kSelCand = 64;                            // blocks of the threshold bin resolved by one wavefront
static_assert(kSelMaxWaves <= 16, "per-wave values are combined inside one row of 16 lanes");

struct SelShared {
  uint32_t hist[kSelBins];
  int wave_tot[16];                    // per-wave values; entries past the last wave hold the identity
  uint32_t red_min[16], red_max[16];
  int red_sum[16];
  int wave_tot3[3][16];
  uint32_t cand_key[kSelCand];
  int cand_w[kSelCand];
  int n_cand;
  uint32_t tau;
  int digit, krem;
  int4 work[kSelWork];                 // (first token, end token, first slot, output offset)
  int work_take[kSelWork];
};

// ---- combining one value per wavefront over the workgroup (at most 16 wavefronts) ----------------
// Every wavefront stores its value at arr[wave]; after a barrier each lane reads arr[lane & 15]
// and a reduction (or scan) inside its row of 16 lanes, on the vector ALU's data-parallel path,
// gives it the workgroup's result: one LDS read and four lane steps instead of a loop over the waves.
__device__ __forceinline__ uint32_t group16_min_u(uint32_t v) {
  uint32_t o;
  o = (uint32_t)dpp_i<kDppSwap1>((int)v); v = o < v ? o : v;
  o = (uint32_t)dpp_i<kDppSwap2>((int)v); v = o < v ? o : v;
  o = (uint32_t)dpp_i<kDppHalfMirror>((int)v); v = o < v ? o : v;
  o = (uint32_t)dpp_i<kDppMirror>((int)v); v = o < v ? o : v;
  return v;
}
// inclusive prefix sum inside each row of 16 lanes
__device__ __forceinline__ int row16_incl_scan_i(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 1, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 2, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 4, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 8, 0xF, 0xF, false);
  return v;
}
// sum of the entries of the waves before `wave` (wave-uniform), given the row scan of the per-wave totals
__device__ __forceinline__ int waves_before(int row_scan, int wave) {
  return wave == 0 ? 0 : __builtin_amdgcn_readlane(row_scan, wave - 1);
}

// exclusive prefix sum of one int per thread over the workgroup, in thread order
template <int NW>
__device__ __forceinline__ int wg_excl_scan(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = threadIdx.x / DSK_WAVE;
  const int incl = wave_incl_scan_i(v, lane);
  __syncthreads();                       // wave_tot may still be read from a previous scan
  if (lane == DSK_WAVE - 1) wave_tot[wave] = incl;
  __syncthreads();
  int off = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const int t = wave_tot[w];
    if (w < wave) off += t;
    total += t;
  }
  return off + incl - v;
}

// Exclusive prefix sums of three ints per thread over the workgroup, in thread order, and the
// workgroup total of the third.  wave_tot3 entries past the last wave must hold 0.
template <int NW>
__device__ __forceinline__ void wg_excl_scan3(int a, int b, int c, int (*wave_tot3)[16], int& a_excl, int& b_excl,
                                              int& c_excl, int& c_total) {
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DSK_WAVE);
  const int ia = wave_incl_scan_i(a, lane);
  const int ib = wave_incl_scan_i(b, lane);
  const int ic = wave_incl_scan_i(c, lane);
  if (lane == DSK_WAVE - 1) { wave_tot3[0][wave] = ia; wave_tot3[1][wave] = ib; wave_tot3[2][wave] = ic; }
  __syncthreads();
  const int sa = row16_incl_scan_i(wave_tot3[0][lane & 15]);
  const int sb = row16_incl_scan_i(wave_tot3[1][lane & 15]);
  const int sc = row16_incl_scan_i(wave_tot3[2][lane & 15]);
  a_excl = waves_before(sa, wave) + ia - a;
  b_excl = waves_before(sb, wave) + ib - b;
  c_excl = waves_before(sc, wave) + ic - c;
  c_total = __builtin_amdgcn_readlane(sc, NW - 1);
}

// After the histogram of one pass is complete: wave 0 finds the digit holding the krem-th slot
// counted from the top digit down; result broadcast through LDS.
__device__ __forceinline__ void pick_digit(SelShared& sh, int krem, int& digit_out, int& krem_out) {
  if (threadIdx.x < DSK_WAVE) {
    const int lane = threadIdx.x;
    int hv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) hv[u] = (int)sh.hist[255 - 4 * lane - u];
    const int mine = hv[0] + hv[1] + hv[2] + hv[3];
    int excl = wave_incl_scan_i(mine, lane) - mine;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (excl < krem && krem <= excl + hv[u]) {   // true for exactly one (lane, u)
        sh.digit = 255 - 4 * lane - u;
        sh.krem = krem - excl;
      }
      excl += hv[u];
    }
  }
  __syncthreads();
  digit_out = sh.digit;
  krem_out = sh.krem;
}

// The bin of the kSelBins-bin histogram that holds the k-th slot counted from the top bin down,
// found by the whole workgroup: thread t owns the BPT bins below kSelBins - t * BPT, a wavefront
// scan and the row scan of the per-wave totals give the slots in higher bins.  wave_tot entries
// past the last wave must hold 0.  Two barriers.
template <int THREADS>
__device__ __forceinline__ void pick_bin(SelShared& sh, int k, int& bin_out, int& krem_out) {
  constexpr int BPT = kSelBins / THREADS;
  constexpr int kTop = kSelBins - 1;
  const int lane = threadIdx.x & (DSK_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DSK_WAVE);
  int hv[BPT];
  int mine = 0;
#pragma unroll
  for (int u = 0; u < BPT; ++u) { hv[u] = (int)sh.hist[kTop - (threadIdx.x * BPT + u)]; mine += hv[u]; }
  const int incl = wave_incl_scan_i(mine, lane);
  if (lane == DSK_WAVE - 1) sh.wave_tot[wave] = incl;
  __syncthreads();
  int excl = waves_before(row16_incl_scan_i(sh.wave_tot[lane & 15]), wave) + incl - mine;
#pragma unroll
  for (int u = 0; u < BPT; ++u) {
    if (excl < k && k <= excl + hv[u]) {   // true for exactly one (thread, u)
      sh.digit = kTop - (threadIdx.x * BPT + u);
      sh.krem = k - excl;
    }
    excl += hv[u];
  }
  __syncthreads();
  bin_out = sh.digit;
  krem_out = sh.krem;
}

__device__ __forceinline__ void write_padding(int count, int k, int64_t obase, int64_t sh_idx,
                                              int32_t* sel_slot, int32_t* sel_start, int32_t* sel_len,
                                              int32_t* sel_count) {
  if (threadIdx.x == 0) sel_count[sh_idx] = count;
  for (int o = count + threadIdx.x; o < k; o += blockDim.x) {
    sel_slot[obase + o] = -1;
    sel_start[obase + o] = 0;
    sel_len[obase + o] = 0;
  }
}

// Same algorithm for sequences whose blocks do not fit the register tile: keys and slot counts
// are re-read from memory (L2) in every pass; thread t owns a contiguous range of blocks.
template <int THREADS>
__device__ __noinline__ void select_big(
    SelShared& sh, const float* __restrict__ scores, int stride, const int32_t* __restrict__ cu_blocks,
    const int32_t* __restrict__ block_start, const int32_t* __restrict__ slot_base, int cap, int Hq,
    int b, int k, int kcap, int per_thread, int blk1_in, int row0, int32_t* __restrict__ sel_slot,
    int32_t* __restrict__ sel_start, int32_t* __restrict__ sel_len, int32_t* __restrict__ sel_count) {
  const int h = blockIdx.x;
  const int s = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & (DSK_WAVE - 1);
  const int wave = tid / DSK_WAVE;
  const int64_t sh_idx = (int64_t)s * Hq + h;
  const int64_t obase = sh_idx * kcap;   // k slots are taken, the arrays have kcap entries per head
  int blk0 = s == 0 ? 0 : cu_blocks[s];
  blk0 = blk0 < cap ? (blk0 > 0 ? blk0 : 0) : cap;       // same clamping as select_kernel
  const int blk1 = blk1_in;                              // end of the sequence's blocks, as select_kernel found it
  const int n = blk1 - blk0;
  constexpr int NW = THREADS / DSK_WAVE;
  if (n <= 0 || sel_fits_tile(n, per_thread, THREADS)) return;    // not ours
  const float* sc = scores + (int64_t)h * stride + blk0;
  const int32_t* sb = slot_base + blk0;
  const int32_t* bs = block_start + blk0;
  const int per = (n + THREADS - 1) / THREADS;
  const int i0 = tid * per < n ? tid * per : n;
  const int i1 = i0 + per < n ? i0 + per : n;

  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  int nslots = 0;
  for (int i = i0; i < i1; ++i) {
    const uint32_t key = float_key(sc[i]);
    const int wi = sb[i + 1] - sb[i];
    kmin = key < kmin ? key : kmin;
    kmax = key > kmax ? key : kmax;
    nslots += wi > 0 ? wi : 0;
  }
  kmin = wave_min_u(kmin);
  kmax = wave_max_u(kmax);
  nslots = wave_sum_i(nslots);
  if (lane == 0) { sh.red_min[wave] = kmin; sh.red_max[wave] = kmax; sh.red_sum[wave] = nslots; }
  if (tid < 256) sh.hist[tid] = 0;
  __syncthreads();
  nslots = 0;
#pragma unroll
  for (int wv = 0; wv < NW; ++wv) {
    kmin = sh.red_min[wv] < kmin ? sh.red_min[wv] : kmin;
    kmax = sh.red_max[wv] > kmax ? sh.red_max[wv] : kmax;
    nslots += sh.red_sum[wv];
  }
  const int count = nslots < k ? nslots : k;
  write_padding(count, kcap, obase, sh_idx, sel_slot, sel_start, sel_len, sel_count);
  if (count <= 0) return;

  const bool take_all = nslots <= k;
  uint32_t tau = 0u;
  int krem = 0;
  if (!take_all) {
    const uint32_t diff = kmin ^ kmax;
    if (diff == 0) {
      tau = kmax;
      krem = k;
    } else {
      int rbits = 32 - __clz((int)diff);
      uint32_t prefix = rbits >= 32 ? 0u : (kmax >> rbits) << rbits;
      uint32_t mask = rbits >= 32 ? 0u : ~((1u << rbits) - 1u);
      krem = k;
      while (rbits > 0) {
        const int dbits = rbits < 8 ? rbits : 8;
        const int shift_d = rbits - dbits;
        const uint32_t dmask = (1u << dbits) - 1u;
        for (int i = tid; i < n; i += THREADS) {
          const uint32_t key = float_key(sc[i]);
          const int wi = sb[i + 1] - sb[i];
          if (wi > 0 && (key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift_d) & dmask], (uint32_t)wi);
        }
        __syncthreads();
        int digit, knew;
        pick_digit(sh, krem, digit, knew);
        krem = knew;
        prefix |= (uint32_t)digit << shift_d;
        mask |= dmask << shift_d;
        rbits = shift_d;
        if (tid < 256) sh.hist[tid] = 0;
        __syncthreads();
      }
      tau = prefix;
    }
  }
  auto take_of = [&](int i, int& tb) -> int {
    const uint32_t key = float_key(sc[i]);
    int wi = sb[i + 1] - sb[i];
    wi = wi > 0 ? wi : 0;
    if (take_all || key > tau) return wi;
    if (key == tau) {
      const int left = krem - tb;
      tb += wi;
      return left <= 0 ? 0 : (left < wi ? left : wi);
    }
    return 0;
  };
  int tie_before = 0;
  if (!take_all) {
    int tie_local = 0;
    for (int i = i0; i < i1; ++i)
      if (float_key(sc[i]) == tau) { const int wi = sb[i + 1] - sb[i]; tie_local += wi > 0 ? wi : 0; }
    int total;
    tie_before = wg_excl_scan<NW>(tie_local, sh.wave_tot, total);
  }
  int sel_local = 0;
  {
    int tb = tie_before;
    for (int i = i0; i < i1; ++i) sel_local += take_of(i, tb);
  }
  int total_sel;
  int off = wg_excl_scan<NW>(sel_local, sh.wave_tot, total_sel);
  int tb = tie_before;
  for (int i = i0; i < i1; ++i) {
    const int take = take_of(i, tb);
    if (take > 0) {
      const int st0 = bs[i], be = bs[i + 1], g0 = sb[i];
      for (int jj = 0; jj < take; ++jj) {
        const int o = off + jj;
        if (o < k) {
          const int st = st0 + jj * b;
          const int ln = be - st < b ? be - st : b;
          sel_slot[obase + o] = g0 + jj;
          sel_start[obase + o] = st + row0;
          sel_len[obase + o] = ln > 0 ? ln : 0;
        }
      }
      off += take;
    }
  }
}

// scores: rows of `stride` floats (stride % 4 == 0, stride >= cap, base 16-byte aligned);
// slot_base, block_start: 16-byte aligned, readable up to a multiple of 4 entries past cap.
template <int PT, int THREADS>
__global__ __launch_bounds__(THREADS) void select_kernel(
    const float* __restrict__ scores, int stride, const int32_t* __restrict__ cu_blocks,
    const int32_t* __restrict__ block_start, const int32_t* __restrict__ slot_base, int cap, int Hq,
    int b, int kcap, const int32_t* __restrict__ budget_per_seq, const int32_t* __restrict__ blocks_used,
    const int32_t* __restrict__ seq_row0, int32_t* __restrict__ sel_slot, int32_t* __restrict__ sel_start,
    int32_t* __restrict__ sel_len, int32_t* __restrict__ sel_count) {
  static_assert(PT == 4 || PT == 8, "register tile");
  constexpr int NW = THREADS / DSK_WAVE;
  constexpr int kSelPerThread = PT;
  constexpr int kSelVecs = PT / 4;
  __shared__ SelShared sh;
  const int h = blockIdx.x;
  const int s = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & (DSK_WAVE - 1);
  const int wave = tid / DSK_WAVE;
  const int64_t sh_idx = (int64_t)s * Hq + h;
  const int64_t obase = sh_idx * kcap;
  // slots to take: kcap, or this sequence's own budget (clamped to 1..kcap slots)
  int k = kcap;
  if (budget_per_seq != nullptr) {
    int ks = budget_per_seq[s] / b;
    ks = ks < 1 ? 1 : ks;
    k = ks < kcap ? ks : kcap;
  }

  // cu_blocks[0] is 0 by definition: sequence 0 can address its loads before anything arrives
  const int blk0_raw = s == 0 ? 0 : cu_blocks[s];
  const int blk0 = blk0_raw < cap ? (blk0_raw > 0 ? blk0_raw : 0) : cap;
  const int shift = blk0 & 3;                         // same for scores rows (stride % 4 == 0)
  const int v_first = (blk0 - shift) / 4 + tid * kSelVecs;   // thread t owns vectors [v_first, v_first + kSelVecs)
  const int max_vec_sc = stride / 4 - 1;              // clamp to the buffers, mask by index later
  const int max_vec_sb = cap / 4;
  const float4* sc4 = reinterpret_cast<const float4*>(scores + (int64_t)h * stride);
  const int4* sb4 = reinterpret_cast<const int4*>(slot_base);
  const int4* bs4 = reinterpret_cast<const int4*>(block_start);
  float4 fv[kSelVecs];
  int4 iv[kSelVecs + 1], bv[kSelVecs + 1];
#pragma unroll
  for (int u = 0; u < kSelVecs; ++u) {
    const int v = v_first + u;
    fv[u] = sc4[v < max_vec_sc ? v : max_vec_sc];
  }
#pragma unroll
  for (int u = 0; u < kSelVecs + 1; ++u) {
    const int v = v_first + u;
    iv[u] = sb4[v < max_vec_sb ? v : max_vec_sb];
  }
#pragma unroll
  for (int u = 0; u < kSelVecs + 1; ++u) {
    const int v = v_first + u;
    bv[u] = bs4[v < max_vec_sb ? v : max_vec_sb];
  }
  // tables with a region per sequence: the blocks in use and the sequence's first K/V row
  int blk1 = blocks_used != nullptr ? blk0_raw + blocks_used[s] : cu_blocks[s + 1];
  const int row0 = seq_row0 != nullptr ? seq_row0[s] : 0;
#pragma unroll
  for (int u = 0; u < kSelVecs; ++u) pin_loaded(fv[u]);              // all vector loads in flight together
#pragma unroll
  for (int u = 0; u < kSelVecs + 1; ++u) pin_loaded(iv[u]);
#pragma unroll
  for (int u = 0; u < kSelVecs + 1; ++u) pin_loaded(bv[u]);
  if (blk1 > cap) blk1 = cap;
  const int n = blk1 - blk0;
  if (n <= 0) {
    write_padding(0, kcap, obase, sh_idx, sel_slot, sel_start, sel_len, sel_count);
    return;
  }
  if (!sel_fits_tile(n, PT, THREADS)) {                            // too many blocks for the register tile
    select_big<THREADS>(sh, scores, stride, cu_blocks, block_start, slot_base, cap, Hq, b, k, kcap, PT, blk1, row0,
                        sel_slot, sel_start, sel_len, sel_count);
    return;
  }

  // registers: key[r], w[r] of block i = tid*32 + r - shift (w = 0 marks "no block")
  uint32_t key[kSelPerThread];
  int w[kSelPerThread];
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  int nslots = 0;
  {
    const float* f = reinterpret_cast<const float*>(fv);
    const int* x = reinterpret_cast<const int*>(iv);
#pragma unroll
    for (int r = 0; r < kSelPerThread; ++r) {
      const int i = tid * kSelPerThread + r - shift;
      const bool ok = i >= 0 && i < n;
      key[r] = float_key(f[r]);
      int wr = x[r + 1] - x[r];
      wr = (ok && wr > 0) ? wr : 0;                   // malformed table: never count backwards
      w[r] = wr;
      kmin = (ok && key[r] < kmin) ? key[r] : kmin;
      kmax = (ok && key[r] > kmax) ? key[r] : kmax;
      nslots += wr;
    }
  }
  // 1. workgroup reductions: smallest and largest key, slot total
  kmin = wave_min_u(kmin);
  kmax = wave_max_u(kmax);
  nslots = wave_sum_i(nslots);
  if (lane == 0) { sh.red_min[wave] = kmin; sh.red_max[wave] = kmax; sh.red_sum[wave] = nslots; }
  if (tid >= NW && tid < 16) {                           // identities of the waves that do not exist
    sh.red_min[tid] = 0xFFFFFFFFu; sh.red_max[tid] = 0u; sh.red_sum[tid] = 0;
    sh.wave_tot[tid] = 0; sh.wave_tot3[0][tid] = 0; sh.wave_tot3[1][tid] = 0; sh.wave_tot3[2][tid] = 0;
  }
  for (int i = tid; i < kSelBins; i += THREADS) sh.hist[i] = 0;
  if (tid == 0) sh.n_cand = 0;
  __syncthreads();
  kmin = group16_min_u(sh.red_min[lane & 15]);
  kmax = ~group16_min_u(~sh.red_max[lane & 15]);
  nslots = group16_sum_i(sh.red_sum[lane & 15]);
  const int count = nslots < k ? nslots : k;
  write_padding(count, kcap, obase, sh_idx, sel_slot, sel_start, sel_len, sel_count);
  if (count <= 0) return;

  // 2. threshold key tau and krem = slots still needed from the blocks whose key == tau.
  //    One slot-weighted histogram pass over the top kSelBinBits bits of (key - smallest key) finds
  //    the bin that holds the k-th best slot; the bin's few blocks go to an LDS list and one
  //    wavefront ranks them against each other (for every listed key: slots of listed keys above
  //    it, slots of listed keys equal to it), which gives tau and krem exactly.  Only when more
  //    than kSelCand blocks share the bin (clustered or tied scores) do 8-bit radix passes over
  //    the remaining low bits decide.
  const bool take_all = nslots <= k;
  uint32_t tau = 0u;       // take_all: every block qualifies
  int krem = 0;
  if (!take_all) {
    const uint32_t range = kmax - kmin;
    if (range == 0) {      // all scores equal: pure index-order tie
      tau = kmax;
      krem = k;
    } else {
      const int rb = 32 - __clz((int)range);               // bits of key - kmin that can be set
      const int sh_b = rb > kSelBinBits ? rb - kSelBinBits : 0;
#pragma unroll
      for (int r = 0; r < kSelPerThread; ++r)
        if (w[r] != 0) atomicAdd(&sh.hist[(key[r] - kmin) >> sh_b], (uint32_t)w[r]);
      __syncthreads();
      int bin, kbin;
      pick_bin<THREADS>(sh, k, bin, kbin);
#pragma unroll
      for (int r = 0; r < kSelPerThread; ++r) {
        if (w[r] != 0 && (int)((key[r] - kmin) >> sh_b) == bin) {
          const int e = atomicAdd(&sh.n_cand, 1);
          if (e < kSelCand) { sh.cand_key[e] = key[r]; sh.cand_w[e] = w[r]; }
        }
      }
      __syncthreads();
      const int n_cand = __builtin_amdgcn_readfirstlane(sh.n_cand);
      if (n_cand <= kSelCand) {
        if (tid < DSK_WAVE) {
          const bool have = tid < n_cand;
          const uint32_t mykey = have ? sh.cand_key[tid] : 0u;
          const int myw = have ? sh.cand_w[tid] : 0;
          int above = 0, equal = 0;
          for (int jj = 0; jj < n_cand; ++jj) {            // lane jj's entry, through scalar registers
            const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)mykey, jj);
            const int wj = __builtin_amdgcn_readlane(myw, jj);
            above += kj > mykey ? wj : 0;
            equal += kj == mykey ? wj : 0;
          }
          if (have && above < kbin && kbin <= above + equal) {   // lanes holding the same key agree
            sh.tau = mykey;
            sh.krem = kbin - above;
          }
        }
        __syncthreads();
        tau = sh.tau;
        krem = sh.krem;
      } else {
        uint32_t prefix = (uint32_t)bin << sh_b;           // of key - kmin
        uint32_t mask = ~((1u << sh_b) - 1u);              // sh_b >= 1: a bin of one key value has one candidate key
        int rbits = sh_b;
        krem = kbin;
        for (int i = tid; i < 256; i += THREADS) sh.hist[i] = 0;
        __syncthreads();
        while (rbits > 0) {
          const int dbits = rbits < 8 ? rbits : 8;
          const int shift_d = rbits - dbits;
          const uint32_t dmask = (1u << dbits) - 1u;
#pragma unroll
          for (int r = 0; r < kSelPerThread; ++r) {
            const uint32_t nk = key[r] - kmin;
            if (w[r] != 0 && (nk & mask) == prefix) atomicAdd(&sh.hist[(nk >> shift_d) & dmask], (uint32_t)w[r]);
          }
          __syncthreads();
          int digit, knew;
          pick_digit(sh, krem, digit, knew);
          krem = knew;
          prefix |= (uint32_t)digit << shift_d;
          mask |= dmask << shift_d;
          rbits = shift_d;
          if (tid < 256) sh.hist[tid] = 0;                 // everyone has read digit / krem
          __syncthreads();
        }
        tau = kmin + prefix;
      }
    }
  }

  // 3. ties by lowest index, output positions (thread order = block order).  One scan of the
  //    triple (slots of tau-scored blocks, slots of better blocks, blocks of either kind) per
  //    thread: the slots emitted before a thread are  better_before + min(tie_before, krem), and
  //    the block count numbers the entries of the work list below.
  int tie_local = 0, gt_local = 0, cnt_local = 0;
  uint32_t on_mask = 0;                                  // blocks r of this thread that get an entry
#pragma unroll
  for (int r = 0; r < kSelPerThread; ++r) {
    const bool gt = take_all || key[r] > tau;
    const bool tie = !gt && key[r] == tau;
    gt_local += gt ? w[r] : 0;
    tie_local += tie ? w[r] : 0;
    const bool on = (gt || tie) && w[r] != 0;
    cnt_local += on ? 1 : 0;
    on_mask |= on ? (1u << r) : 0u;
  }
  int tie_before, gt_before, e0, n_work;
  wg_excl_scan3<NW>(tie_local, gt_local, cnt_local, sh.wave_tot3, tie_before, gt_before, e0, n_work);
  int off = gt_before + (tie_before < krem ? tie_before : krem);
  // Blocks at or above the threshold go through an LDS work list (every entry carries its output
  // offset and the slots taken from it, 0 for tau-scored blocks past the last needed slot) so that
  // their slots are written by all threads in parallel; block_start is already in registers.
  // Entries outside the current round's window are skipped.
  {
    int tb = tie_before;
#pragma unroll
    for (int r = 0; r < kSelPerThread; ++r) {
      const bool gt = take_all || key[r] > tau;
      int take = gt ? w[r] : 0;
      if (!gt && key[r] == tau) {
        const int left = krem - tb;
        take = left <= 0 ? 0 : (left < w[r] ? left : w[r]);
        tb += w[r];
      }
      w[r] = take;                                       // from here on: slots taken from block r
    }
  }
  const int* xs = reinterpret_cast<const int*>(iv);
  const int* xb = reinterpret_cast<const int*>(bv);
  for (int base = 0; base < n_work; base += kSelWork) {
    int e = e0 - base, o = off;
#pragma unroll
    for (int r = 0; r < kSelPerThread; ++r) {
      const bool on = (on_mask >> r) & 1u;
      if (on && e >= 0 && e < kSelWork) {                  // few lanes per step: masked LDS writes
        sh.work[e] = make_int4(xb[r], xb[r + 1], xs[r], o);
        sh.work_take[e] = w[r];
      }
      e += on ? 1 : 0;
      o += w[r];
    }
    __syncthreads();
    const int n_round = n_work - base < kSelWork ? n_work - base : kSelWork;
    for (int j = tid; j < n_round; j += THREADS) {
      const int4 wk = sh.work[j];
      const int take = sh.work_take[j];
      for (int jj = 0; jj < take; ++jj) {
        const int oo = wk.w + jj;
        if (oo < k) {
          const int st = wk.x + jj * b;
          const int ln = wk.y - st < b ? wk.y - st : b;
          sel_slot[obase + oo] = wk.z + jj;
          sel_start[obase + oo] = st + row0;
          sel_len[obase + oo] = ln > 0 ? ln : 0;
        }
      }
    }
    if (base + kSelWork < n_work) __syncthreads();       // the list is refilled for another round
  }
}

hipError_t launch_select(const dsk_select_args& a, const float* scores, int stride, hipStream_t st) {
  const int k = a.budget / a.b;
  // selecting heads: the query heads, or the KV heads when a group shares its selection
  const int Hsel = (a.flags & DSK_SELECT_SHARED_BY_KV_GROUP) ? a.Hkv : a.Hq;
  const dim3 grid((unsigned)Hsel, (unsigned)a.B);
  // a sequence has at most `bound` blocks: the smallest register tile that holds them all does
  // the least per-thread work (larger sequences than the tile still work, through select_big)
  int bound = a.max_blocks_used > 0 ? a.max_blocks_used : a.max_blocks_total;
  if (a.max_blocks_per_seq > 0 && a.max_blocks_per_seq < bound) bound = a.max_blocks_per_seq;
#define DSK_SEL_ARGS                                                                                          \
  scores, stride, a.cu_blocks, a.block_start, a.slot_base, a.max_blocks_total, Hsel, a.b, k, a.budget_per_seq, a.blocks_used, \
      a.seq_row0, a.sel_slot, a.sel_start, a.sel_len, a.sel_count
  if (sel_fits_tile(bound, 4, 256)) select_kernel<4, 256><<<grid, dim3(256), 0, st>>>(DSK_SEL_ARGS);
  else if (sel_fits_tile(bound, 4, 512)) select_kernel<4, 512><<<grid, dim3(512), 0, st>>>(DSK_SEL_ARGS);
  else if (sel_fits_tile(bound, 4, 1024)) select_kernel<4, 1024><<<grid, dim3(1024), 0, st>>>(DSK_SEL_ARGS);
  else select_kernel<kSelMaxPerThread, kSelMaxThreads><<<grid, dim3(kSelMaxThreads), 0, st>>>(DSK_SEL_ARGS);
#undef DSK_SEL_ARGS
  return hipGetLastError();
}

}  // namespace dsk
