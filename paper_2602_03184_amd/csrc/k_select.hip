// Slot top-k (Sec. 4.2, Block-to-Token Mapping; App. B.2 Step 1) per (sequence, query head).
// Every fixed-length slot inherits the score of its semantic block, so the k best slots are
// found on the block scores with each block weighted by its slot count: an MSB-first radix
// select (4 passes of 8 bits over order-preserving keys, weighted LDS histograms) yields the
// threshold score tau and how many slots of the tau-scored blocks are still needed; two
// workgroup scans then resolve ties by lowest slot index and give every chosen slot its
// position in the ascending output.
#include "dsk_common.hpp"
#include "dsk_internal.hpp"

namespace dsk {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / DSK_WAVE;
constexpr int kSelLdsKeys = 6144;   // blocks of one sequence kept in LDS (48 KB); the rest is re-read from L2

struct SelShared {
  uint32_t keys[kSelLdsKeys];
  uint32_t wts[kSelLdsKeys];
  uint32_t hist[256];
  int wave_tot[kSelWaves];
  uint32_t digit;
  int krem;
};

// exclusive prefix sum of one int per thread over the workgroup, in thread order
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
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wave_tot[w];
    if (w < wave) off += t;
    total += t;
  }
  return off + incl - v;
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ cu_blocks,
    const int32_t* __restrict__ block_start, const int32_t* __restrict__ slot_base, int cap, int Hq,
    int b, int k, int32_t* __restrict__ sel_slot, int32_t* __restrict__ sel_start,
    int32_t* __restrict__ sel_len, int32_t* __restrict__ sel_count) {
  __shared__ SelShared sh;
  const int h = blockIdx.x;
  const int s = blockIdx.y;
  const int tid = threadIdx.x;
  const int64_t obase = ((int64_t)s * Hq + h) * k;
  int blk0 = cu_blocks[s];
  int blk1 = cu_blocks[s + 1];
  if (blk1 > cap) blk1 = cap;
  if (blk0 > blk1) blk0 = blk1;
  const int n = blk1 - blk0;
  const int nslots = n > 0 ? slot_base[blk1] - slot_base[blk0] : 0;
  const int count = nslots < k ? nslots : k;
  if (tid == 0) sel_count[(int64_t)s * Hq + h] = count;
  for (int o = count + tid; o < k; o += kSelThreads) {   // padding
    sel_slot[obase + o] = -1;
    sel_start[obase + o] = 0;
    sel_len[obase + o] = 0;
  }
  if (count <= 0) return;

  const float* sc = scores + (int64_t)h * cap + blk0;
  const int32_t* sb = slot_base + blk0;
  for (int i = tid; i < n && i < kSelLdsKeys; i += kSelThreads) {
    sh.keys[i] = float_key(sc[i]);
    sh.wts[i] = (uint32_t)(sb[i + 1] - sb[i]);
  }
  __syncthreads();
  auto key_of = [&](int i) -> uint32_t { return i < kSelLdsKeys ? sh.keys[i] : float_key(sc[i]); };
  auto wt_of = [&](int i) -> int { return i < kSelLdsKeys ? (int)sh.wts[i] : sb[i + 1] - sb[i]; };

  const bool take_all = nslots <= k;
  uint32_t tau = 0;       // key of the threshold score
  int krem = 0;           // slots still needed from blocks whose key == tau
  if (!take_all) {
    uint32_t prefix = 0, mask = 0;
    krem = k;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      sh.hist[tid] = 0;
      __syncthreads();
      for (int i = tid; i < n; i += kSelThreads) {
        const uint32_t key = key_of(i);
        if ((key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], (uint32_t)wt_of(i));
      }
      __syncthreads();
      // thread t looks at digit 255-t: cumulative slot count from the top digit downwards
      const int v = (int)sh.hist[255 - tid];
      int total;
      const int excl = wg_excl_scan(v, sh.wave_tot, total);
      if (excl < krem && krem <= excl + v) {   // exactly one thread: the digit holding the k-th slot
        sh.digit = (uint32_t)(255 - tid);
        sh.krem = krem - excl;
      }
      __syncthreads();
      prefix |= sh.digit << shift;
      mask |= 255u << shift;
      krem = sh.krem;
      __syncthreads();
    }
    tau = prefix;
  }

  // contiguous range of blocks per thread keeps index order inside the scans
  const int per = (n + kSelThreads - 1) / kSelThreads;
  const int i0 = tid * per < n ? tid * per : n;
  const int i1 = i0 + per < n ? i0 + per : n;

  // scan 1: slots of tau-scored blocks before each thread's range (ties go to the lowest slots)
  int tie_before = 0;
  if (!take_all) {
    int tie_local = 0;
    for (int i = i0; i < i1; ++i) if (key_of(i) == tau) tie_local += wt_of(i);
    int total;
    tie_before = wg_excl_scan(tie_local, sh.wave_tot, total);
  }
  // scan 2: selected slots before each thread's range
  int sel_local = 0;
  {
    int tb = tie_before;
    for (int i = i0; i < i1; ++i) {
      const uint32_t key = key_of(i);
      const int w = wt_of(i);
      int take;
      if (take_all || key > tau) take = w;
      else if (key == tau) { int left = krem - tb; take = left <= 0 ? 0 : (left < w ? left : w); tb += w; }
      else take = 0;
      sel_local += take;
    }
  }
  int total_sel;
  int off = wg_excl_scan(sel_local, sh.wave_tot, total_sel);
  {
    int tb = tie_before;
    for (int i = i0; i < i1; ++i) {
      const uint32_t key = key_of(i);
      const int w = wt_of(i);
      int take;
      if (take_all || key > tau) take = w;
      else if (key == tau) { int left = krem - tb; take = left <= 0 ? 0 : (left < w ? left : w); tb += w; }
      else take = 0;
      if (take > 0) {
        const int bs = block_start[blk0 + i];
        const int be = block_start[blk0 + i + 1];
        const int g0 = sb[i];
        for (int jj = 0; jj < take; ++jj) {
          const int o = off + jj;
          if (o < k) {
            const int st = bs + jj * b;
            const int ln = be - st < b ? be - st : b;
            sel_slot[obase + o] = g0 + jj;
            sel_start[obase + o] = st;
            sel_len[obase + o] = ln > 0 ? ln : 0;
          }
        }
        off += take;
      }
    }
  }
}

hipError_t launch_select(const dsk_select_args& a, const float* scores, hipStream_t st) {
  const int k = a.budget / a.b;
  const dim3 grid((unsigned)a.Hq, (unsigned)a.B);
  select_kernel<<<grid, dim3(kSelThreads), 0, st>>>(scores, a.cu_blocks, a.block_start, a.slot_base,
                                                    a.max_blocks_total, a.Hq, a.b, k, a.sel_slot, a.sel_start,
                                                    a.sel_len, a.sel_count);
  return hipGetLastError();
}

}  // namespace dsk
