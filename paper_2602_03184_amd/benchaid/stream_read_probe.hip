// Streaming-read yardstick for bench.py -- NOT part of libdsk and of no use to the method.
// Every byte of a buffer is read exactly once with 16-byte loads, eight in flight per lane, and
// folded into one word that is (almost) never written.  Timed by the caller, it gives the rate a
// plain coalesced read reaches on the device, the practical ceiling next to which the HBM-bound
// kernels of the library are reported.  Built as its own small shared object
// (libdsk_benchaid.so) that only the benchmark loads.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 8;

__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const uint4* __restrict__ p, size_t n_vec,
                                                                    uint32_t* __restrict__ sink) {
  const size_t tile = (size_t)kProbeThreads * kProbeUnroll;
  const size_t n_tiles = (n_vec + tile - 1) / tile;
  uint32_t acc = 0;
  for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const size_t base = t * tile + threadIdx.x;
    uint4 v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
      const size_t i = base + (size_t)u * kProbeThreads;
      v[u] = p[i < n_vec ? i : n_vec - 1];       // the last tile re-reads the final vector
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  // keeps the loads alive; a buffer would have to be built on purpose to hit the constant
  if (acc == 0x9E3779B9u && sink != nullptr) sink[0] = acc;
}

}  // namespace

// Reads the `bytes` (rounded down to a multiple of 16) at device pointer `buf` (16-byte aligned)
// once on `stream`.  `sink` is a device word (or NULL) that the kernel may write.  Returns 0, or
// -1 for a NULL / misaligned buffer, -2 when the launch fails.
extern "C" __attribute__((visibility("default"))) int dsk_benchaid_stream_read(const void* buf, size_t bytes,
                                                                              void* sink, void* stream) {
  if (buf == nullptr || (reinterpret_cast<uintptr_t>(buf) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return -1;
  const size_t n_vec = bytes / sizeof(uint4);
  if (n_vec == 0) return 0;
  const size_t tile = (size_t)kProbeThreads * kProbeUnroll;
  size_t wgs = (n_vec + tile - 1) / tile;
  if (wgs > 8192) wgs = 8192;                    // 32 workgroups per CU, grid-stride over the rest
  stream_read_kernel<<<dim3((unsigned)wgs), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const uint4*>(buf), n_vec, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
