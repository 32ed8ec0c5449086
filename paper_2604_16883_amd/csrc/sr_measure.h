// Streaming read and copy kernels used to calibrate bandwidth figures and profiler counters.
#ifndef SR_MEASURE_H
#define SR_MEASURE_H

#include "sr_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Measurement helpers.
// ------------------------------------------------------------------------------------------
constexpr int kProbeGrid = 1024;

// Streaming read at the pattern that measured fastest on MI355X: every wavefront reads whole 16 KB
// pieces (16 non-temporal 128-bit loads per lane in flight), pieces dealt round-robin to the wavefronts.
__global__ __launch_bounds__(256) void sr_read_probe_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
  constexpr int U = 16;
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6), nw = (size_t)gridDim.x * 4;
  const size_t piece = (size_t)U * 64;                     // 128-bit words per piece
  uint32_t x = 0;
  size_t c = wave * piece;
  for (; c + piece <= n16; c += nw * piece) {
    uint4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = load_stream(p + c + (size_t)u * 64 + lane);
#pragma unroll
    for (int u = 0; u < U; ++u) x ^= a[u].x ^ a[u].y ^ a[u].z ^ a[u].w;
  }
  // the tail that does not fill a whole round of pieces
  const size_t done = n16 / piece * piece;
  for (size_t i = done + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const uint4 a = p[i];
    x ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x ^= __shfl_xor(x, o, 64);
  __shared__ uint32_t red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

__global__ __launch_bounds__(256) void sr_copy_probe_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

#endif
