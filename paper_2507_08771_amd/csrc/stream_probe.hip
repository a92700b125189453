// Measurement helper, not a step of the layer: a plain read stream over a buffer, the ceiling
// the weight-streaming kernels are compared with.  Every workgroup reads a contiguous tile with
// 128-bit loads, lane-contiguous (a wave's load covers 1 KiB), UNROLL loads in flight per lane,
// and folds what it read into one word so that the loads cannot be dropped.  NT: non-temporal
// loads, which is what the weight streams use (7.1-7.2 TB/s on this chip against 6.3-6.5).
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = 256;

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

template <int UNROLL, bool NT>
__global__ __launch_bounds__(kThreads) void stream_read_kernel(const uint4 *__restrict__ p, size_t tile_vec,
                                                               size_t n_vec, uint32_t *__restrict__ sink) {
  const size_t lo = (size_t)blockIdx.x * tile_vec;
  const size_t hi = lo + tile_vec < n_vec ? lo + tile_vec : n_vec;
  uint32_t acc = 0;
  for (size_t i = lo + threadIdx.x; i < hi; i += (size_t)kThreads * UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t j = i + (size_t)u * kThreads;
      if (j >= hi) {
        v[u] = make_uint4(0, 0, 0, 0);
      } else if (NT) {
        const u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p + j));
        v[u] = make_uint4(w.x, w.y, w.z, w.w);
      } else {
        v[u] = p[j];
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;   // practically never: the sink keeps the loads alive
}

}  // namespace

hipError_t launch_stream_read(const void *buf, size_t bytes, int variant, uint32_t *sink, hipStream_t s) {
  const size_t n_vec = bytes / sizeof(uint4);
  if (n_vec == 0) return hipSuccess;
  // variant: tile per workgroup, loads in flight per lane, plain (0-3) or non-temporal (4-7) loads
  const int shape = variant & 3;
  const size_t tile_bytes = shape == 0 ? (size_t)1 << 20 : (shape == 3 ? (size_t)1 << 16 : (size_t)1 << 18);
  const size_t tile_vec = tile_bytes / sizeof(uint4);
  const size_t blocks = (n_vec + tile_vec - 1) / tile_vec;
  if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
  const uint4 *p = static_cast<const uint4 *>(buf);
  const dim3 grid((unsigned)blocks), block(kThreads);
  const bool deep = shape >= 2;
  if (variant < 4) {
    if (!deep) hipLaunchKernelGGL((stream_read_kernel<8, false>), grid, block, 0, s, p, tile_vec, n_vec, sink);
    else hipLaunchKernelGGL((stream_read_kernel<16, false>), grid, block, 0, s, p, tile_vec, n_vec, sink);
  } else {
    if (!deep) hipLaunchKernelGGL((stream_read_kernel<8, true>), grid, block, 0, s, p, tile_vec, n_vec, sink);
    else hipLaunchKernelGGL((stream_read_kernel<16, true>), grid, block, 0, s, p, tile_vec, n_vec, sink);
  }
  return hipGetLastError();
}

}  // namespace blockffn
