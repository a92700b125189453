// Union(x) of Sec. 3.3 and the TLS / CLS counts of Sec. 2.1.
//
// One wavefront per chunk.  Lanes first run over the chunk's tokens and OR their mask words
// (a 6-step cross-lane OR gives the union word to every lane); then lane i stands for expert
// 64*word + i: its slot in the compacted list is the number of set bits below it, which is
// what mbcnt of the union word returns, plus the popcount of the earlier words.  The list
// comes out in ascending expert order with no sorting and no atomics.  Only the two 64-bit
// counters are accumulated with integer atomics (order-independent, exact).
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = 256;
constexpr int kChunksPerBlock = kThreads / kWave;

__global__ __launch_bounds__(kThreads) void chunk_union_kernel(const uint64_t *__restrict__ token_mask,
                                                               int64_t n_chunks, int k, int E, int W,
                                                               uint64_t *__restrict__ union_mask,
                                                               int32_t *__restrict__ active_idx,
                                                               int32_t *__restrict__ n_active,
                                                               unsigned long long *__restrict__ stats) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * kChunksPerBlock + wave;
  if (c >= n_chunks) return;   // whole wave leaves together; no barrier below

  int base = 0;
  long long tok_active = 0;   // set bits over the chunk's token masks (this lane's tokens)
  for (int wd = 0; wd < W; ++wd) {
    uint64_t u = 0;
    for (int t = lane; t < k; t += kWave) {
      const uint64_t m = token_mask[(c * k + t) * W + wd];
      u |= m;
      tok_active += __popcll(m);
    }
    u = wave_or(u);
    if (wd == W - 1 && (E & 63)) u &= (~0ull) >> (64 - (E & 63));   // never trust bits at or above E
    if (lane == 0) union_mask[c * W + wd] = u;
    const int i = wd * 64 + lane;
    const bool bit = (u >> lane) & 1;
    const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(u >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)u, 0));
    if (bit && i < E) active_idx[c * E + base + below] = i;
    base += __popcll(u);
  }
  for (int s = base + lane; s < E; s += kWave) active_idx[c * E + s] = -1;
  if (lane == 0) n_active[c] = base;
  if (stats != nullptr) {
    const long long tot_active = wave_sum_i64(tok_active);
    if (lane == 0) {
      atomicAdd(&stats[0], (unsigned long long)((long long)k * E - tot_active));
      atomicAdd(&stats[1], (unsigned long long)(E - base));
    }
  }
}

}  // namespace

hipError_t launch_chunk_union(const uint64_t *token_mask, int64_t n_chunks, int k, int E,
                              uint64_t *union_mask, int32_t *active_idx, int32_t *n_active,
                              int64_t *stats, hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  const int64_t blocks = (n_chunks + kChunksPerBlock - 1) / kChunksPerBlock;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const int W = (E + 63) / 64;
  hipLaunchKernelGGL(chunk_union_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, token_mask, n_chunks, k, E,
                     W, union_mask, active_idx, n_active, reinterpret_cast<unsigned long long *>(stats));
  return hipGetLastError();
}

}  // namespace blockffn
