// Union(x) of Sec. 3.3 and the TLS / CLS counts of Sec. 2.1.
//
// One wavefront per chunk.  Lanes first run over the chunk's tokens and OR their mask words
// (a 6-step cross-lane OR gives the union word to every lane); then lane i stands for expert
// 64*word + i: its slot in the compacted list is the number of set bits below it, which is
// what mbcnt of the union word returns, plus the popcount of the earlier words.  The list
// comes out in ascending expert order with no sorting and no atomics.  Only the two 64-bit
// counters are accumulated with integer atomics (order-independent, exact): a workgroup takes
// 32 chunks and adds its totals once, so the two addresses see one atomic pair per 32 chunks
// (one pair per chunk cost 100 us of serialised atomics at 4096 chunks).
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kChunksPerBlock = 32;   // 8 chunks per wave: one pair of atomics per 32 chunks

__global__ __launch_bounds__(kThreads) void chunk_union_kernel(const uint64_t *__restrict__ token_mask,
                                                               int64_t n_chunks, int k, int E, int W,
                                                               uint64_t *__restrict__ union_mask,
                                                               int32_t *__restrict__ active_idx,
                                                               int32_t *__restrict__ n_active,
                                                               unsigned long long *__restrict__ stats) {
  __shared__ long long block_tok[kWaves], block_chunk[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  long long tok_inactive = 0, chunk_inactive = 0;   // this wave's share of the two counts
  for (int i = wave; i < kChunksPerBlock; i += kWaves) {
    const int64_t c = (int64_t)blockIdx.x * kChunksPerBlock + i;
    if (c >= n_chunks) break;   // uniform over the wave
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
      const int e = wd * 64 + lane;
      const bool bit = (u >> lane) & 1;
      const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(u >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)u, 0));
      if (bit && e < E) active_idx[c * E + base + below] = e;
      base += __popcll(u);
    }
    for (int s = base + lane; s < E; s += kWave) active_idx[c * E + s] = -1;
    if (lane == 0) n_active[c] = base;
    tok_inactive += (long long)k * E - wave_sum_i64(tok_active);
    chunk_inactive += E - base;
  }
  if (stats == nullptr) return;   // uniform over the workgroup: no barrier is skipped by part of it
  if (lane == 0) {
    block_tok[wave] = tok_inactive;
    block_chunk[wave] = chunk_inactive;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long a = 0, b = 0;
    for (int w = 0; w < kWaves; ++w) { a += block_tok[w]; b += block_chunk[w]; }
    atomicAdd(&stats[0], (unsigned long long)a);
    atomicAdd(&stats[1], (unsigned long long)b);
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
