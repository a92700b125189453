// Sparsity statistics of the activation masks: the CLS_L sweep of Sec. 2.1 (the curve of
// Fig. 1(a)) and the reuse ratio of Sec. 4.1.2 (Table 4).  Pure integer work on the per-token
// mask words the router wrote; only the closing divisions are fp64.
//
// CLS_L sweep.  A thread owns one start token s and grows the window [s, s + L) one token at a
// time, OR-ing the next token's mask words into a running union, so all lengths 1 .. L_max cost
// L_max ORs and popcounts per start.  Every such window is a sliding window; it is also one of
// the disjoint windows exactly when s is a multiple of L inside its sequence, so both families
// come out of the same pass.  A workgroup stages its 256 tokens plus the L_max - 1 that
// follow in LDS, reduces each length's two counts across the wave with shuffles, collects them in
// LDS and adds them to the global 64-bit counters once per workgroup (integer atomics: exact and
// order-independent).
//
// Reuse ratio.  A thread owns the pair (i, i + 1): card = |S_i|, inter = |S_i & S_{i+1}|.  The
// mean of inter / card is kept exact until the end by accumulating, for each value of card,
// the integer sum of inter and the number of pairs; a last single-thread step adds
// num[c] / c in ascending c and divides by the number of pairs.
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxW = 4;        // mask words per token (N_e <= 256)
constexpr int kMaxLen = 64;     // longest window of the sweep

__device__ __forceinline__ uint64_t word_keep(int E, int wd, int W) {
  return (wd == W - 1 && (E & 63)) ? ((~0ull) >> (64 - (E & 63))) : ~0ull;
}

__global__ __launch_bounds__(kThreads) void zero_i64_kernel(long long *__restrict__ p, int n) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(kThreads) void cls_sweep_kernel(const uint64_t *__restrict__ token_mask, int64_t n_tok,
                                                             int64_t seq_len, int E, int W, int L_max,
                                                             unsigned long long *__restrict__ inactive) {
  __shared__ uint64_t rows[(kThreads + kMaxLen) * kMaxW];
  __shared__ unsigned int block_cnt[2 * kMaxLen];   // [family][L - 1]; at most 256 * 256 per workgroup
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t t0 = (int64_t)blockIdx.x * kThreads;
  const int64_t left = n_tok - t0;
  const int n_rows = left < kThreads + L_max - 1 ? (int)left : kThreads + L_max - 1;
  for (int i = tid; i < n_rows * W; i += kThreads) {
    const int wd = i % W;
    rows[i] = token_mask[t0 * W + i] & word_keep(E, wd, W);
  }
  for (int i = tid; i < 2 * kMaxLen; i += kThreads) block_cnt[i] = 0;
  __syncthreads();

  const int64_t s = t0 + tid;
  const int64_t pos = s < n_tok ? s % seq_len : 0;
  // longest window that starts here and stays inside the sequence (0 beyond the stream's end)
  const int cap = s >= n_tok ? 0 : (seq_len - pos < L_max ? (int)(seq_len - pos) : L_max);
  uint64_t u[kMaxW] = {0, 0, 0, 0};
  for (int L = 1; L <= L_max; ++L) {   // uniform trip count: the shuffles below need every lane
    unsigned int packed = 0;          // low half: sliding count, high half: disjoint count
    if (L <= cap) {
      int active = 0;
#pragma unroll
      for (int wd = 0; wd < kMaxW; ++wd)
        if (wd < W) {
          u[wd] |= rows[(tid + L - 1) * W + wd];
          active += __popcll(u[wd]);
        }
      const unsigned int v = (unsigned int)(E - active);   // <= 256; 64 lanes sum to <= 16384
      packed = v | ((pos % L == 0) ? (v << 16) : 0u);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off, kWave);
    if (lane == 0 && packed) {
      atomicAdd(&block_cnt[kMaxLen + L - 1], packed & 0xffffu);
      atomicAdd(&block_cnt[L - 1], packed >> 16);
    }
  }
  __syncthreads();
  for (int i = tid; i < 2 * kMaxLen; i += kThreads) {
    const int family = i / kMaxLen, l = i % kMaxLen;
    if (l < L_max && block_cnt[i]) atomicAdd(&inactive[family * L_max + l], (unsigned long long)block_cnt[i]);
  }
}

__global__ __launch_bounds__(kThreads) void cls_finish_kernel(const long long *__restrict__ inactive, int64_t n_tok,
                                                              int64_t seq_len, int E, int L_max,
                                                              long long *__restrict__ windows,
                                                              double *__restrict__ cls) {
  const int i = threadIdx.x;
  if (i >= 2 * L_max) return;
  const int family = i / L_max, L = i % L_max + 1;
  const int64_t n_seq = n_tok / seq_len;
  const int64_t per_seq = family == 0 ? seq_len / L : (seq_len >= L ? seq_len - L + 1 : 0);
  const long long w = n_seq * per_seq;
  windows[i] = w;
  cls[i] = w > 0 ? (double)inactive[i] / ((double)w * (double)E) : 0.0;
}

__global__ __launch_bounds__(kThreads) void reuse_kernel(const uint64_t *__restrict__ token_mask, int64_t n_tok,
                                                         int64_t seq_len, int E, int W,
                                                         unsigned long long *__restrict__ num,
                                                         unsigned long long *__restrict__ cnt) {
  __shared__ unsigned int b_num[kMaxExperts + 1], b_cnt[kMaxExperts + 1];   // <= 256 * 256 per workgroup
  const int tid = threadIdx.x;
  for (int i = tid; i <= E; i += kThreads) b_num[i] = b_cnt[i] = 0;
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * kThreads + tid;
  if (i < n_tok && i % seq_len != seq_len - 1) {   // token i has a successor in its sequence
    int card = 0, inter = 0;
    for (int wd = 0; wd < W; ++wd) {
      const uint64_t a = token_mask[i * W + wd] & word_keep(E, wd, W);
      const uint64_t b = token_mask[(i + 1) * W + wd];
      card += __popcll(a);
      inter += __popcll(a & b);
    }
    if (card > 0) {
      atomicAdd(&b_num[card], (unsigned int)inter);
      atomicAdd(&b_cnt[card], 1u);
    }
  }
  __syncthreads();
  for (int c = tid; c <= E; c += kThreads)
    if (b_cnt[c]) {
      atomicAdd(&num[c], (unsigned long long)b_num[c]);
      atomicAdd(&cnt[c], (unsigned long long)b_cnt[c]);
    }
}

__global__ void reuse_finish_kernel(const long long *__restrict__ num, const long long *__restrict__ cnt, int E,
                                    double *__restrict__ ratio) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double total = 0.0;
  long long pairs = 0;
  for (int c = 1; c <= E; ++c) {
    total += (double)num[c] / (double)c;
    pairs += cnt[c];
  }
  ratio[0] = pairs > 0 ? total / (double)pairs : 0.0;
}

}  // namespace

int stats_max_window() { return kMaxLen; }

hipError_t launch_cls_sweep(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int E, int L_max,
                            int64_t *inactive, int64_t *windows, double *cls, hipStream_t s) {
  const int W = (E + 63) / 64;
  const int64_t blocks = (n_tok + kThreads - 1) / kThreads;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(zero_i64_kernel, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<long long *>(inactive),
                     2 * L_max);
  if (blocks > 0)
    hipLaunchKernelGGL(cls_sweep_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, token_mask, n_tok, seq_len, E,
                       W, L_max, reinterpret_cast<unsigned long long *>(inactive));
  hipLaunchKernelGGL(cls_finish_kernel, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<const long long *>(inactive),
                     n_tok, seq_len, E, L_max, reinterpret_cast<long long *>(windows), cls);
  return hipGetLastError();
}

hipError_t launch_reuse_ratio(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int E, int64_t *num,
                              int64_t *cnt, double *ratio, hipStream_t s) {
  const int W = (E + 63) / 64;
  const int64_t blocks = (n_tok + kThreads - 1) / kThreads;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const int zb = (E + 1 + kThreads - 1) / kThreads;
  hipLaunchKernelGGL(zero_i64_kernel, dim3(zb), dim3(kThreads), 0, s, reinterpret_cast<long long *>(num), E + 1);
  hipLaunchKernelGGL(zero_i64_kernel, dim3(zb), dim3(kThreads), 0, s, reinterpret_cast<long long *>(cnt), E + 1);
  if (blocks > 0)
    hipLaunchKernelGGL(reuse_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, token_mask, n_tok, seq_len, E, W,
                       reinterpret_cast<unsigned long long *>(num), reinterpret_cast<unsigned long long *>(cnt));
  hipLaunchKernelGGL(reuse_finish_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<const long long *>(num),
                     reinterpret_cast<const long long *>(cnt), E, ratio);
  return hipGetLastError();
}

}  // namespace blockffn
