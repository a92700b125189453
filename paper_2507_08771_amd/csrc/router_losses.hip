// Forward values of the CLS-aware training objectives on router pre-activations A^0:
// the activation locality loss (Eq. 4) and the chunk sparsification loss (Eq. 5).
//
// Both are means of per-(token or chunk, expert) terms, evaluated in fp64 from the fp32
// pre-activations.  One wave takes one token pair (Eq. 4) or one chunk (Eq. 5) at a time in a
// grid-stride walk, lanes standing for experts, and keeps its running sum in a register; each
// wave then writes one partial and a single workgroup adds the partials in a fixed order, so the
// result does not depend on scheduling (no floating-point atomics).
//
// Eq. 4 term for token t, expert i, with z = alpha * A^0[t, i] and z' = alpha * A^0[t + 1, i]:
//   BCE = sigmoid(z') * softplus(-z) + sigmoid(-z') * softplus(z)
// which is -[q ln p + (1 - q) ln(1 - p)] with the logarithms of the sigmoid written as
// softplus, exact also where p rounds to 0 or 1.
//
// Eq. 5 for one chunk of L tokens: p_ik = ReLU(A^0[k, i]) / sum_i ReLU(A^0[k, i]) (0 for a token
// with no active expert), S_i = sum_k log1p(-p_ik), P_i = -expm1(S_i), term = sum_i P_i.
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kMaxBlocks = 256;                              // partials: one per wave
constexpr int kMaxPartials = kMaxBlocks * kWavesPerBlock;    // 1024

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__device__ __forceinline__ double softplus(double z) { return fmax(z, 0.0) + log1p(exp(-fabs(z))); }
__device__ __forceinline__ double sigmoid(double z) {
  // 1 / (1 + e^-z) without overflow for either sign
  const double e = exp(-fabs(z));
  return z >= 0.0 ? 1.0 / (1.0 + e) : e / (1.0 + e);
}

// partial[wave] = sum of the Eq. 4 terms of the token pairs this wave visited
__global__ __launch_bounds__(kThreads) void locality_kernel(const float *__restrict__ a0, int64_t n_tok,
                                                            int64_t seq_len, int E, double alpha,
                                                            double *__restrict__ partial) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
  double acc = 0.0;
  for (int64_t t = wave; t + 1 < n_tok; t += n_waves) {
    if (t % seq_len == seq_len - 1) continue;   // last token of its sequence: no successor
    for (int i = lane; i < E; i += kWave) {
      const double z = alpha * (double)a0[t * E + i];
      const double zs = alpha * (double)a0[(t + 1) * E + i];
      acc += sigmoid(zs) * softplus(-z) + sigmoid(-zs) * softplus(z);
    }
  }
  acc = wave_sum_f64(acc);
  if (lane == 0) partial[wave] = acc;
}

// partial[wave] = sum over the chunks this wave visited of sum_i P^i_act
__global__ __launch_bounds__(kThreads) void chunk_sparsification_kernel(const float *__restrict__ a0,
                                                                        int64_t n_seq, int64_t seq_len, int E,
                                                                        int L, double *__restrict__ partial) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
  const int64_t per_seq = seq_len / L, n_chunks = n_seq * per_seq;
  double acc = 0.0;
  for (int64_t c = wave; c < n_chunks; c += n_waves) {
    const int64_t first = (c / per_seq) * seq_len + (c % per_seq) * L;   // chunk's first token
    double log_idle[kMaxMaskWords] = {0.0, 0.0, 0.0, 0.0};               // S_i of experts lane + 64 * j
    for (int kk = 0; kk < L; ++kk) {
      const float *row = a0 + (first + kk) * E;
      double a1[kMaxMaskWords];
      double norm = 0.0;
#pragma unroll
      for (int j = 0; j < kMaxMaskWords; ++j) {
        const int i = j * 64 + lane;
        a1[j] = i < E ? fmax((double)row[i], 0.0) : 0.0;
        norm += a1[j];
      }
      norm = wave_sum_f64(norm);   // every lane reaches this: the loop bounds are wave-uniform
      if (norm > 0.0) {
#pragma unroll
        for (int j = 0; j < kMaxMaskWords; ++j) log_idle[j] += log1p(-(a1[j] / norm));
      }
    }
#pragma unroll
    for (int j = 0; j < kMaxMaskWords; ++j)
      if (j * 64 + lane < E) acc += -expm1(log_idle[j]);
  }
  acc = wave_sum_f64(acc);
  if (lane == 0) partial[wave] = acc;
}

// losses[0] = (sum of partial_al) / n_al, losses[1] = (sum of partial_cs) / n_cs; one workgroup,
// pairwise tree over a fixed layout.
__global__ __launch_bounds__(kThreads) void losses_finish_kernel(const double *__restrict__ partial_al, int n_al_parts,
                                                                 double n_al, const double *__restrict__ partial_cs,
                                                                 int n_cs_parts, double n_cs,
                                                                 double *__restrict__ losses) {
  __shared__ double red[2][kThreads];
  const int tid = threadIdx.x;
  double a = 0.0, c = 0.0;
  for (int i = tid; i < n_al_parts; i += kThreads) a += partial_al[i];
  for (int i = tid; i < n_cs_parts; i += kThreads) c += partial_cs[i];
  red[0][tid] = a;
  red[1][tid] = c;
  __syncthreads();
  for (int half = kThreads / 2; half > 0; half >>= 1) {
    if (tid < half) {
      red[0][tid] += red[0][tid + half];
      red[1][tid] += red[1][tid + half];
    }
    __syncthreads();
  }
  if (tid == 0) {
    losses[0] = n_al > 0.0 ? red[0][0] / n_al : 0.0;
    losses[1] = n_cs > 0.0 ? red[1][0] / n_cs : 0.0;
  }
}

}  // namespace

size_t losses_workspace_bytes() { return 2 * (size_t)kMaxPartials * sizeof(double); }

hipError_t launch_router_losses(const float *a0, int64_t n_tok, int64_t seq_len, int E, int L, float alpha,
                                double *losses, void *workspace, hipStream_t s) {
  double *partial_al = static_cast<double *>(workspace);
  double *partial_cs = partial_al + kMaxPartials;
  const int64_t n_seq = n_tok / seq_len;
  const int64_t pairs = n_seq * (seq_len - 1);
  const int64_t chunks = n_seq * (seq_len / L);
  auto blocks_for = [](int64_t units) {
    const int64_t b = (units + kWavesPerBlock - 1) / kWavesPerBlock;
    return (int)(b < 1 ? 0 : (b > kMaxBlocks ? kMaxBlocks : b));
  };
  const int b_al = pairs > 0 ? blocks_for(n_tok) : 0, b_cs = blocks_for(chunks);
  if (b_al > 0)
    hipLaunchKernelGGL(locality_kernel, dim3(b_al), dim3(kThreads), 0, s, a0, n_tok, seq_len, E, (double)alpha,
                       partial_al);
  if (b_cs > 0)
    hipLaunchKernelGGL(chunk_sparsification_kernel, dim3(b_cs), dim3(kThreads), 0, s, a0, n_seq, seq_len, E, L,
                       partial_cs);
  hipLaunchKernelGGL(losses_finish_kernel, dim3(1), dim3(kThreads), 0, s, partial_al, b_al * kWavesPerBlock,
                     (double)pairs * (double)E, partial_cs, b_cs * kWavesPerBlock, (double)chunks * (double)E, losses);
  return hipGetLastError();
}

}  // namespace blockffn
