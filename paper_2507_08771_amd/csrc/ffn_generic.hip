// Chunk-sparse expert FFN (Sec. 3.3), shape-generic form.
//
// Two kernels mirror the paper's two-loop structure: the up projection's outer loop and the
// down projection's inner (reduction) loop run over the experts of Union(x) only.
//
//   up    grid (chunk, slot): expert e = active_idx[chunk][slot]; every neuron row of W_up^(e)
//         (and W_gate^(e)) is read once with 128-bit loads and applied to all k tokens of the
//         chunk; Swish / gating, the router score and the token's mask bit are applied before
//         mid[chunk][slot][token][neuron] is written (a masked entry is written as zero).
//   down  grid (chunk, 256 output columns): y[t][col] = sum over slots and neurons of
//         mid * W_down^(e)[col][neuron]; one writer per output element, so no atomics and
//         run-to-run identical results; an empty union writes zeros.
//
// These kernels accept every shape inside the library's limits and both weight dtypes; the
// streaming kernels in ffn_stream.hip take over for the shapes they are specialised for.
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = 256;
constexpr int kTok = 8;

template <typename WT, bool GATED>
__global__ __launch_bounds__(kThreads) void up_generic_kernel(LayerView L, const int32_t *__restrict__ chunk_layer,
                                                              const float *__restrict__ x,
                                                              const float *__restrict__ scores,
                                                              const uint64_t *__restrict__ token_mask,
                                                              const int32_t *__restrict__ active_idx,
                                                              const int32_t *__restrict__ n_active, int k,
                                                              float *__restrict__ mid) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int64_t c = blockIdx.x / E;
  const int s = (int)(blockIdx.x % E);
  int e = s;
  if (active_idx != nullptr) {
    if (s >= n_active[c]) return;
    e = active_idx[c * E + s];
    if (e < 0 || e >= E) return;
  }
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const size_t w_base = ((size_t)layer * E + e) * d_e * d;
  float *mid_cs = mid + ((size_t)c * E + s) * k * d_e;

  for (int t0 = 0; t0 < k; t0 += kTok) {
    const int nt = min(kTok, k - t0);
    for (int j = wave; j < d_e; j += kThreads / kWave) {
      float au[kTok], ag[kTok];
#pragma unroll
      for (int t = 0; t < kTok; ++t) au[t] = ag[t] = 0.0f;
      for (int col = lane * 8; col < d; col += kWave * 8) {
        float wu[8], wg[8];
        load8<WT>(L.w_up, w_base + (size_t)j * d + col, wu);
        if (GATED) load8<WT>(L.w_gate, w_base + (size_t)j * d + col, wg);
#pragma unroll
        for (int t = 0; t < kTok; ++t) {
          if (t < nt) {
            const float4 *p = reinterpret_cast<const float4 *>(x + (c * k + t0 + t) * d + col);
            const float4 a = p[0], b = p[1];
            const float xv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              au[t] = fmaf(wu[q], xv[q], au[t]);
              if (GATED) ag[t] = fmaf(wg[q], xv[q], ag[t]);
            }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < kTok; ++t) {
        au[t] = wave_sum(au[t]);
        if (GATED) ag[t] = wave_sum(ag[t]);
      }
      // lane t finishes token t0 + t
      float u = 0.0f, g = 0.0f;
#pragma unroll
      for (int t = 0; t < kTok; ++t)
        if (lane == t) { u = au[t]; g = ag[t]; }
      if (lane < nt) {
        const int64_t tok = c * k + t0 + lane;
        const float h = GATED ? swish(g) * u : swish(u);
        bool on = true;
        if (token_mask != nullptr) on = (token_mask[tok * L.W + (e >> 6)] >> (e & 63)) & 1;
        const float a = scores[tok * E + e];
        mid_cs[(size_t)(t0 + lane) * d_e + j] = on ? a * h : 0.0f;
      }
    }
  }
}

template <typename WT>
__global__ __launch_bounds__(kThreads) void down_generic_kernel(LayerView L, const int32_t *__restrict__ chunk_layer,
                                                                const int32_t *__restrict__ active_idx,
                                                                const int32_t *__restrict__ n_active, int k,
                                                                int col_tiles, const float *__restrict__ mid,
                                                                float *__restrict__ y) {
  __shared__ float mid_s[kTok][kMaxDe];
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int64_t c = blockIdx.x / col_tiles;
  const int col = (int)(blockIdx.x % col_tiles) * kThreads + threadIdx.x;
  const bool col_ok = col < d;
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  int n_act = E;
  if (active_idx != nullptr) n_act = min(max(n_active[c], 0), E);

  for (int t0 = 0; t0 < k; t0 += kTok) {
    const int nt = min(kTok, k - t0);
    float acc[kTok];
#pragma unroll
    for (int t = 0; t < kTok; ++t) acc[t] = 0.0f;
    for (int s = 0; s < n_act; ++s) {
      int e = s;
      if (active_idx != nullptr) e = active_idx[c * E + s];
      if (e < 0 || e >= E) continue;   // uniform across the workgroup
      const float *mid_cs = mid + ((size_t)c * E + s) * k * d_e + (size_t)t0 * d_e;
      __syncthreads();
      for (int i = threadIdx.x; i < nt * d_e; i += kThreads) mid_s[i / d_e][i % d_e] = mid_cs[i];
      __syncthreads();
      if (col_ok) {
        // one expert's contribution is summed on its own and then added: the rounding error grows
        // with sqrt(d_e) + sqrt(slots) instead of sqrt(d_e * slots)
        float part[kTok];
#pragma unroll
        for (int t = 0; t < kTok; ++t) part[t] = 0.0f;
        const size_t row = (((size_t)layer * E + e) * d + col) * d_e;
        for (int j = 0; j < d_e; j += 8) {
          float w[8];
          load8<WT>(L.w_down, row + j, w);
#pragma unroll
          for (int t = 0; t < kTok; ++t) {
            if (t < nt) {
#pragma unroll
              for (int q = 0; q < 8; ++q) part[t] = fmaf(w[q], mid_s[t][j + q], part[t]);
            }
          }
        }
#pragma unroll
        for (int t = 0; t < kTok; ++t) acc[t] += part[t];
      }
    }
    if (col_ok) {
#pragma unroll
      for (int t = 0; t < kTok; ++t)
        if (t < nt) y[(c * k + t0 + t) * d + col] = acc[t];
    }
  }
}

}  // namespace

hipError_t launch_up_generic(const LayerView &L, int wdtype, bool gated, const int32_t *chunk_layer, const float *x,
                             const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                             const int32_t *n_active, int64_t n_chunks, int k, float *mid, hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  const int64_t up_blocks = n_chunks * L.E;
  if (up_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 block(kThreads);
#define BLOCKFFN_UP(WT, G)                                                                                  \
  hipLaunchKernelGGL((up_generic_kernel<WT, G>), dim3((unsigned)up_blocks), block, 0, s, L, chunk_layer, x, \
                     scores, token_mask, active_idx, n_active, k, mid)
  if (wdtype == BLOCKFFN_BF16) {
    if (gated) BLOCKFFN_UP(bf16_t, true); else BLOCKFFN_UP(bf16_t, false);
  } else {
    if (gated) BLOCKFFN_UP(float, true); else BLOCKFFN_UP(float, false);
  }
#undef BLOCKFFN_UP
  return hipGetLastError();
}

hipError_t launch_down_generic(const LayerView &L, int wdtype, const int32_t *chunk_layer, const int32_t *active_idx,
                               const int32_t *n_active, int64_t n_chunks, int k, const float *mid, float *y,
                               hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  const int col_tiles = (L.d + kThreads - 1) / kThreads;
  const int64_t down_blocks = n_chunks * col_tiles;
  if (down_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 block(kThreads);
  if (wdtype == BLOCKFFN_BF16)
    hipLaunchKernelGGL(down_generic_kernel<bf16_t>, dim3((unsigned)down_blocks), block, 0, s, L, chunk_layer,
                       active_idx, n_active, k, col_tiles, mid, y);
  else
    hipLaunchKernelGGL(down_generic_kernel<float>, dim3((unsigned)down_blocks), block, 0, s, L, chunk_layer,
                       active_idx, n_active, k, col_tiles, mid, y);
  return hipGetLastError();
}

}  // namespace blockffn
