// Router of the BlockFFN layer (Eq. 3): A^0 = W_router^T x + b, A^1 = ReLU(A^0),
// A = RMSNorm(A^1), plus the per-token activation mask (bit set iff A^0 > 0).
//
// One workgroup (4 waves) takes a tile of up to 8 consecutive tokens of one chunk.  Each lane
// keeps its 8 columns of the 8 tokens in registers (64 VGPRs) and walks over all experts: one
// 128-bit load of a W_router row segment feeds 64 fp32 FMAs.  Partial sums of 8 experts x 8
// tokens are reduced across the wave with a 63-step reduce-scatter (lane q ends with entry q),
// the four waves' column quarters are combined in LDS.  Everything is fp32 on the vector ALUs:
// the sign of A^0 decides a mask bit, so no reduced-precision product is used here.
#include "common.hpp"

namespace blockffn {

namespace {

constexpr int kTok = 8;        // tokens per workgroup
constexpr int kThreads = 256;  // 4 waves
constexpr int kColsPerBlock = kThreads * 8;

// v[q] (q = 0..63) summed over the 64 lanes; lane q returns the total of entry q.
// Each step halves the number of live entries: a lane keeps the half selected by one bit of
// its id and receives the partner's copy of the same half.
template <int HALF>
__device__ __forceinline__ void reduce_scatter_step(float (&v)[64], int lane) {
  const bool upper = (lane & HALF) != 0;
#pragma unroll
  for (int i = 0; i < HALF; ++i) {
    const float send = upper ? v[i] : v[i + HALF];
    const float keep = upper ? v[i + HALF] : v[i];
    v[i] = keep + __shfl_xor(send, HALF, kWave);
  }
}

__device__ __forceinline__ float reduce_scatter64(float (&v)[64], int lane) {
  reduce_scatter_step<32>(v, lane);
  reduce_scatter_step<16>(v, lane);
  reduce_scatter_step<8>(v, lane);
  reduce_scatter_step<4>(v, lane);
  reduce_scatter_step<2>(v, lane);
  reduce_scatter_step<1>(v, lane);
  return v[0];
}

// SPLIT = false: one workgroup runs all experts of its token tile and finishes the tokens.
// SPLIT = true (few tokens in the launch): blockIdx.y selects one group of 8 experts; the
// workgroup writes that group's pre-activations A^0 into `scores` and router_finish_kernel
// normalises in place.  Both give the same bits: the summation order of A^0 is the same.
template <typename WT, bool SPLIT>
__global__ __launch_bounds__(kThreads) void router_kernel(LayerView L, const int32_t *__restrict__ chunk_layer,
                                                          const float *__restrict__ x, int k, int tiles_per_chunk,
                                                          float *__restrict__ scores,
                                                          uint64_t *__restrict__ token_mask,
                                                          float *__restrict__ preact) {
  // part[wave][expert][token]
  __shared__ float part[4][kMaxExperts][kTok];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t c = blockIdx.x / tiles_per_chunk;
  const int t0 = (int)(blockIdx.x % tiles_per_chunk) * kTok;
  const int nt = min(kTok, k - t0);
  const int64_t tok0 = c * (int64_t)k + t0;
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int d = L.d, E = L.E;
  const size_t wr_base = (size_t)layer * E * d;
  const int n_groups = (E + 7) / 8;
  const int g_lo = SPLIT ? (int)blockIdx.y : 0, g_hi = SPLIT ? (int)blockIdx.y + 1 : n_groups;

  for (int g = g_lo; g < g_hi; ++g)
    if (lane < 64) part[wave][g * 8 + (lane >> 3)][lane & 7] = 0.0f;   // each lane owns one entry per group

  for (int cb = 0; cb < d; cb += kColsPerBlock) {
    const int col = cb + tid * 8;
    const bool col_ok = col < d;
    float xr[kTok][8];
#pragma unroll
    for (int t = 0; t < kTok; ++t) {
      if (col_ok && t < nt) {
        const float4 *p = reinterpret_cast<const float4 *>(x + (tok0 + t) * d + col);
        const float4 a = p[0], b = p[1];
        xr[t][0] = a.x; xr[t][1] = a.y; xr[t][2] = a.z; xr[t][3] = a.w;
        xr[t][4] = b.x; xr[t][5] = b.y; xr[t][6] = b.z; xr[t][7] = b.w;
      } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) xr[t][q] = 0.0f;
      }
    }
    for (int g = g_lo; g < g_hi; ++g) {
      float v[64];
#pragma unroll
      for (int el = 0; el < 8; ++el) {
        const int i = g * 8 + el;
        float w[8];
        if (col_ok && i < E) {
          load8<WT>(L.w_router, wr_base + (size_t)i * d + col, w);
        } else {
#pragma unroll
          for (int q = 0; q < 8; ++q) w[q] = 0.0f;
        }
#pragma unroll
        for (int t = 0; t < kTok; ++t) {
          float s = 0.0f;
#pragma unroll
          for (int q = 0; q < 8; ++q) s = fmaf(w[q], xr[t][q], s);
          v[el * 8 + t] = s;
        }
      }
      const float tot = reduce_scatter64(v, lane);
      part[wave][g * 8 + (lane >> 3)][lane & 7] += tot;
    }
  }
  __syncthreads();

  if (SPLIT) {
    // thread (el, t) of the first wave writes A^0 of expert g_lo*8 + el, token t
    if (wave == 0) {
      const int i = g_lo * 8 + (lane >> 3), t = lane & 7;
      if (i < E && t < nt) {
        float a0 = L.b_router ? L.b_router[(size_t)layer * E + i] : 0.0f;
        a0 += (part[0][i][t] + part[1][i][t]) + (part[2][i][t] + part[3][i][t]);
        scores[(tok0 + t) * E + i] = a0;
      }
    }
    return;
  }

  // Each wave finishes tokens wave, wave+4: lanes run over experts, one mask word at a time.
  for (int t = wave; t < nt; t += 4) {
    const int64_t tok = tok0 + t;
    float a1[kMaxMaskWords];
    float sumsq = 0.0f;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      a1[wd] = 0.0f;
      if (wd < L.W) {
        const int i = wd * 64 + lane;
        float a0 = 0.0f;
        if (i < E) {
          a0 = L.b_router ? L.b_router[(size_t)layer * E + i] : 0.0f;
          a0 += (part[0][i][t] + part[1][i][t]) + (part[2][i][t] + part[3][i][t]);
        }
        if (preact && i < E) preact[tok * E + i] = a0;
        const bool active = (i < E) && (a0 > 0.0f);
        const uint64_t word = __ballot(active);
        if (lane == 0) token_mask[tok * L.W + wd] = word;
        a1[wd] = active ? a0 : 0.0f;
        sumsq = fmaf(a1[wd], a1[wd], sumsq);
      }
    }
    const float ms = wave_sum(sumsq) / (float)E;
    const float rms = sqrtf(ms + L.eps);
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      if (wd < L.W) {
        const int i = wd * 64 + lane;
        if (i < E) {
          const float g = L.g_rms ? L.g_rms[(size_t)layer * E + i] : 1.0f;
          scores[tok * E + i] = a1[wd] > 0.0f ? g * a1[wd] / rms : 0.0f;
        }
      }
    }
  }
}

// Second half of the split router: one wave per token turns A^0 (in `scores`) into the mask word(s)
// and the RMSNorm'ed scores, in place.
__global__ __launch_bounds__(kThreads) void router_finish_kernel(LayerView L, const int32_t *__restrict__ chunk_layer,
                                                                 int64_t n_tok, int k, float *__restrict__ scores,
                                                                 uint64_t *__restrict__ token_mask,
                                                                 float *__restrict__ preact) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t tok = (int64_t)blockIdx.x * 4 + wave;
  if (tok >= n_tok) return;
  const int E = L.E;
  const int layer = clamp_layer(chunk_layer, tok / k, L.n_layers);
  float a1[kMaxMaskWords];
  float sumsq = 0.0f;
#pragma unroll
  for (int wd = 0; wd < kMaxMaskWords; ++wd) {
    a1[wd] = 0.0f;
    if (wd < L.W) {
      const int i = wd * 64 + lane;
      const float a0 = i < E ? scores[tok * E + i] : 0.0f;
      if (preact && i < E) preact[tok * E + i] = a0;
      const bool active = (i < E) && (a0 > 0.0f);
      const uint64_t word = __ballot(active);
      if (lane == 0) token_mask[tok * L.W + wd] = word;
      a1[wd] = active ? a0 : 0.0f;
      sumsq = fmaf(a1[wd], a1[wd], sumsq);
    }
  }
  const float ms = wave_sum(sumsq) / (float)E;
  const float rms = sqrtf(ms + L.eps);
#pragma unroll
  for (int wd = 0; wd < kMaxMaskWords; ++wd) {
    if (wd < L.W) {
      const int i = wd * 64 + lane;
      if (i < E) {
        const float g = L.g_rms ? L.g_rms[(size_t)layer * E + i] : 1.0f;
        scores[tok * E + i] = a1[wd] > 0.0f ? g * a1[wd] / rms : 0.0f;
      }
    }
  }
}

}  // namespace

hipError_t launch_router(const LayerView &L, int wdtype, const int32_t *chunk_layer, const float *x,
                         int64_t n_chunks, int k, float *scores, uint64_t *token_mask, float *preact,
                         hipStream_t s) {
  const int tiles = (k + kTok - 1) / kTok;
  const int64_t blocks = n_chunks * tiles;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 block(kThreads);
  const int n_groups = (L.E + 7) / 8;
  if (blocks * 2 <= 256 && n_groups > 1) {
    // few token tiles: spread the expert groups over workgroups, then normalise
    dim3 grid((unsigned)blocks, (unsigned)n_groups);
    if (wdtype == BLOCKFFN_BF16)
      hipLaunchKernelGGL((router_kernel<bf16_t, true>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores, token_mask,
                         preact);
    else
      hipLaunchKernelGGL((router_kernel<float, true>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores, token_mask,
                         preact);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t n_tok = n_chunks * k;
    hipLaunchKernelGGL(router_finish_kernel, dim3((unsigned)((n_tok + 3) / 4)), block, 0, s, L, chunk_layer, n_tok, k,
                       scores, token_mask, preact);
    return hipGetLastError();
  }
  dim3 grid((unsigned)blocks);
  if (wdtype == BLOCKFFN_BF16)
    hipLaunchKernelGGL((router_kernel<bf16_t, false>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores, token_mask,
                         preact);
  else
    hipLaunchKernelGGL((router_kernel<float, false>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores, token_mask,
                         preact);
  return hipGetLastError();
}

}  // namespace blockffn
