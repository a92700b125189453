// Chunk-sparse expert FFN (Sec. 3.3) for large chunks (33 .. 512 tokens, e.g. a prefill chunk):
// here one expert's weights are reused by hundreds of tokens, the work is a dense grouped
// contraction over the experts of the union and the matrix cores are the bound, not HBM.
//
//   x  -> bf16 once (round to nearest even); products are bf16 x bf16 accumulated in fp32.
//   up    one workgroup = (item of the (chunk, slot) list, 128 tokens, 64 neurons): a
//         128 x 128 x d contraction (64 W_up rows and the 64 matching W_gate rows against 128
//         tokens), both operands staged through double-buffered LDS in MFMA fragment order
//         (global loads use the lane pattern of the operand, so LDS writes and reads are
//         linear in the lane id and conflict free).  Swish/gating, score and mask are applied
//         on the accumulators; mid is written as bf16 [chunk][slot][token][neuron].
//   down  one workgroup = (chunk, 128 output columns, 128 tokens, split): the contraction runs
//         over the slots of the split and the expert's neurons.  When a launch would have too
//         few workgroups to fill the chip the slots are split and the partial sums are added
//         by a second kernel in a fixed order (no atomics; results repeat bit for bit).
//
// As in the paper's kernel every token of the chunk is computed for every expert of the union
// and the sparse pattern of A is applied afterwards.
#include <algorithm>

#include "common.hpp"

namespace blockffn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kTileM = 128;               // weight rows per workgroup
constexpr int kTileN = 128;               // tokens per workgroup
constexpr int kTileK = 64;                // contraction elements per stage (two MFMA K-steps)
constexpr int kStageVec = (kTileM + kTileN) * kTileK * 2 / 16;   // uint4 per stage (2048)
constexpr int kLdsBytes = 2 * kStageVec * 16;                    // two stages, 64 KiB

__device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

__device__ __forceinline__ uint32_t bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}

__global__ __launch_bounds__(kThreads) void cvt_bf16_kernel(const float *__restrict__ x, uint16_t *__restrict__ xb,
                                                            size_t n8) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += (size_t)gridDim.x * kThreads) {
    const float4 a = reinterpret_cast<const float4 *>(x)[2 * i], b = reinterpret_cast<const float4 *>(x)[2 * i + 1];
    uint4 o;
    o.x = bf16_bits(a.x) | bf16_bits(a.y) << 16;
    o.y = bf16_bits(a.z) | bf16_bits(a.w) << 16;
    o.z = bf16_bits(b.x) | bf16_bits(b.y) << 16;
    o.w = bf16_bits(b.z) | bf16_bits(b.w) << 16;
    reinterpret_cast<uint4 *>(xb)[i] = o;
  }
}

// One stage in LDS: fragments [0, 16) are the A operand (8 row fragments x 2 K-steps), [16, 32)
// the B operand (8 token fragments x 2 K-steps); fragment = 64 lanes x 16 bytes.
// Wave w loads fragments [8w, 8w + 8) of every stage.
struct StageRegs {
  uint4 v[8];
};

// Shared main loop.  a_ptr[f] / b_ptr[f] (f = 0..3: the 4 of this wave's 8 fragments that are
// A resp. B ... ) are not used: every wave computes its own 8 source pointers with `src`.
template <typename SrcFn>
__device__ __forceinline__ void gemm_mainloop(uint4 *lds, int n_stages, SrcFn src, f32x4 (&acc)[4][4],
                                              const int (&a_frag)[4], int wc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  StageRegs regs;
  if (n_stages > 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) regs.v[i] = src(0, wave * 8 + i);
#pragma unroll
    for (int i = 0; i < 8; ++i) lds[(wave * 8 + i) * 64 + lane] = regs.v[i];
  }
  __syncthreads();
  for (int st = 0; st < n_stages; ++st) {
    const bool more = st + 1 < n_stages;
    if (more) {
#pragma unroll
      for (int i = 0; i < 8; ++i) regs.v[i] = src(st + 1, wave * 8 + i);
    }
    const uint4 *cur = lds + (st & 1) * kStageVec;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      uint4 a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = cur[(a_frag[i] * 2 + ks) * 64 + lane];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = cur[(16 + (wc * 4 + j) * 2 + ks) * 64 + lane];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mfma16(a[i], b[j], acc[i][j]);
    }
    if (more) {
      uint4 *nxt = lds + ((st + 1) & 1) * kStageVec;
#pragma unroll
      for (int i = 0; i < 8; ++i) nxt[(wave * 8 + i) * 64 + lane] = regs.v[i];
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------ up

template <int NM>
__global__ __launch_bounds__(kThreads, 2) void up_gemm_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const uint16_t *__restrict__ xb,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ items, const int32_t *__restrict__ total_ptr, int k, int tiles_t, int tiles_j,
    uint16_t *__restrict__ H) {
  extern __shared__ uint4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int per_item = tiles_t * tiles_j;
  const int item = blockIdx.x / per_item;
  if (item >= *total_ptr) return;
  const int tt = (blockIdx.x % per_item) / tiles_j, tj = blockIdx.x % tiles_j;
  const int code = items[item];
  const int64_t c = code / E;
  const int s = code - (int)c * E;
  int e = active_idx ? active_idx[c * E + s] : s;
  e = min(max(e, 0), E - 1);
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int t0 = tt * kTileN;
  constexpr int kNeurons = NM == 2 ? 64 : 128;   // neurons per workgroup
  const int j0 = tj * kNeurons;
  const size_t w_expert = ((size_t)layer * E + e) * d_e;
  const int wr = wave & 1, wc = wave >> 1;

  // A fragment fa (0..7): NM == 2: fa < 4 -> W_up rows j0 + 16 fa, else W_gate rows j0 + 16 (fa - 4);
  //                       NM == 1: W_up rows j0 + 16 fa.
  auto src = [&](int st, int id) -> uint4 {
    const int part = id >> 4, frag = (id >> 1) & 7, ks = id & 1;
    const size_t koff = (size_t)st * kTileK + ks * 32 + g * 8;
    if (part == 0) {
      const void *w = (NM == 2 && frag >= 4) ? L.w_gate : L.w_up;
      const int row = j0 + (NM == 2 ? (frag & 3) : frag) * 16 + r;
      return *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(w) + (w_expert + row) * d + koff);
    }
    const int t = t0 + frag * 16 + r;
    if (t >= k) return make_uint4(0, 0, 0, 0);
    return *reinterpret_cast<const uint4 *>(xb + (size_t)(c * k + t) * d + koff);
  };

  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  // this wave's A fragments: NM == 2: up {2wr, 2wr+1} and the matching gate {4+2wr, 5+2wr}
  int a_frag[4];
  if (NM == 2) { a_frag[0] = 2 * wr; a_frag[1] = 2 * wr + 1; a_frag[2] = 4 + 2 * wr; a_frag[3] = 5 + 2 * wr; }
  else { a_frag[0] = 4 * wr; a_frag[1] = 4 * wr + 1; a_frag[2] = 4 * wr + 2; a_frag[3] = 4 * wr + 3; }
  gemm_mainloop(lds, d / kTileK, src, acc, a_frag, wc);

  // D[i = neuron 4g + q of the fragment][j = token n of the fragment]
  const int n = lane & 15;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t = t0 + wc * 64 + j * 16 + n;
    if (t >= k) continue;
    const int64_t tok = c * k + t;
    const bool on = token_mask ? (bool)((token_mask[tok * L.W + (e >> 6)] >> (e & 63)) & 1) : true;
    const float f = scores[tok * E + e];
    constexpr int kOut = NM == 2 ? 2 : 4;
#pragma unroll
    for (int i = 0; i < kOut; ++i) {
      uint32_t p[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float u = acc[i][j][q];
        const float h = NM == 2 ? swish(acc[i + 2][j][q]) * u : swish(u);
        p[q] = bf16_bits(on ? f * h : 0.0f);
      }
      const int neuron = j0 + (NM == 2 ? (2 * wr + i) : (4 * wr + i)) * 16 + 4 * g;
      *reinterpret_cast<uint2 *>(H + (((size_t)c * E + s) * k + t) * d_e + neuron) =
          make_uint2(p[0] | p[1] << 16, p[2] | p[3] << 16);
    }
  }
}

// ------------------------------------------------------------------------------------------------ down

__global__ __launch_bounds__(kThreads, 2) void down_gemm_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int k, int tiles_t, int tiles_c, int splits,
    const uint16_t *__restrict__ H, float *__restrict__ out, size_t split_stride) {
  extern __shared__ uint4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int E = L.E, d = L.d, d_e = L.d_e;
  int b = blockIdx.x;
  const int sp = b % splits; b /= splits;
  const int tc = b % tiles_c; b /= tiles_c;
  const int tt = b % tiles_t;
  const int64_t c = b / tiles_t;
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int n_act = active_idx ? min(max(n_active[c], 0), E) : E;
  const int s_lo = (int)((int64_t)n_act * sp / splits), s_hi = (int)((int64_t)n_act * (sp + 1) / splits);
  const int t0 = tt * kTileN, col0 = tc * kTileM;
  const int wr = wave & 1, wc = wave >> 1;
  const int st_per_slot = d_e / kTileK;

  auto src = [&](int st, int id) -> uint4 {
    const int part = id >> 4, frag = (id >> 1) & 7, ks = id & 1;
    const int s = s_lo + st / st_per_slot;
    const size_t koff = (size_t)(st % st_per_slot) * kTileK + ks * 32 + g * 8;
    if (part == 0) {
      int e = active_idx ? active_idx[c * E + s] : s;
      e = min(max(e, 0), E - 1);
      const size_t row = ((size_t)layer * E + e) * d + col0 + frag * 16 + r;
      return *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(L.w_down) + row * d_e + koff);
    }
    const int t = t0 + frag * 16 + r;
    if (t >= k) return make_uint4(0, 0, 0, 0);
    return *reinterpret_cast<const uint4 *>(H + (((size_t)c * E + s) * k + t) * d_e + koff);
  };

  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int a_frag[4] = {4 * wr, 4 * wr + 1, 4 * wr + 2, 4 * wr + 3};
  gemm_mainloop(lds, (s_hi - s_lo) * st_per_slot, src, acc, a_frag, wc);

  const int n = lane & 15;
  float *dst = out + (size_t)sp * split_stride;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t = t0 + wc * 64 + j * 16 + n;
    if (t >= k) continue;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int col = col0 + (4 * wr + i) * 16 + 4 * g;
      *reinterpret_cast<float4 *>(dst + (size_t)(c * k + t) * d + col) =
          make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
    }
  }
}

__global__ __launch_bounds__(kThreads) void reduce_splits_kernel(const float *__restrict__ part, int splits,
                                                                 size_t split_stride, size_t n4,
                                                                 float *__restrict__ y) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    float4 a = reinterpret_cast<const float4 *>(part)[i];
    for (int sp = 1; sp < splits; ++sp) {
      const float4 b = reinterpret_cast<const float4 *>(part + (size_t)sp * split_stride)[i];
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    reinterpret_cast<float4 *>(y)[i] = a;
  }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int down_splits(const LayerView &L, int64_t n_chunks, int k) {
  const int64_t base = n_chunks * ((k + kTileN - 1) / kTileN) * (L.d / kTileM);
  if (base >= 512) return 1;
  return (int)std::min<int64_t>(8, (512 + base - 1) / base);
}

struct GemmWs {
  uint16_t *xb, *H;
  int32_t *total, *items;
  float *part;
};

GemmWs carve(const LayerView &L, int64_t n_chunks, int k, void *ws) {
  char *p = static_cast<char *>(ws);
  GemmWs w;
  w.xb = reinterpret_cast<uint16_t *>(p);
  p += align256((size_t)n_chunks * k * L.d * 2);
  w.H = reinterpret_cast<uint16_t *>(p);
  p += align256((size_t)n_chunks * L.E * k * L.d_e * 2);
  w.total = reinterpret_cast<int32_t *>(p);
  w.items = w.total + 64;
  p += align256(((size_t)n_chunks * L.E + 64) * sizeof(int32_t));
  w.part = reinterpret_cast<float *>(p);
  return w;
}

}  // namespace

bool gemm_supported(const LayerView &L, int wdtype, int k, bool gated) {
  return wdtype == BLOCKFFN_BF16 && k > 32 && L.d % 128 == 0 && L.d_e % (gated ? 64 : 128) == 0;
}

size_t gemm_workspace_bytes(const LayerView &L, int64_t n_chunks, int k) {
  const int splits = down_splits(L, n_chunks, k);
  size_t b = align256((size_t)n_chunks * k * L.d * 2) + align256((size_t)n_chunks * L.E * k * L.d_e * 2) +
             align256(((size_t)n_chunks * L.E + 64) * sizeof(int32_t));
  if (splits > 1) b += align256((size_t)splits * n_chunks * k * L.d * sizeof(float));
  return b;
}

hipError_t launch_up_gemm(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                          const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                          const int32_t *n_active, int64_t n_chunks, int k, void *ws, hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  GemmWs w = carve(L, n_chunks, k, ws);
  const size_t n8 = (size_t)n_chunks * k * L.d / 8;
  hipLaunchKernelGGL(cvt_bf16_kernel, dim3((unsigned)std::min<size_t>((n8 + kThreads - 1) / kThreads, 4096)),
                     dim3(kThreads), 0, s, x, w.xb, n8);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  err = launch_worklist(n_active, n_chunks, L.E, w.items, w.total, s);
  if (err != hipSuccess) return err;
  const int tiles_t = (k + kTileN - 1) / kTileN, tiles_j = L.d_e / (gated ? 64 : 128);
  const int64_t grid = n_chunks * L.E * tiles_t * tiles_j;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void *>(up_gemm_kernel<1>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void *>(up_gemm_kernel<2>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e1 != hipSuccess || e2 != hipSuccess) return e1 != hipSuccess ? e1 : e2;
    attr_set = true;
  }
  if (gated)
    hipLaunchKernelGGL(up_gemm_kernel<2>, dim3((unsigned)grid), dim3(kThreads), kLdsBytes, s, L, chunk_layer, w.xb,
                       scores, token_mask, active_idx, w.items, w.total, k, tiles_t, tiles_j, w.H);
  else
    hipLaunchKernelGGL(up_gemm_kernel<1>, dim3((unsigned)grid), dim3(kThreads), kLdsBytes, s, L, chunk_layer, w.xb,
                       scores, token_mask, active_idx, w.items, w.total, k, tiles_t, tiles_j, w.H);
  return hipGetLastError();
}

hipError_t launch_down_gemm(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, const void *ws, float *y,
                            hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  GemmWs w = carve(L, n_chunks, k, const_cast<void *>(ws));
  const int splits = down_splits(L, n_chunks, k);
  const int tiles_t = (k + kTileN - 1) / kTileN, tiles_c = L.d / kTileM;
  const int64_t grid = n_chunks * tiles_t * tiles_c * splits;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(down_gemm_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const size_t stride = (size_t)n_chunks * k * L.d;
  float *out = splits > 1 ? w.part : y;
  hipLaunchKernelGGL(down_gemm_kernel, dim3((unsigned)grid), dim3(kThreads), kLdsBytes, s, L, chunk_layer, active_idx,
                     n_active, k, tiles_t, tiles_c, splits, w.H, out, stride);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || splits == 1) return err;
  const size_t n4 = stride / 4;
  hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)std::min<size_t>((n4 + kThreads - 1) / kThreads, 4096)),
                     dim3(kThreads), 0, s, w.part, splits, stride, n4, y);
  return hipGetLastError();
}

}  // namespace blockffn
