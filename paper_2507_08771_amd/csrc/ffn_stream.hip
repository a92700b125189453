// Chunk-sparse expert FFN (Sec. 3.3), weight-streaming kernels for bf16 weights and chunks of
// up to 32 tokens.
//
// The work is bound by the HBM stream of the active experts' weights (k flop per weight byte),
// so the kernels are built around keeping 16 KB of 128-bit weight loads in flight per wave and
// doing nothing else on the vector ALUs.  The contraction itself runs on the matrix cores:
// a v_mfma_f32_16x16x32_bf16 takes 16 weight rows x 32 contraction elements as its A operand
// straight from the registers the loads land in (lane l = row l%16, 16 bytes at element
// 8*(l/16)), so no unpacking, no cross-lane reduction and no LDS staging of weights is needed.
// The fp32 activations are carried as two bf16 halves (x = hi + lo, 16 significant bits).
// Products of bf16 pairs are exact in fp32 and accumulation is fp32, so the result is within
// ~2^-17 of an fp32-activation product.
//
// B-operand fragments (16 token columns x 32 contraction elements each), NB per K-step:
//   k <= 8   NB = 1: columns 0-7 are the tokens' hi halves, columns 8-15 their lo halves; the two
//                    column groups of the accumulator are added at the end;
//   k <= 16  NB = 2: fragment 0 = hi, fragment 1 = lo of 16 tokens, both accumulated into the
//                    same tile;
//   k <= 32  NB = 4: (group 0 hi, group 0 lo, group 1 hi, group 1 lo), two accumulator tiles.
//
//   up    persistent workgroups walk a flat list of (chunk, slot) items.  The chunk's x is split
//         into hi/lo bf16 once per item into LDS in B-operand order; each wave owns distinct
//         neuron rows of W_up (and W_gate) over the full contraction, so waves never exchange
//         partial sums.  Swish/gating, router score and mask are applied in registers and mid
//         is written already split into bf16 hi/lo in the B-operand order of the down kernel.
//   down  grid (chunk, 512 output columns); the reduction runs over the union's slots and the
//         expert's neurons; mid of the next slot is staged through LDS (double buffered) while
//         the current slot's W_down rows stream; one writer per output element.
#include <algorithm>

#include "common.hpp"

namespace blockffn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRing = 16;          // 128-bit loads in flight per lane
constexpr int kXBytes = 64 * 1024; // LDS for the split activations of one K-chunk

__device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

__device__ __forceinline__ uint32_t bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}

// x = hi + lo with hi = bf16(x) and lo = bf16(x - hi); 16-bit patterns in the low halves
__device__ __forceinline__ void split_bf16(float x, uint32_t &hi, uint32_t &lo) {
  hi = bf16_bits(x);
  lo = bf16_bits(x - __uint_as_float(hi << 16));
}

constexpr int acc_tiles(int NB) { return NB == 4 ? 2 : 1; }
constexpr int acc_of(int NB, int bf) { return NB == 4 ? bf / 2 : 0; }
constexpr int tokens_of(int NB) { return NB == 1 ? 8 : (NB == 2 ? 16 : 32); }

// Flat (chunk, slot) work list: items[i] = chunk * E + slot for every slot below n_active[chunk].
__global__ __launch_bounds__(1024) void worklist_kernel(const int32_t *__restrict__ n_active, int64_t n_chunks, int E,
                                                        int32_t *__restrict__ items, int32_t *__restrict__ total) {
  __shared__ int wave_tot[16];
  __shared__ int carry;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int64_t c0 = 0; c0 < n_chunks; c0 += 1024) {
    const int64_t c = c0 + tid;
    int n = 0;
    if (c < n_chunks) n = n_active ? min(max(n_active[c], 0), E) : E;
    int incl = n;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, kWave);
      if (lane >= off) incl += v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int base = carry;
    for (int w = 0; w < wave; ++w) base += wave_tot[w];
    const int start = base + incl - n;
    for (int s = 0; s < n; ++s) items[start + s] = (int32_t)(c * E + s);
    __syncthreads();
    if (tid == 1023) carry = base + incl;
    __syncthreads();
  }
  if (tid == 0) *total = carry;
}

// ------------------------------------------------------------------------------------------------ up

// NB: B fragments per K-step (see the top of the file); NM: 1 (Eq. 2) or 2 (gated); RT: 64-row
// groups of the expert (d_e = 64 * RT).  Wave w owns row tiles rr*4 + w.
template <int NB, int NM, int RT>
__global__ __launch_bounds__(kThreads, 2) void up_stream_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const float *__restrict__ x,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ items, const int32_t *__restrict__ total_ptr, int k, uint16_t *__restrict__ midB) {
  extern __shared__ uint4 xB[];   // [K-step][NB][64 lanes] of 8 bf16
  constexpr int KC = 2048 / NB;   // contraction elements per LDS fill
  constexpr int NA = acc_tiles(NB);
  constexpr int TOK = tokens_of(NB);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int total = *total_ptr;
  const size_t row_bytes = (size_t)d * 2;

  auto item_expert = [&](int item, int64_t &c, int &s, int &e) {
    const int code = items[item];   // chunk * E + slot
    c = code / E;
    s = code - (int)c * E;
    e = active_idx ? active_idx[c * E + s] : s;
    e = min(max(e, 0), E - 1);
  };
  // per-lane byte pointer to the first fragment of (layer, expert, tile rr, matrix m)
  auto tile_ptr = [&](int layer, int e, int rr, int m) -> const char * {
    const char *w = static_cast<const char *>(m == 0 ? L.w_up : L.w_gate);
    const size_t row = ((size_t)layer * E + e) * d_e + (rr * 4 + wave) * 16 + r;
    return w + row * row_bytes + g * 16;
  };

  uint4 ring[kRing];
  int item = blockIdx.x;
  if (item >= total) return;
  int64_t c;
  int s, e;
  item_expert(item, c, s, e);
  int layer = clamp_layer(chunk_layer, c, L.n_layers);
  {
    const char *p = tile_ptr(layer, e, 0, 0);
#pragma unroll
    for (int i = 0; i < kRing; ++i) ring[i] = *reinterpret_cast<const uint4 *>(p + i * 64);
  }

  while (true) {
    const int next_item = item + gridDim.x;
    const bool has_next = next_item < total;
    int64_t c_n = 0;
    int s_n = 0, e_n = 0, layer_n = 0;
    if (has_next) {
      item_expert(next_item, c_n, s_n, e_n);
      layer_n = clamp_layer(chunk_layer, c_n, L.n_layers);
    }

    f32x4 acc[RT][NM][NA];
#pragma unroll
    for (int a = 0; a < RT; ++a)
#pragma unroll
      for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int q = 0; q < NA; ++q) acc[a][m][q] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int kc0 = 0; kc0 < d; kc0 += KC) {
      const int kc_len = min(KC, d - kc0);
      const int nkb = kc_len / 512;
      __syncthreads();   // every wave is done with the previous contents of xB
      // split x[c*k + tok][kc0 .. kc0 + kc_len) into hi/lo bf16 in B-operand order
      for (int it = tid; it < (kc_len / 8) * TOK; it += kThreads) {
        const int tok = it % TOK, cg = it / TOK;   // cg: group of 8 columns
        const int kstep = cg >> 2, gg = cg & 3;
        uint32_t hi[8], lo[8];
        if (tok < k) {
          const float4 *p = reinterpret_cast<const float4 *>(x + (c * k + tok) * d + kc0 + cg * 8);
          const float4 a = p[0], b = p[1];
          const float xv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
          for (int q = 0; q < 8; ++q) split_bf16(xv[q], hi[q], lo[q]);
        } else {
#pragma unroll
          for (int q = 0; q < 8; ++q) hi[q] = lo[q] = 0;
        }
        const uint4 vhi = make_uint4(hi[0] | hi[1] << 16, hi[2] | hi[3] << 16, hi[4] | hi[5] << 16, hi[6] | hi[7] << 16);
        const uint4 vlo = make_uint4(lo[0] | lo[1] << 16, lo[2] | lo[3] << 16, lo[4] | lo[5] << 16, lo[6] | lo[7] << 16);
        if (NB == 1) {
          uint4 *dst = xB + (size_t)kstep * 64 + gg * 16 + tok;
          dst[0] = vhi;
          dst[8] = vlo;
        } else {
          const int grp = tok >> 4, n = tok & 15;
          uint4 *dst = xB + (size_t)(kstep * NB + grp * 2) * 64 + gg * 16 + n;
          dst[0] = vhi;
          dst[64] = vlo;
        }
      }
      __syncthreads();
      const bool last_kc = kc0 + KC >= d;
#pragma unroll
      for (int rr = 0; rr < RT; ++rr) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const char *cur = tile_ptr(layer, e, rr, m) + (size_t)kc0 * 2;
          // first block of the tile that follows this one in (K-chunk, rr, m) order
          const char *nxt_tile;
          bool nxt_ok = true;
          if (m + 1 < NM) nxt_tile = tile_ptr(layer, e, rr, m + 1) + (size_t)kc0 * 2;
          else if (rr + 1 < RT) nxt_tile = tile_ptr(layer, e, rr + 1, 0) + (size_t)kc0 * 2;
          else if (!last_kc) nxt_tile = tile_ptr(layer, e, 0, 0) + (size_t)(kc0 + KC) * 2;
          else {
            nxt_tile = tile_ptr(layer_n, e_n, 0, 0);
            nxt_ok = has_next;
          }
          for (int kb = 0; kb < nkb; ++kb) {
            const bool tail = kb + 1 == nkb;
            const char *nxt = tail ? nxt_tile : cur + (size_t)(kb + 1) * 1024;
            const bool ok = tail ? nxt_ok : true;
#pragma unroll
            for (int i = 0; i < kRing; ++i) {
#pragma unroll
              for (int bf = 0; bf < NB; ++bf) {
                const uint4 b = xB[(size_t)((kb * kRing + i) * NB + bf) * 64 + lane];
                acc[rr][m][acc_of(NB, bf)] = mfma16(ring[i], b, acc[rr][m][acc_of(NB, bf)]);
              }
              if (ok) ring[i] = *reinterpret_cast<const uint4 *>(nxt + i * 64);
            }
          }
        }
      }
    }

    // epilogue, entirely inside the wave: lane (n = lane%16, g) holds rows 4g..4g+3 of each tile
    const int n = lane & 15;
#pragma unroll
    for (int q = 0; q < NA; ++q) {
      const int t = NB == 1 ? (n & 7) : q * 16 + n;
      float f = 0.0f;
      bool on = false;
      if (t < k) {
        const int64_t tok = c * k + t;
        on = token_mask ? (bool)((token_mask[tok * L.W + (e >> 6)] >> (e & 63)) & 1) : true;
        f = scores[tok * E + e];
      }
#pragma unroll
      for (int rr = 0; rr < RT; ++rr) {
        uint32_t phi[4], plo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float u = acc[rr][0][q][j];
          if (NB == 1) u += __shfl_xor(u, 8, kWave);
          float h;
          if (NM == 2) {
            float gt = acc[rr][NM - 1][q][j];
            if (NB == 1) gt += __shfl_xor(gt, 8, kWave);
            h = swish(gt) * u;
          } else {
            h = swish(u);
          }
          split_bf16(on ? f * h : 0.0f, phi[j], plo[j]);
        }
        const uint2 vhi = make_uint2(phi[0] | phi[1] << 16, phi[2] | phi[3] << 16);
        const uint2 vlo = make_uint2(plo[0] | plo[1] << 16, plo[2] | plo[3] << 16);
        const size_t col = (rr * 4 + wave) * 16 + 4 * g;
        uint16_t *base = midB + ((size_t)c * E + s) * NB * 16 * d_e;
        if (NB == 1) {
          // fragment row n: hi for n < 8, lo of token n - 8 for n >= 8
          *reinterpret_cast<uint2 *>(base + (size_t)n * d_e + col) = n < 8 ? vhi : vlo;
        } else {
          *reinterpret_cast<uint2 *>(base + ((size_t)(q * 2) * 16 + n) * d_e + col) = vhi;
          *reinterpret_cast<uint2 *>(base + ((size_t)(q * 2 + 1) * 16 + n) * d_e + col) = vlo;
        }
      }
    }

    if (!has_next) break;
    item = next_item;
    c = c_n; s = s_n; e = e_n; layer = layer_n;
  }
}

// ------------------------------------------------------------------------------------------------ down

// KSD = d_e / 32 K-steps per slot, MW row tiles (16 output columns each) per wave.
template <int NB, int KSD, int MW>
__global__ __launch_bounds__(kThreads, 2) void down_stream_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int k, int col_blocks, const uint16_t *__restrict__ midB,
    float *__restrict__ y) {
  constexpr int kFrag = KSD * MW;             // weight fragments per slot and wave
  static_assert(kFrag % kRing == 0, "ring must divide the fragments of a slot");
  constexpr int kStage = KSD * NB * 64;       // uint4 of mid per slot
  constexpr int kPerThread = (kStage + kThreads - 1) / kThreads;
  constexpr int NA = acc_tiles(NB);
  __shared__ uint4 midS[2][kStage];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int E = L.E, d = L.d;
  constexpr int d_e = KSD * 32;
  const int64_t c = blockIdx.x / col_blocks;
  const int col0 = (int)(blockIdx.x % col_blocks) * (4 * MW * 16) + wave * (MW * 16);
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int n_act = active_idx ? min(max(n_active[c], 0), E) : E;

  auto slot_expert = [&](int s) {
    int e = active_idx ? active_idx[c * E + s] : s;
    return min(max(e, 0), E - 1);
  };
  auto slot_ptr = [&](int e) -> const char * {
    const size_t row = ((size_t)layer * E + e) * d + col0 + r;
    return static_cast<const char *>(L.w_down) + row * (d_e * 2) + g * 16;
  };
  // fragment f of a slot: row tile f / KSD, K-step f % KSD.  The K-steps of one row tile are
  // consecutive so that the 64-byte halves of each 128-byte line are requested back to back
  // (requested several loads apart they were fetched from the fabric twice).
  auto frag_off = [&](int f) { return (size_t)(f / KSD) * 16 * d_e * 2 + (size_t)(f % KSD) * 64; };

  f32x4 acc[MW][NA];
#pragma unroll
  for (int a = 0; a < MW; ++a)
#pragma unroll
    for (int q = 0; q < NA; ++q) acc[a][q] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (n_act > 0) {
    uint4 ring[kRing];
    int e = slot_expert(0);
    {
      const char *p = slot_ptr(e);
#pragma unroll
      for (int i = 0; i < kRing; ++i) ring[i] = *reinterpret_cast<const uint4 *>(p + frag_off(i));
    }
    const uint4 *mid_c = reinterpret_cast<const uint4 *>(midB + (size_t)c * E * (NB * 16) * d_e);
    // mid of one slot is [NB][16][d_e] bf16; B-operand order is [K-step][NB][lane = g*16 + n]
    auto stage_src = [&](int s, int idx) {
      const int ln = idx & 63, bf = (idx >> 6) % NB, ks = idx / (64 * NB);
      const int n = ln & 15, gg = ln >> 4;
      return mid_c + (((size_t)s * NB + bf) * 16 + n) * (d_e / 8) + ks * 4 + gg;
    };
#pragma unroll
    for (int q = 0; q < kPerThread; ++q) {
      const int idx = tid + q * kThreads;
      if (idx < kStage) midS[0][idx] = *stage_src(0, idx);
    }
    __syncthreads();

    for (int s = 0; s < n_act; ++s) {
      const bool has_next = s + 1 < n_act;
      const int e_n = has_next ? slot_expert(s + 1) : e;
      const char *nxt = slot_ptr(e_n);
      // mid of the next slot (the last slot re-reads itself; the copy is harmless and keeps the
      // staging registers unconditional)
      const int s_stage = has_next ? s + 1 : s;
      uint4 stage[kPerThread];
#pragma unroll
      for (int q = 0; q < kPerThread; ++q) {
        const int idx = tid + q * kThreads;
        stage[q] = *stage_src(s_stage, idx < kStage ? idx : 0);
      }
      const char *cur = slot_ptr(e);
      const uint4 *bS = midS[s & 1];
#pragma unroll
      for (int tile = 0; tile < MW; ++tile) {
#pragma unroll
        for (int ks = 0; ks < KSD; ++ks) {
          const int f = tile * KSD + ks;
#pragma unroll
          for (int bf = 0; bf < NB; ++bf)
            acc[tile][acc_of(NB, bf)] =
                mfma16(ring[f % kRing], bS[(ks * NB + bf) * 64 + lane], acc[tile][acc_of(NB, bf)]);
          const int fn = f + kRing;
          if (fn < kFrag) ring[f % kRing] = *reinterpret_cast<const uint4 *>(cur + frag_off(fn));
          else if (has_next) ring[f % kRing] = *reinterpret_cast<const uint4 *>(nxt + frag_off(fn - kFrag));
        }
      }
#pragma unroll
      for (int q = 0; q < kPerThread; ++q) {
        const int idx = tid + q * kThreads;
        if (idx < kStage) midS[(s + 1) & 1][idx] = stage[q];
      }
      __syncthreads();
      e = e_n;
    }
  }

  const int n = lane & 15;
#pragma unroll
  for (int q = 0; q < NA; ++q) {
    const int t = NB == 1 ? (n & 7) : q * 16 + n;
    const bool writer = (NB == 1 ? n < 8 : true) && t < k;
#pragma unroll
    for (int tile = 0; tile < MW; ++tile) {
      float4 v;
      float *vp = reinterpret_cast<float *>(&v);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = acc[tile][q][j];
        vp[j] = NB == 1 ? a + __shfl_xor(a, 8, kWave) : a;
      }
      if (writer) *reinterpret_cast<float4 *>(y + (c * k + t) * d + col0 + tile * 16 + 4 * g) = v;
    }
  }
}

int g_num_cus = 0;

int num_cus() {
  if (g_num_cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      g_num_cus = n;
    else
      g_num_cus = 256;
  }
  return g_num_cus;
}

template <int NB, int NM, int RT>
hipError_t launch_up(const LayerView &L, const int32_t *chunk_layer, const float *x, const float *scores,
                     const uint64_t *token_mask, const int32_t *active_idx, const int32_t *items,
                     const int32_t *total, int64_t max_items, int k, uint16_t *midB, hipStream_t s) {
  static bool attr_set = false;
  auto kern = up_stream_kernel<NB, NM, RT>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kXBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t grid = std::min<int64_t>(max_items, (int64_t)num_cus() * 2);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), kXBytes, s, L, chunk_layer, x, scores, token_mask,
                     active_idx, items, total, k, midB);
  return hipGetLastError();
}

template <int NB, int KSD>
hipError_t launch_down(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                       const int32_t *n_active, int64_t n_chunks, int k, const uint16_t *midB, float *y,
                       hipStream_t s) {
  constexpr int MW = (NB == 4 && KSD >= 4) ? 4 : 8;   // two accumulator tiles per row tile at NB = 4
  const int col_blocks = L.d / (4 * MW * 16);
  const int64_t grid = n_chunks * col_blocks;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((down_stream_kernel<NB, KSD, MW>), dim3((unsigned)grid), dim3(kThreads), 0, s, L, chunk_layer,
                     active_idx, n_active, k, col_blocks, midB, y);
  return hipGetLastError();
}

int b_frags(int k) { return k <= 8 ? 1 : (k <= 16 ? 2 : 4); }

struct StreamWs {
  uint16_t *midB;
  int32_t *items, *total;
};

size_t mid_bytes(const LayerView &L, int64_t n_chunks, int k) {
  return ((size_t)n_chunks * L.E * b_frags(k) * 16 * L.d_e * 2 + 255) & ~(size_t)255;
}

StreamWs carve(const LayerView &L, int64_t n_chunks, int k, void *ws) {
  char *p = static_cast<char *>(ws);
  StreamWs w;
  w.midB = reinterpret_cast<uint16_t *>(p);
  w.total = reinterpret_cast<int32_t *>(p + mid_bytes(L, n_chunks, k));
  w.items = w.total + 64;
  return w;
}

}  // namespace

hipError_t launch_worklist(const int32_t *n_active, int64_t n_chunks, int E, int32_t *items, int32_t *total,
                           hipStream_t s) {
  hipLaunchKernelGGL(worklist_kernel, dim3(1), dim3(1024), 0, s, n_active, n_chunks, E, items, total);
  return hipGetLastError();
}

bool stream_supported(const LayerView &L, int wdtype, int k) {
  return wdtype == BLOCKFFN_BF16 && k <= 32 && L.d % 512 == 0 &&
         (L.d_e == 64 || L.d_e == 128 || L.d_e == 256);
}

size_t stream_workspace_bytes(const LayerView &L, int64_t n_chunks, int k) {
  // mid as bf16 hi/lo fragments [chunk][slot][NB][16][d_e], then the item count and the item list
  const size_t items = ((size_t)n_chunks * L.E + 64) * sizeof(int32_t);
  return mid_bytes(L, n_chunks, k) + ((items + 255) & ~(size_t)255);
}

hipError_t launch_up_stream(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                            const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, void *ws, hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  if (n_chunks * L.E > 0x7fffffffLL) return hipErrorInvalidValue;
  StreamWs w = carve(L, n_chunks, k, ws);
  hipError_t err = launch_worklist(n_active, n_chunks, L.E, w.items, w.total, s);
  if (err != hipSuccess) return err;
  const int NB = b_frags(k), RT = L.d_e / 64;
  const int64_t max_items = n_chunks * L.E;
#define BLOCKFFN_CASE(nb, nm, rt)                                                                         \
  if (NB == nb && (gated ? 2 : 1) == nm && RT == rt)                                                      \
    return launch_up<nb, nm, rt>(L, chunk_layer, x, scores, token_mask, active_idx, w.items, w.total, max_items, k, \
                                 w.midB, s);
  BLOCKFFN_CASE(1, 1, 1) BLOCKFFN_CASE(1, 1, 2) BLOCKFFN_CASE(1, 1, 4)
  BLOCKFFN_CASE(1, 2, 1) BLOCKFFN_CASE(1, 2, 2) BLOCKFFN_CASE(1, 2, 4)
  BLOCKFFN_CASE(2, 1, 1) BLOCKFFN_CASE(2, 1, 2) BLOCKFFN_CASE(2, 1, 4)
  BLOCKFFN_CASE(2, 2, 1) BLOCKFFN_CASE(2, 2, 2) BLOCKFFN_CASE(2, 2, 4)
  BLOCKFFN_CASE(4, 1, 1) BLOCKFFN_CASE(4, 1, 2) BLOCKFFN_CASE(4, 1, 4)
  BLOCKFFN_CASE(4, 2, 1) BLOCKFFN_CASE(4, 2, 2) BLOCKFFN_CASE(4, 2, 4)
#undef BLOCKFFN_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_down_stream(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                              const int32_t *n_active, int64_t n_chunks, int k, const void *ws, float *y,
                              hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  StreamWs w = carve(L, n_chunks, k, const_cast<void *>(ws));
  const int NB = b_frags(k), KSD = L.d_e / 32;
#define BLOCKFFN_CASE(nb, ksd) \
  if (NB == nb && KSD == ksd) return launch_down<nb, ksd>(L, chunk_layer, active_idx, n_active, n_chunks, k, w.midB, y, s);
  BLOCKFFN_CASE(1, 2) BLOCKFFN_CASE(1, 4) BLOCKFFN_CASE(1, 8)
  BLOCKFFN_CASE(2, 2) BLOCKFFN_CASE(2, 4) BLOCKFFN_CASE(2, 8)
  BLOCKFFN_CASE(4, 2) BLOCKFFN_CASE(4, 4) BLOCKFFN_CASE(4, 8)
#undef BLOCKFFN_CASE
  return hipErrorInvalidValue;
}

}  // namespace blockffn
