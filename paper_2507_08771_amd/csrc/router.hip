// Router of the BlockFFN layer (Eq. 3): A^0 = W_router^T x + b, A^1 = ReLU(A^0),
// A = RMSNorm(A^1), plus the per-token activation mask (bit set iff A^0 > 0).
//
// The sign of A^0 decides a mask bit, so every product is an exact fp32 product and every sum is
// fp32.
//
// router_mfma_kernel (bf16 weights, enough tokens to fill the chip): x is carried as three bf16
// pieces that add up to the fp32 value exactly, and the matrix cores do the contraction; a
// workgroup (4 waves) takes tiles of 16 tokens.
// router_kernel (fp32 weights, and launches of tens of tiles, where blockIdx.y spreads the expert
// groups over workgroups; a handful of tiles take router_expert_kernel, one workgroup per
// expert and share of the tile's tokens): vector ALUs, a workgroup per tile of up to 8 tokens of
// one chunk.  Each lane keeps its 8 columns of the 8 tokens in registers (64 VGPRs) and walks
// over the experts: one 128-bit load of a W_router row segment feeds 64 fp32 FMAs; partial sums
// of 8 experts x 8 tokens are reduced across the wave with a 63-step reduce-scatter (lane q ends
// with entry q).
// All of them leave the four waves' partial sums in LDS for the same finishing step (bias, mask
// ballot, RMSNorm, gain).
#include "common.hpp"
#include "stream_common.hpp"

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

// The four waves' partial sums part[wave][expert][token] of a tile of NT tokens starting at token
// tok0 become A^0 (+ bias), the mask words and the RMSNorm'ed scores, for the tokens whose bit is
// set in `which` (all of them tokens of `layer`).  Each wave finishes tokens wave, wave + 4, ...:
// lanes run over experts, one mask word at a time.
template <int ROWS, int NT>
__device__ __forceinline__ void finish_tile(const LayerView &L, int layer, const float (&part)[4][ROWS][NT],
                                            int64_t tok0, uint32_t which, float *__restrict__ scores,
                                            uint64_t *__restrict__ token_mask, float *__restrict__ preact) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int E = L.E;
  for (int t = wave; t < NT; t += 4) {
    if (!((which >> t) & 1u)) continue;   // uniform over the wave
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

// SPLIT = false: one workgroup runs all experts of its token tile and finishes the tokens.
// SPLIT = true (few tokens in the launch): blockIdx.y selects one group of 8 experts; the
// workgroup writes that group's pre-activations A^0 into `scores` and router_finish_kernel
// normalises in place.
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

  finish_tile(L, layer, part, tok0, (1u << nt) - 1u, scores, token_mask, preact);
}

// A handful of token tiles (one chunk walking through a layer stack): one workgroup per (tile,
// expert, share of the tile's tokens), so that E or more workgroups pull the router matrix instead
// of E / 8.  Each thread takes 8 columns of the expert's row and of its tokens; the partial sums
// meet by wave reduction and a four-entry LDS step.  What a workgroup has to pull is mostly the
// tile's x (64 KiB for 8 tokens at d = 2048, against 4 KiB of W_router), and a CU takes in about
// 20 GB/s: with the tile's tokens dealt over gridDim.z workgroups each pulls its share only (a
// pre-activation belongs to one token and one expert, so nothing crosses workgroups).  Writes A^0
// (+ bias) into `scores`; router_finish_kernel normalises.  TPW: tokens per workgroup.
template <typename WT, int TPW>
__global__ __launch_bounds__(kThreads) void router_expert_kernel(LayerView L, const int32_t *__restrict__ chunk_layer,
                                                                 const float *__restrict__ x, int k,
                                                                 int tiles_per_chunk, float *__restrict__ scores) {
  __shared__ float part[4][TPW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t c = blockIdx.x / tiles_per_chunk;
  const int t0 = (int)(blockIdx.x % tiles_per_chunk) * kTok + (int)blockIdx.z * TPW;
  const int nt = min(TPW, k - t0);
  if (nt <= 0) return;   // uniform over the workgroup
  const int64_t tok0 = c * (int64_t)k + t0;
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int d = L.d, E = L.E, e = blockIdx.y;
  const size_t w_row = ((size_t)layer * E + e) * d;
  float acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) acc[t] = 0.0f;
  for (int cb = 0; cb < d; cb += kColsPerBlock) {
    const int col = cb + tid * 8;
    if (col < d) {
      float w[8];
      load8<WT>(L.w_router, w_row + col, w);
#pragma unroll
      for (int t = 0; t < TPW; ++t) {
        if (t < nt) {
          const float4 *p = reinterpret_cast<const float4 *>(x + (tok0 + t) * d + col);
          const float4 a = p[0], b = p[1];
          float s = acc[t];
          s = fmaf(w[0], a.x, s); s = fmaf(w[1], a.y, s); s = fmaf(w[2], a.z, s); s = fmaf(w[3], a.w, s);
          s = fmaf(w[4], b.x, s); s = fmaf(w[5], b.y, s); s = fmaf(w[6], b.z, s); s = fmaf(w[7], b.w, s);
          acc[t] = s;
        }
      }
    }
  }
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const float v = wave_sum(acc[t]);
    if (lane == 0) part[wave][t] = v;
  }
  __syncthreads();
  if (tid < nt) {
    float a0 = L.b_router ? L.b_router[(size_t)layer * E + e] : 0.0f;
    a0 += (part[0][tid] + part[1][tid]) + (part[2][tid] + part[3][tid]);
    scores[(tok0 + tid) * E + e] = a0;
  }
}

// bf16 weights, many tokens: the same contraction on the matrix cores without giving up fp32
// products.  An fp32 x is the exact sum of three bf16 numbers (24 significant bits in three
// pieces of 8: h = bf16(x), m = bf16(x - h), l = x - h - m), and a bf16 piece times a bf16
// weight is exact in fp32, so three MFMAs per 16 tokens (B operands: the 16 tokens' h, their m,
// their l) accumulate in fp32 exactly the products the vector ALUs would: only the order of the
// fp32 additions differs.  The sign of A^0 still decides the mask bit, and it is still backed by
// full fp32 products.
//
// Tiles of 16 tokens (the 16 columns of an MFMA) are cut from the launch's token stream
// (tiles_per_chunk = 0: tile j holds tokens 16 j .. 16 j + 15 whatever chunks they belong to, so
// that short chunks - k = 1: one token each - still fill the columns and pull the router matrix
// once per 16 tokens) or from each chunk (tile j is tile j mod tiles_per_chunk of chunk
// j / tiles_per_chunk; the launcher's choice when the chunks may be of different layers and k is
// no multiple of 16).  A workgroup takes T consecutive tiles; its four waves take the pairs of
// K-steps (64 contraction elements) w, w + 4, ... .  Per pair a wave loads RT tiles of W_router
// (16 experts x 64 elements each) as whole 128-byte lines - 8 lanes per expert row, two registers
// per tile, which a CU takes in nearly twice as fast as the 64-byte halves of operand order - and
// rearranges them into the two K-steps' A operands in registers (line_operands); lane (n, g)
// loads elements 8 g .. 8 g + 7 of token n of each K-step, splits them and issues 3 * RT MFMAs
// per tile and K-step.  KP pairs are loaded together so that their memory latency is paid once.
// At the end a lane adds its h, m and l sums and the four waves meet in the LDS layout the
// finishing step reads.
// The tokens of a workgroup may belong to chunks of different layers (different router
// matrices): the workgroup then makes one pass per distinct layer, with the other tokens'
// columns zero, and finishes after each pass the tokens of that layer.  A token's sums are the
// same whatever its column and whoever shares its tile.
constexpr int kTile = 16;   // tokens per tile of the MFMA kernel

template <int RT, int KP, int T>
__global__ __launch_bounds__(kThreads, RT >= 16 ? 1 : 2) void router_mfma_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const float *__restrict__ x, int k, int64_t n_chunks,
    int tiles_per_chunk, float *__restrict__ scores, uint64_t *__restrict__ token_mask, float *__restrict__ preact) {
  static_assert(T * kTile <= 32, "one bit per token of the workgroup");
  __shared__ float part[T][4][RT * 16][kTile];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, g = lane >> 4;
  const int lsrc = line_src(lane);
  const int d = L.d, E = L.E;
  const int64_t n_tok = n_chunks * k;
  int64_t tile_tok0[T];   // first token of each tile
  const float *xrow[T];
  int lay[T];   // layer of this lane's token of each tile, -1 where the tile has no such token
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
    const int64_t tile = (int64_t)blockIdx.x * T + tt;
    int64_t c;
    bool in;
    if (tiles_per_chunk > 0) {
      c = tile / tiles_per_chunk;
      const int i0 = (int)(tile - c * tiles_per_chunk) * kTile;
      tile_tok0[tt] = c * k + i0;
      in = c < n_chunks && i0 + n < k;
    } else {
      tile_tok0[tt] = tile * kTile;
      in = tile_tok0[tt] + n < n_tok;
      c = (tile_tok0[tt] + n) / k;
    }
    xrow[tt] = x + (in ? tile_tok0[tt] + n : 0) * d;
    lay[tt] = in ? clamp_layer(chunk_layer, c, L.n_layers) : -1;
  }
  // bit i: token i of the workgroup is still to do (lanes 0-15 hold tokens 0-15 of a tile)
  uint32_t pend = 0;
#pragma unroll
  for (int tt = 0; tt < T; ++tt) pend |= (uint32_t)(__ballot(lay[tt] >= 0) & 0xffffu) << (tt * kTile);
  const int n_pairs = (d + 63) / 64;

  while (pend) {
    // this pass: the layer of the first token still to do and every such token of the same layer
    const int first = __builtin_ctz(pend);
    int layer = 0;
    int64_t t_first = 0;
#pragma unroll
    for (int tt = 0; tt < T; ++tt) {
      const int v = __builtin_amdgcn_readlane(lay[tt], first & (kTile - 1));
      layer = (first / kTile == tt) ? v : layer;
      t_first = (first / kTile == tt) ? tile_tok0[tt] + (first & (kTile - 1)) : t_first;
    }
    uint32_t act = 0;
    bool tok_ok[T];
    // a lane without a token in this pass reads the first token's row again: no memory traffic of its own
    const float *xr[T];
#pragma unroll
    for (int tt = 0; tt < T; ++tt) {
      tok_ok[tt] = ((pend >> (tt * kTile + n)) & 1u) && lay[tt] == layer;
      act |= (uint32_t)(__ballot(tok_ok[tt]) & 0xffffu) << (tt * kTile);
      xr[tt] = tok_ok[tt] ? xrow[tt] : x + t_first * d;
    }
    pend &= ~act;
    const uint16_t *wr = static_cast<const uint16_t *>(L.w_router) + (size_t)layer * E * d;

    f32x4 acc[T][RT][3];   // sums of the h, m and l pieces
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) acc[tt][rt][pc] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int p0 = wave; p0 < n_pairs; p0 += 4 * KP) {
      uint4 a[KP][RT][2];            // per tile: the lines of experts 0-7 and of experts 8-15
      float4 xa[KP][2][T], xb[KP][2][T];
      bool xok[KP][2];
      // No load sits under a condition (a branch around a load makes the compiler wait for every
      // load before it at the join): past the end of a row (d is a multiple of 8: a lane's 8
      // elements are all in or all out) a lane reads column 0 instead, of W_router - a finite weight
      // times a zero piece of x adds nothing, and a weight that is not finite has spoilt its
      // expert's sum at column 0 already - and of x, which is then replaced by zero.
#pragma unroll
      for (int u = 0; u < KP; ++u) {
        const int pair = p0 + 4 * u;
        const int wcol = pair * 64 + (lane & 7) * 8;
        const int wc = wcol < d ? wcol : 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int col = (pair * 2 + h) * 32 + g * 8;
          xok[u][h] = col < d;
#pragma unroll
          for (int tt = 0; tt < T; ++tt) {
            const float4 *px = reinterpret_cast<const float4 *>(xr[tt] + (xok[u][h] ? col : 0));
            xa[u][h][tt] = px[0];
            xb[u][h][tt] = px[1];
          }
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            // rows at or above E repeat the last one; never read back
            const int row = min(rt * 16 + hh * 8 + line_row(lane), E - 1);
            a[u][rt][hh] = *reinterpret_cast<const uint4 *>(wr + (size_t)row * d + wc);
          }
      }
      // every load of the iteration is in flight before the first is used: left alone, the
      // scheduler (short of registers) sinks each tile's loads to its use and waits for them there
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < KP; ++u) {
        uint4 bh[2][T], bm[2][T], bl[2][T];   // B operands of the pair's two K-steps: the h, m and l pieces
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
          for (int tt = 0; tt < T; ++tt) {
            const bool ok = tok_ok[tt] && xok[u][h];
            const float xv[8] = {xa[u][h][tt].x, xa[u][h][tt].y, xa[u][h][tt].z, xa[u][h][tt].w,
                                 xb[u][h][tt].x, xb[u][h][tt].y, xb[u][h][tt].z, xb[u][h][tt].w};
            uint32_t hp[8], mp[8], lp[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const float v = ok ? xv[q] : 0.0f;
              hp[q] = bf16_bits(v);
              const float r1 = v - __uint_as_float(hp[q] << 16);
              mp[q] = bf16_bits(r1);
              const float r2 = r1 - __uint_as_float(mp[q] << 16);
              lp[q] = bf16_bits(r2);
            }
            bh[h][tt] = make_uint4(hp[0] | hp[1] << 16, hp[2] | hp[3] << 16, hp[4] | hp[5] << 16, hp[6] | hp[7] << 16);
            bm[h][tt] = make_uint4(mp[0] | mp[1] << 16, mp[2] | mp[3] << 16, mp[4] | mp[5] << 16, mp[6] | mp[7] << 16);
            bl[h][tt] = make_uint4(lp[0] | lp[1] << 16, lp[2] | lp[3] << 16, lp[4] | lp[5] << 16, lp[6] | lp[7] << 16);
          }
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          uint4 f[2];   // A operands of the pair's two K-steps
          line_operands(a[u][rt][0], a[u][rt][1], lsrc, f[0], f[1]);
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int tt = 0; tt < T; ++tt) {
              acc[tt][rt][0] = mfma16(f[h], bh[h][tt], acc[tt][rt][0]);
              acc[tt][rt][1] = mfma16(f[h], bm[h][tt], acc[tt][rt][1]);
              acc[tt][rt][2] = mfma16(f[h], bl[h][tt], acc[tt][rt][2]);
            }
        }
      }
    }
    // accumulator element q of lane (n, g) is expert rt * 16 + 4 * g + q, token n of the tile
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          part[tt][wave][rt * 16 + 4 * g + q][n] = (acc[tt][rt][0][q] + acc[tt][rt][1][q]) + acc[tt][rt][2][q];
    __syncthreads();
#pragma unroll
    for (int tt = 0; tt < T; ++tt) {
      const uint32_t which = (act >> (tt * kTile)) & 0xffffu;
      if (which) finish_tile(L, layer, part[tt], tile_tok0[tt], which, scores, token_mask, preact);
    }
    if (pend) __syncthreads();   // the next pass writes part again
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

// Whether launch_router takes its few-tile path with one workgroup per expert for this launch.
bool router_few(const LayerView &L, int64_t n_chunks, int k) {
  const int64_t blocks = n_chunks * ((k + kTok - 1) / kTok);
  return blocks > 0 && blocks * 2 <= 256 && (L.E + 7) / 8 > 1 && blocks * L.E <= 4096;
}

// First half of that path alone: A^0 (+ bias) into `preact` [token][E], nothing else.
hipError_t launch_router_preact_few(const LayerView &L, int wdtype, const int32_t *chunk_layer, const float *x,
                                    int64_t n_chunks, int k, float *preact, hipStream_t s) {
  if (!router_few(L, n_chunks, k)) return hipErrorInvalidValue;
  const int tiles = (k + kTok - 1) / kTok;
  const int64_t blocks = n_chunks * tiles;
  dim3 block(kThreads);
  const int64_t wgs = blocks * L.E;
  const int tpw = wgs * 4 <= 2 * num_cus() ? 2 : (wgs * 2 <= 2 * num_cus() ? 4 : 8);
  dim3 grid((unsigned)blocks, (unsigned)L.E, (unsigned)(kTok / tpw));
#define BLOCKFFN_ROUTER_EXPERT(WT)                                                                                  \
  if (tpw == 2) hipLaunchKernelGGL((router_expert_kernel<WT, 2>), grid, block, 0, s, L, chunk_layer, x, k, tiles, preact); \
  else if (tpw == 4) hipLaunchKernelGGL((router_expert_kernel<WT, 4>), grid, block, 0, s, L, chunk_layer, x, k, tiles, preact); \
  else hipLaunchKernelGGL((router_expert_kernel<WT, 8>), grid, block, 0, s, L, chunk_layer, x, k, tiles, preact)
  if (wdtype == BLOCKFFN_BF16) { BLOCKFFN_ROUTER_EXPERT(bf16_t); } else { BLOCKFFN_ROUTER_EXPERT(float); }
#undef BLOCKFFN_ROUTER_EXPERT
  return hipGetLastError();
}

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
    // few token tiles: spread the experts (or, with many tiles and experts, groups of 8 of them)
    // over workgroups, then normalise
    if (blocks * L.E <= 4096) {
      const hipError_t e = launch_router_preact_few(L, wdtype, chunk_layer, x, n_chunks, k, scores, s);
      if (e != hipSuccess) return e;
    } else {
      dim3 grid((unsigned)blocks, (unsigned)n_groups);
      if (wdtype == BLOCKFFN_BF16)
        hipLaunchKernelGGL((router_kernel<bf16_t, true>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores,
                           token_mask, preact);
      else
        hipLaunchKernelGGL((router_kernel<float, true>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores,
                           token_mask, preact);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t n_tok = n_chunks * k;
    hipLaunchKernelGGL(router_finish_kernel, dim3((unsigned)((n_tok + 3) / 4)), block, 0, s, L, chunk_layer, n_tok, k,
                       scores, token_mask, preact);
    return hipGetLastError();
  }
  dim3 grid((unsigned)blocks);
  if (wdtype == BLOCKFFN_BF16) {
    const int rt = (L.E + 15) / 16;
    const bool one_layer = chunk_layer == nullptr || L.n_layers == 1;
    // Tiles of 16 tokens, of the token stream where every chunk is of the same layer for sure or
    // where they are the chunks' own tiles anyway; else tiles of each chunk: a tile across chunks
    // of different layers takes one pass over a router matrix per layer, one after the other.
    const bool stream_tiles = one_layer || k % kTile == 0;
    const int tiles16 = (k + kTile - 1) / kTile;
    const int64_t n_tiles = stream_tiles ? (n_chunks * k + kTile - 1) / kTile : n_chunks * tiles16;
    const int tpc = stream_tiles ? 0 : tiles16;
#define BLOCKFFN_ROUTER(RT, KP, T)                                                                                 \
  hipLaunchKernelGGL((router_mfma_kernel<RT, KP, T>), dim3((unsigned)((n_tiles + T - 1) / T)), block, 0, s, L, chunk_layer, \
                     x, k, n_chunks, tpc, scores, token_mask, preact)
    // Every workgroup pulls the whole router matrix of its tokens' layer through its L1 (512 KiB at
    // E = 128, d = 2048, against 128 KiB of x per 16 tokens): up to 64 experts a workgroup takes 2
    // tiles per pass over the matrix (the accumulators allow it), where tiles that follow each other
    // are of one layer (for sure, or because the chunk has two) and the launch still has four
    // workgroups per CU.
    const bool two = (one_layer || tiles16 >= 2) && n_tiles / 2 >= 1024;
    if (rt <= 1) { if (two) BLOCKFFN_ROUTER(1, 2, 2); else BLOCKFFN_ROUTER(1, 2, 1); }
    else if (rt <= 2) { if (two) BLOCKFFN_ROUTER(2, 1, 2); else BLOCKFFN_ROUTER(2, 1, 1); }
    else if (rt <= 4) { if (two) BLOCKFFN_ROUTER(4, 1, 2); else BLOCKFFN_ROUTER(4, 1, 1); }
    else if (rt <= 8) BLOCKFFN_ROUTER(8, 1, 1);
    else BLOCKFFN_ROUTER(16, 1, 1);
#undef BLOCKFFN_ROUTER
  } else
    hipLaunchKernelGGL((router_kernel<float, false>), grid, block, 0, s, L, chunk_layer, x, k, tiles, scores, token_mask,
                         preact);
  return hipGetLastError();
}

}  // namespace blockffn
