// Chunk-sparse expert FFN (Sec. 3.3) for large chunks (33 .. 512 tokens, e.g. a prefill chunk):
// here one expert's weights are reused by hundreds of tokens, the work is a dense grouped
// contraction over the experts of the union and the matrix cores are the bound, not HBM.
//
//   x  -> two bf16 planes, hi = bf16(x) and lo = bf16(x - hi) (x = hi + lo to 16 significant
//         bits, as on the streaming path); products are bf16 x bf16, exact in fp32, accumulated
//         in fp32.  The up projection walks the contraction twice per stage, once against each
//         plane, with the same weight lines (the second request finds them in L2), so the fp32
//         activations the configurations state reach the product to 2^-17 and mid is the only
//         value rounded to bf16 on the way to y (once, 2^-9 relative per element).
//   up    one workgroup = (item of the (chunk, slot) list, TN tokens, TM/2 neurons): a
//         TM x TN x 2d contraction (TM/2 W_up rows and the matching W_gate rows against TN
//         tokens; TM = TN = 256, or 128 for short chunks), both operands staged through
//         double-buffered LDS (LDS-direct global loads of whole 128-byte lines, 8 lanes per
//         row; an XOR swizzle of the pieces keeps the fragment reads conflict free).
//         Swish/gating, score and mask are applied on the accumulators; mid is written as
//         bf16 [chunk][slot][token][neuron].
//   down  one workgroup = (chunk, TM output columns, TN tokens, split): the contraction runs
//         over the slots of the split and the expert's neurons.  When a launch would have too
//         few workgroups to fill the chip the slots are split and the partial sums are added
//         by a second kernel in a fixed order (no atomics; results repeat bit for bit).
//
// The paper's kernel computes every token of the chunk for every expert of the union and applies
// the sparse pattern of A afterwards; that is right for chunks of up to 32 tokens.  In a chunk
// of hundreds of tokens the union holds nearly every expert while a token has a fifth of them,
// so here the up projection of (chunk, expert) gathers the expert's own tokens (prepare_kernel)
// into 128-column tiles and scatters their rows of mid; the other rows stay zero (mid is zeroed
// first).  The terms left out are exactly those the mask would have zeroed.
#include <algorithm>

#include "common.hpp"

namespace blockffn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

// Workgroup tile: TM weight rows x TN tokens, WR x WC waves.  The chip's L2 delivers about
// 10-15 TB/s to the CUs (measured), the matrix cores want 2.5 PFLOP/s: a tile has to reuse every
// byte it pulls from L2 for > 100 flop, which takes 256 x 256 (128 flop per byte); 128 x 128
// (64 flop per byte) is kept for chunks too short to fill 256 token columns.
template <int TM_, int TN_, int WR_, int WC_, int KS_, bool RING_>
struct Tile {
  static constexpr int TM = TM_, TN = TN_, WR = WR_, WC = WC_;
  static constexpr bool RING = RING_;                      // five half-stage buffers (see gemm_mainloop_ring)
  static constexpr int KS = KS_;                           // MFMA K-steps (32 elements) per stage
  static constexpr int TK = 32 * KS;                       // contraction elements per stage
  static constexpr int WAVES = WR * WC, THREADS = WAVES * 64;
  static constexpr int FA = TM / 16, FB = TN / 16;        // operand fragments per K-step
  static constexpr int FI = FA / WR, FJ = FB / WC;         // a wave's tile, in fragments
  static constexpr int NL = (FA + FB) * KS / WAVES;        // 1 KiB block loads per wave and stage
  static constexpr int STAGE_VEC = (FA + FB) * KS * 64;    // uint4 per stage
  static constexpr int HALF_VEC = (FA + FB) * 64;          // uint4 per half stage (one K-step) of the ring
  static constexpr int LDS_BYTES = RING ? 5 * HALF_VEC * 16 : 2 * STAGE_VEC * 16;
  static constexpr int WF = FA / WAVES;                    // A fragments (and B fragments) a wave loads
  static constexpr int NOFF = RING ? 2 * WF : NL;          // distinct lane offsets of a wave's loads
  static_assert(FA == FB && FA % WAVES == 0 && NL == 4 * WF, "every wave loads WF fragments of each operand");
  static_assert((FA / 2) % WF == 0, "a wave's A fragments must not straddle W_up / W_gate");
};
// (A 4-wave variant of the 256-wide tile with 128 x 128 per wave, which halves the LDS reads per
// MFMA, was slower: one wave per SIMD leaves nothing to cover LDS and memory latency with.)
using TileSmall = Tile<128, 128, 2, 2, 2, false>;   // 4 waves, 64 KiB LDS, 2 workgroups per CU
using TileBig = Tile<256, 256, 2, 4, 2, true>;       // 8 waves, 160 KiB LDS (5 x 32 KiB), 1 workgroup per CU

__device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

__device__ __forceinline__ uint32_t bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}

// Swish for a result that is rounded to bf16 right away: hardware exp2 and reciprocal (about
// 1e-6 relative, against the 2^-9 of the rounding).  u -> -inf gives u * 0.
__device__ __forceinline__ float swish_fast(float u) {
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * u));
}

// The tokens of a chunk that have expert e (mask bit set), in ascending order: lists[(c E + e) k ..],
// counts[c E + e].  One wave per (chunk, expert).  At the 512-token prefill chunk the union holds
// nearly every expert but a token only a fifth of them, so the up projection of an expert runs
// over its own tokens only (the product is the same: the other tokens' terms are masked to zero).
__device__ __forceinline__ void token_list_wave(const uint64_t *__restrict__ token_mask, int W, int E, int k,
                                                int64_t pair, int lane, int32_t *__restrict__ lists,
                                                int32_t *__restrict__ counts) {
  const int64_t c = pair / E;
  const int e = (int)(pair % E);
  int32_t *list = lists + (size_t)pair * k;
  int base = 0;
  for (int t0 = 0; t0 < k; t0 += 64) {
    const int t = t0 + lane;
    const bool bit = t < k && ((token_mask[(c * k + t) * W + (e >> 6)] >> (e & 63)) & 1);
    const uint64_t b = __ballot(bit);
    if (bit) list[base + __popcll(b & ((1ull << lane) - 1))] = t;
    base += __popcll(b);
  }
  if (lane == 0) counts[pair] = base;
}

// The three passes ahead of the up projection in one launch (they are independent, and as three
// launches of a few microseconds each they ran one after the other): blocks [0, cvt_blocks) split
// x into its bf16 planes (hi at xb, lo at xb + 8 n8), the next zero_blocks clear mid, the rest
// build the token lists, one wave per (chunk, expert).  Without a mask there are no lists and
// nothing to clear.
__global__ __launch_bounds__(kThreads) void prepare_kernel(const float *__restrict__ x, uint16_t *__restrict__ xb,
                                                           size_t n8, int cvt_blocks, uint4 *__restrict__ H, size_t n16,
                                                           int zero_blocks, const uint64_t *__restrict__ token_mask, int W,
                                                           int E, int k, int64_t n_pairs, int32_t *__restrict__ lists,
                                                           int32_t *__restrict__ counts) {
  const int b = blockIdx.x;
  if (b < cvt_blocks) {
    for (size_t i = (size_t)b * kThreads + threadIdx.x; i < n8; i += (size_t)cvt_blocks * kThreads) {
      const float4 a = reinterpret_cast<const float4 *>(x)[2 * i], c = reinterpret_cast<const float4 *>(x)[2 * i + 1];
      const float v[8] = {a.x, a.y, a.z, a.w, c.x, c.y, c.z, c.w};
      uint32_t hi[8], lo[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        hi[q] = bf16_bits(v[q]);
        lo[q] = bf16_bits(v[q] - __uint_as_float(hi[q] << 16));
      }
      reinterpret_cast<uint4 *>(xb)[i] =
          make_uint4(hi[0] | hi[1] << 16, hi[2] | hi[3] << 16, hi[4] | hi[5] << 16, hi[6] | hi[7] << 16);
      reinterpret_cast<uint4 *>(xb)[n8 + i] =
          make_uint4(lo[0] | lo[1] << 16, lo[2] | lo[3] << 16, lo[4] | lo[5] << 16, lo[6] | lo[7] << 16);
    }
  } else if (b < cvt_blocks + zero_blocks) {
    for (size_t i = (size_t)(b - cvt_blocks) * kThreads + threadIdx.x; i < n16; i += (size_t)zero_blocks * kThreads)
      H[i] = make_uint4(0, 0, 0, 0);
  } else {
    const int64_t pair = (int64_t)(b - cvt_blocks - zero_blocks) * (kThreads / 64) + (threadIdx.x >> 6);
    if (pair < n_pairs) token_list_wave(token_mask, W, E, k, pair, threadIdx.x & 63, lists, counts);
  }
}

// One stage in LDS: operand fragment F (A fragments first, then B) owns 2 KiB: block h (1 KiB)
// holds rows 8h .. 8h + 7 of the fragment, both K-steps: a whole 128-byte line per row.  The
// stage is filled by LDS-direct loads (global_load_lds_dwordx4: lane j's 16 bytes land at the
// block's base + 16 j, no staging registers and no LDS store instructions): lane j of block h
// loads piece (j & 7) XOR r of row r = (j >> 3) XOR h, so the 8 lanes of a row together request
// the row's whole line, and the 16-byte piece p of row r sits at slot 8 (r XOR h) + (p XOR r) of
// its block.  A fragment read for K-step ks takes piece 4 ks + g of row n for lane (n, g): the 16
// lanes of one g (two blocks) hit 16 different 16-byte bank groups of the 64-bank LDS, so the
// reads are conflict free - without the row swap in odd blocks the two blocks collided and every
// read took 8 instead of 4 cycles (SQ_LDS_BANK_CONFLICT was half of SQ_LDS_IDX_ACTIVE).  Wave w fills A fragments and B
// fragments [WF w, WF w + WF) (half of its loads each: the two operands come back at different
// speeds, and waves that loaded only the slow one kept the others waiting at the barrier).  The
// loads of one operand share a base pointer (base_a(stage) / base_b(stage), uniform over the
// wave) and differ only by the lane offsets off[] (elements; A blocks first), fixed for the whole
// loop.  The loads for stage st + 1 are issued while stage st is computed and awaited before the
// barrier that ends it.

template <typename T, typename BaseA, typename BaseB>
__device__ __forceinline__ void gemm_mainloop(uint4 *lds, int n_stages, BaseA base_a, BaseB base_b,
                                              const int (&off)[T::NL],
                                              f32x4 (&acc)[T::FI][T::FJ], int a_lo, int a_hi, int wc) {
  // this wave's A fragments: a_lo + i for the first FI/2, a_hi + (i - FI/2) for the rest
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (n_stages <= 0) return;   // uniform over the workgroup
  static_assert(T::KS == 2, "a stage row is one 128-byte line");
  const int my_a = wave * T::WF * 128, my_b = (T::FA + wave * T::WF) * 128;   // first slots of this wave's blocks
  const int n = lane & 15, g = lane >> 4;
  const int xs = ((n & 7) ^ (n >> 3)) * 8;                             // rows of odd blocks are swapped in pairs
  const int rd0 = (n >> 3) * 64 + xs + (g ^ (n & 7));         // this lane's slot when reading K-step 0
  const int rd1 = (n >> 3) * 64 + xs + ((4 + g) ^ (n & 7));   // and K-step 1
  auto fill = [&](int st, uint4 *buf) {
    const uint16_t *pa = base_a(st), *pb = base_b(st);
#pragma unroll
    for (int i = 0; i < T::NL / 2; ++i) {
      load_to_lds16(pa + off[i], buf + my_a + i * 64);
      load_to_lds16(pb + off[T::NL / 2 + i], buf + my_b + i * 64);
    }
  };
  fill(0, lds);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int st = 0; st < n_stages; ++st) {
    const uint4 *cur = lds + (st & 1) * T::STAGE_VEC;
#pragma unroll
    for (int ks = 0; ks < T::KS; ++ks) {
      // the next stage's loads go out first (its buffer was released by the barrier that ended
      // the previous stage) and have the whole stage's matrix work to arrive in
      if (ks == 0 && st + 1 < n_stages) fill(st + 1, lds + ((st + 1) & 1) * T::STAGE_VEC);   // uniform branch
      uint4 a[T::FI], b[T::FJ];
#pragma unroll
      for (int i = 0; i < T::FI; ++i)
        a[i] = cur[(i < T::FI / 2 ? a_lo + i : a_hi + i - T::FI / 2) * 128 + (ks ? rd1 : rd0)];
#pragma unroll
      for (int j = 0; j < T::FJ; ++j) b[j] = cur[(T::FA + wc * T::FJ + j) * 128 + (ks ? rd1 : rd0)];
#pragma unroll
      for (int i = 0; i < T::FI; ++i)
#pragma unroll
        for (int j = 0; j < T::FJ; ++j) acc[i][j] = mfma16(a[i], b[j], acc[i][j]);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of the next stage is in LDS
    __syncthreads();
  }
}

// Which piece of the tile lane `lane` fetches with its load i: operand (A or B), fragment
// relative to the wave's first one, row of the fragment, 16-byte piece of the stage's row.
template <typename T>
__device__ __forceinline__ void load_role(int i, int lane, bool &is_b, int &f_rel, int &rf, int &piece) {
  if constexpr (T::RING) {
    is_b = i >= T::WF;
    f_rel = i % T::WF;
    rf = lane >> 2;
    piece = (lane & 3) ^ ((rf >> 2) & 3);
  } else {
    const int h = i % 2, r = (lane >> 3) ^ h;   // block of the fragment, row of the block
    is_b = i >= T::NL / 2;
    f_rel = (i % (T::NL / 2)) / 2;
    rf = h * 8 + r;
    piece = (lane & 7) ^ r;   // piece (j & 7) XOR r of the row's line
  }
}

// The 256 x 256 tile's pipeline.  With two 64 KiB stages a CU has one stage of loads in flight
// for about half a stage of matrix work; a loaded round trip to L2 is far longer than that and
// the matrix cores waited (stage period 2.2 us for 0.85 us of matrix work).  Here the 160 KiB of
// LDS are five buffers of one K-step each (32 contraction elements of all 512 operand rows,
// 32 KiB).  Loads are issued a pair of K-steps (one 128-byte line per row) at a time, the two
// 64-byte halves of a line back to back by the same lanes, into two different buffers: pair j + 2
// goes out in the middle of pair j, so every pair has one and a half pairs of matrix work to
// arrive in and up to 128 KiB per CU are in flight.  Buffer of K-step h: h mod 5.
//   fragment F of a buffer: 1 KiB = 16 rows x 64 bytes; lane j of the load fetches row j >> 2,
//   piece (j & 3) XOR ((j >> 4) & 3), which lands at slot j; the fragment read of lane (n, g)
//   takes slot 4 n + (g XOR (n >> 2)): for one g the 16 lanes touch 16 different 16-byte bank
//   groups.
// Loads return in issue order, so `s_waitcnt vmcnt(loads of one pair)` is "the older pair has
// landed" while the newest stays in flight.
template <typename T, typename BaseA, typename BaseB>
__device__ __forceinline__ void gemm_mainloop_ring(uint4 *lds, int n_pairs, BaseA base_a, BaseB base_b,
                                                   const int (&off)[T::NOFF], f32x4 (&acc)[T::FI][T::FJ], int a_lo,
                                                   int a_hi, int wc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (n_pairs <= 0) return;   // uniform over the workgroup
  constexpr int HV = T::HALF_VEC;
  constexpr int kPairLoads = 4 * T::WF;   // loads a wave issues per pair
  const int my_a = wave * T::WF * 64, my_b = (T::FA + wave * T::WF) * 64;
  const int n = lane & 15, g = lane >> 4;
  const int rd = n * 4 + (g ^ ((n >> 2) & 3));
  auto issue = [&](int pair, int b0, int b1) {
    const uint16_t *pa = base_a(pair), *pb = base_b(pair);
    uint4 *d0 = lds + b0 * HV, *d1 = lds + b1 * HV;
#pragma unroll
    for (int i = 0; i < T::WF; ++i) {
      load_to_lds16(pa + off[i], d0 + my_a + i * 64);
      load_to_lds16(pa + off[i] + 32, d1 + my_a + i * 64);
      load_to_lds16(pb + off[T::WF + i], d0 + my_b + i * 64);
      load_to_lds16(pb + off[T::WF + i] + 32, d1 + my_b + i * 64);
    }
  };
  // Fragment reads run one K-step ahead of the matrix work, into a second set of operand
  // registers: the reads of K-step h + 1 are issued in the middle of K-step h, right after the
  // barrier that says its buffer is complete, and their latency is covered by the second half of
  // K-step h's MFMAs.  One barrier per K-step: it also tells that every wave has finished reading
  // K-step h's buffer (each wave's reads completed before its first MFMA of the step), so the
  // loads issued after it may overwrite that buffer and the one of K-step h - 1.
  auto read = [&](uint4 (&a)[T::FI], uint4 (&b)[T::FJ], const uint4 *cur) {
#pragma unroll
    for (int j = 0; j < T::FJ; ++j) b[j] = cur[(T::FA + wc * T::FJ + j) * 64 + rd];
#pragma unroll
    for (int i = 0; i < T::FI; ++i) a[i] = cur[(i < T::FI / 2 ? a_lo + i : a_hi + i - T::FI / 2) * 64 + rd];
  };
  auto mma = [&](const uint4 (&a)[T::FI], const uint4 (&b)[T::FJ], int i_lo, int i_hi) {
#pragma unroll
    for (int i = i_lo; i < i_hi; ++i)
#pragma unroll
      for (int j = 0; j < T::FJ; ++j) acc[i][j] = mfma16(a[i], b[j], acc[i][j]);
  };
  auto buf = [&](int b) { return lds + (b >= 5 ? b - 5 : b) * HV; };
  uint4 a0[T::FI], b0[T::FJ], a1[T::FI], b1[T::FJ];
  issue(0, 0, 1);
  if (n_pairs > 1) {
    issue(1, 2, 3);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kPairLoads) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  read(a0, b0, lds);
  int b = 0;   // buffer of the pair's first K-step
  for (int j = 0; j < n_pairs; ++j) {
    // K-step 2 j: operands in (a0, b0)
    mma(a0, b0, 0, T::FI / 2);
    __syncthreads();
    if (j + 2 < n_pairs) issue(j + 2, b + 4 >= 5 ? b - 1 : b + 4, b);   // uniform branch
    read(a1, b1, buf(b + 1));
    mma(a0, b0, T::FI / 2, T::FI);
    // K-step 2 j + 1: operands in (a1, b1)
    mma(a1, b1, 0, T::FI / 2);
    if (j + 1 < n_pairs) {
      // pair j + 1 has landed (the loads of pair j + 2, if any, stay in flight)
      if (j + 2 < n_pairs) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kPairLoads) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      read(a0, b0, buf(b + 2));
    }
    mma(a1, b1, T::FI / 2, T::FI);
    b = b + 2 >= 5 ? b - 3 : b + 2;
  }
}

template <typename T, typename BaseA, typename BaseB>
__device__ __forceinline__ void run_mainloop(uint4 *lds, int n_stages, BaseA base_a, BaseB base_b,
                                             const int (&off)[T::NOFF], f32x4 (&acc)[T::FI][T::FJ], int a_lo, int a_hi,
                                             int wc) {
  if constexpr (T::RING) gemm_mainloop_ring<T>(lds, n_stages, base_a, base_b, off, acc, a_lo, a_hi, wc);
  else gemm_mainloop<T>(lds, n_stages, base_a, base_b, off, acc, a_lo, a_hi, wc);
}

// ------------------------------------------------------------------------------------------------ up

template <typename T, int NM>
__global__ __launch_bounds__(T::THREADS) void up_gemm_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const uint16_t *__restrict__ xb,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ items, const int32_t *__restrict__ total_ptr, const int32_t *__restrict__ lists,
    const int32_t *__restrict__ counts, int k, int tiles_t, int tiles_j, size_t x_plane, uint16_t *__restrict__ H) {
  extern __shared__ uint4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4;
  const int E = L.E, d = L.d, d_e = L.d_e;
  // Workgroups go to the 8 XCDs round robin (workgroup v runs on XCD v mod 8) and each XCD has
  // its own L2: the tiles of one item share the expert's weight rows, so they are given ids that
  // differ by multiples of 8 and meet in one L2; the weights cross the fabric once per item.
  const int per_item = tiles_t * tiles_j;
  const int q = blockIdx.x >> 3, within = q % per_item;
  const int item = (q / per_item) * 8 + (blockIdx.x & 7);
  if (item >= *total_ptr) return;
  const int tt = within / tiles_j, tj = within % tiles_j;
  const int code = items[item];
  const int64_t c = code / E;
  const int s = code - (int)c * E;
  const int e = active_idx ? active_idx[c * E + s] : s;
  // a list entry outside [0, E) (an invalid input) is an empty slot: its rows of H stay zero
  if ((unsigned)e >= (unsigned)E) return;   // uniform over the workgroup
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int t0 = tt * T::TN;
  // with token lists the tile's columns are the expert's own tokens list[t0 ..]; H was zeroed and
  // the rows of the other tokens stay zero
  const int32_t *list = lists ? lists + ((size_t)c * E + e) * k : nullptr;
  const int m_e = lists ? min(max(counts[(size_t)c * E + e], 0), k) : k;
  if (t0 >= m_e) return;   // uniform over the workgroup
  constexpr int kNeurons = T::TM / NM;   // neurons per workgroup
  const int j0 = tj * kNeurons;
  const size_t w_expert = ((size_t)layer * E + e) * d_e;
  const int wr = wave % T::WR, wc = wave / T::WR;

  // A fragment f: gated: f < FA/2 -> W_up rows j0 + 16 f, else W_gate rows j0 + 16 (f - FA/2);
  // Eq. 2: W_up rows j0 + 16 f.  B fragment f: tokens t0 + 16 f.  A token index past the chunk
  // is clamped: its column of the product comes from a valid row and is never stored.
  const int f0 = wave * T::WF;   // first fragment of each operand this wave loads
  const bool gate_wave = NM == 2 && f0 >= T::FA / 2;
  int off[T::NOFF];
#pragma unroll
  for (int i = 0; i < T::NOFF; ++i) {
    bool is_b;
    int f_rel, rf, piece;
    load_role<T>(i, lane, is_b, f_rel, rf, piece);
    const int f = f0 + f_rel;
    int row = j0 + (gate_wave ? f - T::FA / 2 : f) * 16 + rf;
    if (is_b) {
      const int idx = min(t0 + f * 16 + rf, m_e - 1);
      row = list ? list[idx] : idx;
    }
    off[i] = row * d + piece * 8;
  }
  const uint16_t *wsel = static_cast<const uint16_t *>(gate_wave ? L.w_gate : L.w_up) + w_expert * d;
  const uint16_t *xsel = xb + (size_t)c * k * d;
  // every tile of the launch reads the chunk's x: each starts at another stage of the
  // contraction, so that they do not all ask the L2 for the same lines at the same moment.
  // Stage (or pair of K-steps) 2 v is stage v of the contraction against the hi plane of x,
  // 2 v + 1 the same weight lines against the lo plane.
  const int n_st = d / T::TK, rot = (int)(((unsigned)item * 5u) % (unsigned)n_st);
  auto stage_of = [&](int st) { const int v = (st >> 1) + rot; return v >= n_st ? v - n_st : v; };
  auto base_a = [&](int st) { return wsel + (size_t)stage_of(st) * T::TK; };
  auto base_b = [&](int st) { return xsel + (st & 1 ? x_plane : (size_t)0) + (size_t)stage_of(st) * T::TK; };

  f32x4 acc[T::FI][T::FJ];
#pragma unroll
  for (int i = 0; i < T::FI; ++i)
#pragma unroll
    for (int j = 0; j < T::FJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  // this wave's A fragments: gated: FI/2 up fragments and the FI/2 matching gate fragments
  const int a_lo = NM == 2 ? wr * (T::FI / 2) : wr * T::FI;
  const int a_hi = NM == 2 ? T::FA / 2 + wr * (T::FI / 2) : wr * T::FI + T::FI / 2;
  // score and mask bit of this lane's tokens: requested before the contraction so that the
  // epilogue does not start with a round trip to memory
  const int n = lane & 15;
  float f_tok[T::FJ];
  int tok_of[T::FJ];   // the chunk's token behind column j of this lane, -1 past the list
#pragma unroll
  for (int j = 0; j < T::FJ; ++j) {
    const int idx = t0 + (wc * T::FJ + j) * 16 + n;
    const int t = idx < m_e ? (list ? list[idx] : idx) : -1;
    tok_of[j] = t;
    f_tok[j] = 0.0f;
    if (t >= 0) {
      const int64_t tok = c * k + t;
      const bool on = token_mask ? (bool)((token_mask[tok * L.W + (e >> 6)] >> (e & 63)) & 1) : true;
      f_tok[j] = on ? scores[tok * E + e] : 0.0f;
    }
  }
  run_mainloop<T>(lds, 2 * (d / T::TK), base_a, base_b, off, acc, a_lo, a_hi, wc);

  // D[i = neuron 4g + q of the fragment][j = token n of the fragment]
#pragma unroll
  for (int j = 0; j < T::FJ; ++j) {
    const int t = tok_of[j];
    if (t < 0) continue;
    const bool on = f_tok[j] != 0.0f;   // a masked term, and one scaled by a zero score, store +0
    const float f = f_tok[j];
    constexpr int kOut = T::FI / NM;
#pragma unroll
    for (int i = 0; i < kOut; ++i) {
      uint32_t p[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float u = acc[i][j][q];
        const float h = NM == 2 ? swish_fast(acc[i + (NM - 1) * kOut][j][q]) * u : swish_fast(u);
        p[q] = bf16_bits(on ? f * h : 0.0f);
      }
      const int neuron = j0 + (wr * kOut + i) * 16 + 4 * g;
      *reinterpret_cast<uint2 *>(H + (((size_t)c * E + s) * k + t) * d_e + neuron) =
          make_uint2(p[0] | p[1] << 16, p[2] | p[3] << 16);
    }
  }
}

// ------------------------------------------------------------------------------------------------ down

template <typename T>
__global__ __launch_bounds__(T::THREADS) void down_gemm_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int k, int tiles_t, int tiles_c, int splits, int64_t n_groups,
    const uint16_t *__restrict__ H, float *__restrict__ out, size_t split_stride) {
  extern __shared__ uint4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4;
  const int E = L.E, d = L.d, d_e = L.d_e;
  // all tiles of one (chunk, split) on one XCD (ids differing by multiples of 8): they share the
  // split's W_down rows (the token tiles) and its mid rows (the column tiles) in that XCD's L2
  const int per_group = tiles_t * tiles_c;
  const int q = blockIdx.x >> 3, within = q % per_group;
  const int64_t grp = (int64_t)(q / per_group) * 8 + (blockIdx.x & 7);
  if (grp >= n_groups) return;   // uniform over the workgroup
  const int sp = (int)(grp % splits);
  const int64_t c = grp / splits;
  const int tc = within % tiles_c, tt = within / tiles_c;
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int n_act = active_idx ? min(max(n_active[c], 0), E) : E;
  const int s_lo = (int)((int64_t)n_act * sp / splits), s_hi = (int)((int64_t)n_act * (sp + 1) / splits);
  const int t0 = tt * T::TN, col0 = tc * T::TM;
  const int wr = wave % T::WR, wc = wave / T::WR;
  const int st_per_slot = d_e / T::TK;

  // A fragment f: W_down rows col0 + 16 f of the stage's expert; B fragment f: mid rows of tokens
  // t0 + 16 f (clamped as in the up kernel) of the stage's slot.
  const int f0 = wave * T::WF;   // first fragment of each operand this wave loads
  int off[T::NOFF];
#pragma unroll
  for (int i = 0; i < T::NOFF; ++i) {
    bool is_b;
    int f_rel, rf, piece;
    load_role<T>(i, lane, is_b, f_rel, rf, piece);
    const int f = f0 + f_rel;
    const int row = is_b ? min(t0 + f * 16 + rf, k - 1) : col0 + f * 16 + rf;
    off[i] = row * d_e + piece * 8;
  }
  auto base_a = [&](int st) -> const uint16_t * {
    const int s = s_lo + st / st_per_slot;
    int e = active_idx ? active_idx[c * E + s] : s;
    e = min(max(e, 0), E - 1);
    return static_cast<const uint16_t *>(L.w_down) + ((size_t)layer * E + e) * d * d_e +
           (size_t)(st % st_per_slot) * T::TK;
  };
  auto base_b = [&](int st) -> const uint16_t * {
    const int s = s_lo + st / st_per_slot;
    return H + ((size_t)c * E + s) * k * d_e + (size_t)(st % st_per_slot) * T::TK;
  };

  f32x4 acc[T::FI][T::FJ];
#pragma unroll
  for (int i = 0; i < T::FI; ++i)
#pragma unroll
    for (int j = 0; j < T::FJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  run_mainloop<T>(lds, (s_hi - s_lo) * st_per_slot, base_a, base_b, off, acc, wr * T::FI, wr * T::FI + T::FI / 2, wc);

  const int n = lane & 15;
  float *dst = out + (size_t)sp * split_stride;
#pragma unroll
  for (int j = 0; j < T::FJ; ++j) {
    const int t = t0 + (wc * T::FJ + j) * 16 + n;
    if (t >= k) continue;
#pragma unroll
    for (int i = 0; i < T::FI; ++i) {
      const int col = col0 + (wr * T::FI + i) * 16 + 4 * g;
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

// 256-wide tiles when the chunk fills them and the shape divides; else 128-wide.
bool big_up(const LayerView &L, int k, bool gated) {
  return k >= 192 && L.d % 256 == 0 && L.d_e % (gated ? 128 : 256) == 0;
}
bool big_down(const LayerView &L, int k) { return k >= 192 && L.d % 256 == 0; }

int down_splits(const LayerView &L, int64_t n_chunks, int k) {
  const bool big = big_down(L, k);
  const int tile = big ? 256 : 128, want = big ? 256 : 512;
  const int64_t base = n_chunks * ((k + tile - 1) / tile) * (L.d / tile);
  if (base >= want) return 1;
  return (int)std::min<int64_t>(16, (want + base - 1) / base);
}

struct GemmWs {
  uint16_t *xb, *H;
  int32_t *total, *items;
  int32_t *lists, *counts;   // per (chunk, expert): its tokens
  float *part;
};

GemmWs carve(const LayerView &L, int64_t n_chunks, int k, void *ws) {
  char *p = static_cast<char *>(ws);
  GemmWs w;
  w.xb = reinterpret_cast<uint16_t *>(p);   // two planes: bf16 hi, bf16 lo
  p += align256((size_t)n_chunks * k * L.d * 2 * 2);
  w.H = reinterpret_cast<uint16_t *>(p);
  p += align256((size_t)n_chunks * L.E * k * L.d_e * 2);
  w.total = reinterpret_cast<int32_t *>(p);
  w.items = w.total + 64;
  p += align256(((size_t)n_chunks * L.E + 64) * sizeof(int32_t));
  w.lists = reinterpret_cast<int32_t *>(p);
  p += align256((size_t)n_chunks * L.E * k * sizeof(int32_t));
  w.counts = reinterpret_cast<int32_t *>(p);
  p += align256((size_t)n_chunks * L.E * sizeof(int32_t));
  w.part = reinterpret_cast<float *>(p);
  return w;
}

template <typename T>
hipError_t launch_up_tile(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *scores,
                          const uint64_t *token_mask, const int32_t *active_idx, const GemmWs &w, int64_t n_chunks,
                          int k, hipStream_t s) {
  const int tiles_t = (k + T::TN - 1) / T::TN, tiles_j = L.d_e / (T::TM / (gated ? 2 : 1));
  const int64_t grid = (n_chunks * L.E + 7) / 8 * 8 * tiles_t * tiles_j;   // items rounded up to the 8 XCDs
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  const int32_t *lists = token_mask ? w.lists : nullptr;   // no mask: every token has every expert
  static PerDeviceOnce lds_limit;   // one per tile type
  const hipError_t e = lds_limit.run([&] {
    const hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void *>(up_gemm_kernel<T, 1>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    const hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void *>(up_gemm_kernel<T, 2>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    return e1 != hipSuccess ? e1 : e2;
  });
  if (e != hipSuccess) return e;
  const size_t x_plane = (size_t)n_chunks * k * L.d;   // elements between the hi and the lo plane of x
  if (gated)
    hipLaunchKernelGGL((up_gemm_kernel<T, 2>), dim3((unsigned)grid), dim3(T::THREADS), T::LDS_BYTES, s, L, chunk_layer,
                       w.xb, scores, token_mask, active_idx, w.items, w.total, lists, w.counts, k, tiles_t, tiles_j,
                       x_plane, w.H);
  else
    hipLaunchKernelGGL((up_gemm_kernel<T, 1>), dim3((unsigned)grid), dim3(T::THREADS), T::LDS_BYTES, s, L, chunk_layer,
                       w.xb, scores, token_mask, active_idx, w.items, w.total, lists, w.counts, k, tiles_t, tiles_j,
                       x_plane, w.H);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_down_tile(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, int splits, const uint16_t *H,
                            float *out, size_t stride, hipStream_t s) {
  const int tiles_t = (k + T::TN - 1) / T::TN, tiles_c = L.d / T::TM;
  const int64_t n_groups = n_chunks * splits;
  const int64_t grid = (n_groups + 7) / 8 * 8 * tiles_t * tiles_c;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  static PerDeviceOnce lds_limit;   // one per tile type
  const hipError_t e = lds_limit.run([&] {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(down_gemm_kernel<T>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
  });
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((down_gemm_kernel<T>), dim3((unsigned)grid), dim3(T::THREADS), T::LDS_BYTES, s, L, chunk_layer,
                     active_idx, n_active, k, tiles_t, tiles_c, splits, n_groups, H, out, stride);
  return hipGetLastError();
}

}  // namespace

bool gemm_supported(const LayerView &L, int wdtype, int k, bool gated) {
  return wdtype == BLOCKFFN_BF16 && k > 32 && L.d % 128 == 0 && L.d_e % (gated ? 64 : 128) == 0;
}

size_t gemm_workspace_bytes(const LayerView &L, int64_t n_chunks, int k) {
  const int splits = down_splits(L, n_chunks, k);
  size_t b = align256((size_t)n_chunks * k * L.d * 2 * 2) + align256((size_t)n_chunks * L.E * k * L.d_e * 2) +
             align256(((size_t)n_chunks * L.E + 64) * sizeof(int32_t)) +
             align256((size_t)n_chunks * L.E * k * sizeof(int32_t)) + align256((size_t)n_chunks * L.E * sizeof(int32_t));
  if (splits > 1) b += align256((size_t)splits * n_chunks * k * L.d * sizeof(float));
  return b;
}

hipError_t launch_up_gemm(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                          const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                          const int32_t *n_active, int64_t n_chunks, int k, void *ws, hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  GemmWs w = carve(L, n_chunks, k, ws);
  const size_t n8 = (size_t)n_chunks * k * L.d / 8;
  const size_t n16 = token_mask ? (size_t)n_chunks * L.E * k * L.d_e / 8 : 0;
  const int64_t n_pairs = token_mask ? n_chunks * L.E : 0;
  const int cvt_blocks = (int)std::min<size_t>((n8 + kThreads - 1) / kThreads, 2048);
  const int zero_blocks = (int)std::min<size_t>((n16 + kThreads - 1) / kThreads, 2048);
  const int64_t list_blocks = (n_pairs + kThreads / 64 - 1) / (kThreads / 64);
  if (cvt_blocks + zero_blocks + list_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(prepare_kernel, dim3((unsigned)(cvt_blocks + zero_blocks + list_blocks)), dim3(kThreads), 0, s, x,
                     w.xb, n8, cvt_blocks, reinterpret_cast<uint4 *>(w.H), n16, zero_blocks, token_mask, L.W, L.E, k,
                     n_pairs, w.lists, w.counts);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  err = launch_worklist(n_active, n_chunks, L.E, 1, w.items, w.total, s);
  if (err != hipSuccess) return err;
  // With token lists an expert's tile has about k / 5 columns (102 of 512): 128 token columns hold
  // them, and the 256-wide tile would spend more than half of its matrix work on padding.
  if (big_up(L, k, gated) && !token_mask)
    return launch_up_tile<TileBig>(L, gated, chunk_layer, scores, token_mask, active_idx, w, n_chunks, k, s);
  return launch_up_tile<TileSmall>(L, gated, chunk_layer, scores, token_mask, active_idx, w, n_chunks, k, s);
}

hipError_t launch_down_gemm(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, const void *ws, float *y,
                            hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  GemmWs w = carve(L, n_chunks, k, const_cast<void *>(ws));
  const int splits = down_splits(L, n_chunks, k);
  const size_t stride = (size_t)n_chunks * k * L.d;
  float *out = splits > 1 ? w.part : y;
  hipError_t err =
      big_down(L, k)
          ? launch_down_tile<TileBig>(L, chunk_layer, active_idx, n_active, n_chunks, k, splits, w.H, out, stride, s)
          : launch_down_tile<TileSmall>(L, chunk_layer, active_idx, n_active, n_chunks, k, splits, w.H, out, stride, s);
  if (err != hipSuccess || splits == 1) return err;
  const size_t n4 = stride / 4;
  hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)std::min<size_t>((n4 + kThreads - 1) / kThreads, 4096)),
                     dim3(kThreads), 0, s, w.part, splits, stride, n4, y);
  return hipGetLastError();
}

}  // namespace blockffn
