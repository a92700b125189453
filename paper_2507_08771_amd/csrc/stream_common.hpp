// What the weight-streaming kernels of ffn_stream.hip and the single-launch kernel for a few chunks
// (ffn_few.hip) share: the matrix-core step, the bf16 hi/lo split of an fp32 value, the layout
// of mid at k <= 8 and the carving of the workspace.
#pragma once

#include <algorithm>

#include "common.hpp"

namespace blockffn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kStreamThreads = 256;

__device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

__device__ __forceinline__ uint32_t bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}

// ---- the weight stream: non-temporal loads of whole 128-byte lines
//
// Every weight byte is used once per launch, so nothing is gained by keeping it in the caches,
// and a read stream of non-temporal loads runs at 7.1-7.2 TB/s on this chip where plain loads
// reach 6.3-6.5 - provided a load instruction takes whole 128-byte lines (eight neighbouring
// lanes per line).  With the 64-byte half lines of the matrix core's operand order (lane = 16 g +
// row: 16 bytes of 16 rows per group of 16 lanes) non-temporal loads are slower than plain ones
// (6.0 TB/s): the other half of a line is fetched again.  So a 16-row tile is requested as two
// registers per line index: `lo8` = the line of rows 0-7, `hi8` = of rows 8-15, lane = 8 row +
// piece, and the two A operands the line holds (K-steps 2p and 2p + 1: its first and second 64
// bytes) are put together in registers: one ds_bpermute per dword brings, for its eight rows,
// K-step 2p to the lanes of rows 0-7 and K-step 2p + 1 to the lanes of rows 8-15; a DPP move
// (rotate by 8 within the 16 lanes of a row group, written to half of the lanes) then swaps
// what sits in the wrong half between the two.  x, mid, scores and lists, which other
// workgroups read again, keep plain loads.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const void *p) {
  const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
// 8 bytes of mid (k <= 8, where the 64 lanes of a store cover 512 contiguous bytes), written once
// and read once by a later launch: a non-temporal store.  The few
// stores of the up projection (0.4 % of its bytes at k = 8) cost 8 % of its time as plain stores
// - the launch is a pure read stream but for them - and half of that as non-temporal ones.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_stream(uint2 *p, uint2 v) {
  const u32x2_t w = {v.x, v.y};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x2_t *>(p));
}
// 16 bytes of y, written once per launch and not read by it: non-temporal as well (`spec_k8`:
// streaming down kernel - 3.6 %).
typedef float f32x4_nt_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream(float4 *p, float4 v) {
  const f32x4_nt_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<f32x4_nt_t *>(p));
}
// row within the first eight rows of a tile and byte offset within a line, of this lane's loads
__device__ __forceinline__ int line_row(int lane) { return lane >> 3; }
__device__ __forceinline__ int line_byte(int lane) { return (lane & 7) * 16; }
// ds_bpermute address: the operand's lane (g, r) reads lane 8 (r & 7) + 4 (r >> 3) + g
__device__ __forceinline__ int line_src(int lane) {
  const int r = lane & 15, g = lane >> 4;
  return ((r & 7) * 8 + 4 * (r >> 3) + g) * 4;
}
template <int BANKS>   // `src` rotated by 8 lanes within each group of 16, written to the 4-lane banks in BANKS; `old` elsewhere
__device__ __forceinline__ uint32_t ror8_into(uint32_t old, uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, 0x128, 0xf, BANKS, false);
}
__device__ __forceinline__ void line_operands(uint4 lo8, uint4 hi8, int src_bytes, uint4 &f0, uint4 &f1) {
  const uint32_t l[4] = {lo8.x, lo8.y, lo8.z, lo8.w}, h[4] = {hi8.x, hi8.y, hi8.z, hi8.w};
  uint32_t a[4], b[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t dl = (uint32_t)__builtin_amdgcn_ds_bpermute(src_bytes, (int)l[q]);   // rows 0-7: K-step 2p | 2p + 1
    const uint32_t dh = (uint32_t)__builtin_amdgcn_ds_bpermute(src_bytes, (int)h[q]);   // rows 8-15: likewise
    a[q] = ror8_into<0xc>(dl, dh);   // lanes of rows 8-15 take K-step 2p of rows 8-15
    b[q] = ror8_into<0x3>(dh, dl);   // lanes of rows 0-7 take K-step 2p + 1 of rows 0-7
  }
  f0 = make_uint4(a[0], a[1], a[2], a[3]);
  f1 = make_uint4(b[0], b[1], b[2], b[3]);
}

// x = hi + lo with hi = bf16(x) and lo = bf16(x - hi); 16-bit patterns in the low halves
__device__ __forceinline__ void split_bf16(float x, uint32_t &hi, uint32_t &lo) {
  hi = bf16_bits(x);
  lo = bf16_bits(x - __uint_as_float(hi << 16));
}

// mid in memory, k <= 8 (one B fragment per K-step): in the order the down kernel's B operand is
// read from LDS, [chunk][slot][K-step = d_e / 32][64 lanes] of 8 bf16, lane gg * 16 + n holding the
// expert's neurons 32 * K-step + 8 gg .. + 7 for fragment column n (0-7: hi of tokens 0-7, 8-15:
// their lo).  The up kernels hold, per lane (n, g) of row tile T, the four neurons 16 T + 4 g .. + 3:
// half (g & 1) of the 16-byte entry of lane (2 (T & 1) + g / 2) * 16 + n in K-step T / 2, so the 64
// lanes of one store cover 512 contiguous bytes and the down kernel's staging is a linear copy.
__device__ __forceinline__ uint2 *mid_entry(uint16_t *midB, size_t kstep0, int T, int g, int n) {
  const size_t entry = (kstep0 + (T >> 1)) * 64 + ((T & 1) * 2 + (g >> 1)) * 16 + n;
  return reinterpret_cast<uint2 *>(midB) + entry * 2 + (g & 1);
}

// ------------------------------------------------------------------------------------------------ workspace

inline int b_frags(int k) { return k <= 8 ? 1 : (k <= 16 ? 2 : 4); }

struct StreamWs {
  uint16_t *midB;
  int32_t *items, *total;
  uint32_t *tok_bits;    // [chunk * E + slot]: the tokens whose rows of mid are written (k > 8)
  const uint4 *zero16;   // 16 bytes of zeros, written with the work list
  uint4 *xS;     // the chunks' x split into bf16 hi/lo in B-operand order
  float *part;   // partial sums of the split down projection (few chunks only)
};

inline size_t xs_bytes(const LayerView &L, int64_t n_chunks, int k) {
  return (size_t)n_chunks * (L.d / 32) * b_frags(k) * 64 * sizeof(uint4);   // a multiple of 1024
}

inline size_t mid_bytes(const LayerView &L, int64_t n_chunks, int k) {
  return ((size_t)n_chunks * L.E * b_frags(k) * 16 * L.d_e * 2 + 255) & ~(size_t)255;
}

inline size_t item_bytes(const LayerView &L, int64_t n_chunks) {
  // 64 words of counters and constants, the item list, the token bits of every slot
  return (((size_t)n_chunks * L.E * 2 + 64) * sizeof(int32_t) + 255) & ~(size_t)255;
}

inline StreamWs carve_stream(const LayerView &L, int64_t n_chunks, int k, void *ws) {
  char *p = static_cast<char *>(ws);
  StreamWs w;
  w.midB = reinterpret_cast<uint16_t *>(p);
  w.total = reinterpret_cast<int32_t *>(p + mid_bytes(L, n_chunks, k));
  w.items = w.total + 64;
  w.tok_bits = reinterpret_cast<uint32_t *>(w.items + (size_t)n_chunks * L.E);
  w.zero16 = reinterpret_cast<const uint4 *>(w.total + 16);
  w.xS = reinterpret_cast<uint4 *>(p + mid_bytes(L, n_chunks, k) + item_bytes(L, n_chunks));
  w.part = reinterpret_cast<float *>(p + mid_bytes(L, n_chunks, k) + item_bytes(L, n_chunks) + xs_bytes(L, n_chunks, k));
  return w;
}

// Few chunks: narrow column blocks (8 fragments per slot and wave) and up to 8 slot splits, so
// that one chunk still spreads over the whole chip.  0: the wide, unsplit configuration.
inline int down_splits(const LayerView &L, int64_t n_chunks) {
  const int64_t wide = n_chunks * (L.d / 512);
  if (wide >= 2 * num_cus()) return 0;
  const int ksd = L.d_e / 32;
  const int64_t narrow = n_chunks * (L.d / (64 * (8 / ksd)));
  return (int)std::min<int64_t>(8, std::max<int64_t>(1, (num_cus() + narrow - 1) / narrow));
}

// A launch with this few (chunk, slot) pairs cannot occupy the chip with one workgroup per pair:
// the up projection runs one workgroup per (pair, 16-row tile) with the contraction split over the
// waves (k <= 8, d = 1024 or 2048).
inline bool few_chunks(const LayerView &L, int64_t n_chunks, int k) {
  return k <= 8 && n_chunks * L.E <= 2048 && (L.d == 1024 || L.d == 2048);
}

// k = 1 on the many-chunk streaming kernels: of the 16 columns of mid's k <= 8 layout only two
// hold anything (the token's hi and lo parts), and what a store costs the weight stream goes by
// the 128-byte lines it touches, not by its bytes (32 lines per slot at d_e = 128, mostly zeros).
// Mid is then [chunk][slot][hi | lo][d_e] bf16: 4 lines per slot; the down kernel stages the
// other 14 columns from a block of zeros.  (`decode_k1`: up kernel - 4.3 %.)  The chunk's split x
// likewise keeps its two columns only (split_x1_kernel).
inline bool mid_one_token(const LayerView &L, int64_t n_chunks, int k) {
  return k == 1 && n_chunks >= 64 && !few_chunks(L, n_chunks, k);
}

}  // namespace blockffn
