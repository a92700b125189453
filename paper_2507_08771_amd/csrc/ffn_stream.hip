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
//         is written already split into bf16 hi/lo: in the B-operand order of the down kernel at
//         k <= 8, token-major with the rows of absent tokens left out at k > 8.
//   down  grid (chunk, 512 output columns); the reduction runs over the union's slots and the
//         expert's neurons; mid of the next slot is staged through LDS (double buffered) while
//         the current slot's W_down rows stream; one writer per output element.
#include "stream_common.hpp"

namespace blockffn {

namespace {

constexpr int kThreads = kStreamThreads;
constexpr int kRing = 16;          // 128-bit loads in flight per lane
constexpr int kXBytes = 64 * 1024; // LDS for the split activations of one K-chunk

constexpr int acc_tiles(int NB) { return NB == 4 ? 2 : 1; }
constexpr int acc_of(int NB, int bf) { return NB == 4 ? bf / 2 : 0; }
constexpr int tokens_of(int NB) { return NB == 1 ? 8 : (NB == 2 ? 16 : 32); }
// Slots per item of the double-buffered up kernel: as many as keep the accumulators at 16 tiles
// (NB = 4) or 8 tiles (more spilled), at most 4; with 1 the single-buffer kernel is used.
constexpr int up_group(int NB, int RT, int NM) {
  const int per_slot = RT * NM * acc_tiles(NB), cap = NB == 4 ? 16 : 8;
  return cap / per_slot > 4 ? 4 : (cap / per_slot < 1 ? 1 : cap / per_slot);
}

// Groups of four waves per workgroup of the double-buffered up kernel.  Two where the accumulators
// allow the full four slots per group of waves: an item is then eight slots, and the chunk's x
// goes through LDS once per eight slots instead of four, with items no longer in time (k = 32,
// Eq. 2 experts of 128: the fills were 7 % of the kernel).
constexpr int up_halves(int NB, int RT, int NM) { return NB == 4 && up_group(NB, RT, NM) == 4 ? 2 : 1; }
// Shapes the double-buffered kernel takes (given more than one K-chunk): those where it holds more
// than one slot per group of waves; 8 fragments per tile (k > 16) need an even number of tiles
// per slot.  (One slot per group of waves, two groups: `tree_k32` 24.6 ms against 23.7 ms for the
// single-buffer kernel.)
constexpr bool up_db_shape(int NB, int RT, int NM) {
  return (NB == 2 || (NB == 4 && (RT * NM) % 2 == 0)) && up_group(NB, RT, NM) > 1;
}

// Flat work list: items[i] = chunk * E + slot for every `group`-th slot below n_active[chunk]
// (an item stands for up to `group` consecutive slots of one chunk).  The persistent workgroups
// take items at a fixed stride, so the list is ordered by size: first every item of `group`
// slots, chunk after chunk (pass 0), then the chunks' last, shorter items, longest first (pass p
// holds the chunks whose last item has group - p slots).  Every workgroup then gets the same
// number of full items (to within one) and the short ones fill the end of the launch; in chunk
// order a workgroup could draw several short items and another none (7 % between the busiest
// workgroup and the mean at 39 active experts per chunk, group = 4).
//
// One workgroup per 1024 chunks.  A chunk's place in the list depends on the counts of all chunks
// (earlier passes) and of the chunks before it (its own pass); instead of a scan across
// workgroups, which needs a second launch or workgroups waiting for each other, every workgroup
// counts for itself: the totals of each pass and what lies before its own first chunk.  That is
// one coalesced sweep over n_active per workgroup (64 workgroups x 256 KiB at 65 536 chunks),
// far less than a launch costs, and no workgroup ever waits for another.
constexpr int kListChunks = 1024;   // chunks per workgroup = threads per workgroup
constexpr int kMaxGroup = 8;

__device__ __forceinline__ int items_of(int n_act, int group, int pass, int &first) {
  const int full = n_act / group, rem = n_act - full * group;
  first = pass == 0 ? 0 : full;
  return pass == 0 ? full : (rem == group - pass ? 1 : 0);
}

__global__ __launch_bounds__(kListChunks) void worklist_kernel(const int32_t *__restrict__ n_active, int64_t n_chunks,
                                                               int E, int group, int32_t *__restrict__ items,
                                                               int32_t *__restrict__ total) {
  __shared__ int red[2 * kMaxGroup][kListChunks / 64];
  __shared__ int pass_base[kMaxGroup + 1];   // first list index of each pass for this workgroup's first chunk; [group]: list length
  __shared__ int wave_tot[kListChunks / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t c_first = (int64_t)blockIdx.x * kListChunks;
  auto n_act_of = [&](int64_t c) { return n_active ? min(max(n_active[c], 0), E) : E; };

  // all[p]: items of pass p over every chunk; before[p]: over the chunks ahead of this workgroup's
  int all[kMaxGroup], before[kMaxGroup];
#pragma unroll
  for (int p = 0; p < kMaxGroup; ++p) all[p] = before[p] = 0;
  for (int64_t c = tid; c < n_chunks; c += kListChunks) {
    const int n_act = n_act_of(c);
#pragma unroll
    for (int p = 0; p < kMaxGroup; ++p) {
      int first;
      const int n = p < group ? items_of(n_act, group, p, first) : 0;
      all[p] += n;
      before[p] += c < c_first ? n : 0;
    }
  }
#pragma unroll
  for (int p = 0; p < kMaxGroup; ++p) {
    int a = all[p], b = before[p];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      a += __shfl_xor(a, off, kWave);
      b += __shfl_xor(b, off, kWave);
    }
    if (lane == 0) {
      red[p][wave] = a;
      red[kMaxGroup + p][wave] = b;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int start = 0;
    for (int p = 0; p < group; ++p) {
      int a = 0, b = 0;
      for (int w = 0; w < kListChunks / 64; ++w) {
        a += red[p][w];
        b += red[kMaxGroup + p][w];
      }
      pass_base[p] = start + b;
      start += a;
    }
    pass_base[group] = start;
  }
  __syncthreads();

  const int64_t c = c_first + tid;
  const int n_act = c < n_chunks ? n_act_of(c) : 0;
  for (int pass = 0; pass < group; ++pass) {
    int first = 0;
    const int n = c < n_chunks ? items_of(n_act, group, pass, first) : 0;
    int incl = n;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, kWave);
      if (lane >= off) incl += v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int base = pass_base[pass];
    for (int w = 0; w < wave; ++w) base += wave_tot[w];
    const int start = base + incl - n;
    for (int s = 0; s < n; ++s) items[start + s] = (int32_t)(c * E + (first + s) * group);
    __syncthreads();   // wave_tot is rewritten by the next pass
  }
  if (blockIdx.x == 0) {
    if (tid == 0) *total = pass_base[group];
    if (tid < 4) total[16 + tid] = 0;   // the block of zeros the down kernel stages absent tokens from
  }
}

// ------------------------------------------------------------------------------------------------ x split

// x of every chunk split into bf16 hi/lo, stored in the B-operand order the up kernel reads from
// LDS: xS [chunk][K-step = d / 32][NB][64 lanes] of 8 bf16, lane = gg * 16 + n holding the 8
// contraction elements 8 * gg .. 8 * gg + 7 of the K-step for column n of the fragment.
// NB = 1: columns 0-7 are the hi parts of tokens 0-7, columns 8-15 their lo parts.
// NB = 2, 4: fragment 2 * grp is the hi part of tokens 16 * grp .. 16 * grp + 15, fragment
// 2 * grp + 1 their lo part.  Tokens at or above k are zero.  One thread per 16-byte entry.
template <int NB>
__global__ __launch_bounds__(kThreads) void split_x_kernel(const float *__restrict__ x, int64_t n_chunks, int k, int d,
                                                           uint4 *__restrict__ xS) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t per_chunk = (int64_t)(d / 32) * NB * 64;
  if (idx >= n_chunks * per_chunk) return;
  const int64_t c = idx / per_chunk;
  const int rem = (int)(idx - c * per_chunk);
  const int kstep = rem / (NB * 64), bf = (rem >> 6) % NB, lane = rem & 63;
  const int gg = lane >> 4, n = lane & 15;
  const int tok = NB == 1 ? (n & 7) : (bf >> 1) * 16 + n;
  const bool want_lo = NB == 1 ? n >= 8 : (bf & 1);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (tok < k) {
    const float4 *p = reinterpret_cast<const float4 *>(x + (c * k + tok) * d + kstep * 32 + gg * 8);
    const float4 a = p[0], b = p[1];
    const float xv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t h[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      uint32_t hi, lo;
      split_bf16(xv[q], hi, lo);
      h[q] = want_lo ? lo : hi;
    }
    v = make_uint4(h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16);
  }
  xS[idx] = v;
}

// ------------------------------------------------------------------------------------------------ up

// Router scores and mask words of the slot's tokens for expert e: what the epilogue multiplies
// with.  Requested when the slot starts (a load issued in the epilogue would return behind the
// ring's and stop the stream for a memory round trip), by LDS-direct loads into an area of the
// wave's own, [score, mask lo, mask hi][token]: loaded into registers they made the epilogue
// start with a wait for "every load so far" (the compiler cannot count across the loops in
// between), i.e. for the 16 loads of the ring, already refilled for the next slot - the ring
// drained once per slot, 8 % of the kernel at k = 8.  The kernel waits for them itself (they are
// older than the ring's loads, which return in order) and reads them from LDS.
// The loads are unconditional: a token past the chunk reads the chunk's last token.
__device__ __forceinline__ void request_scores(uint32_t (&area)[3][64], const LayerView &L,
                                               const float *__restrict__ scores,
                                               const uint64_t *__restrict__ token_mask, int64_t c, int e, int k, int lane) {
  const int64_t tok = c * k + min(lane & 31, k - 1);
  load_to_lds4(scores + tok * L.E + e, &area[0][0]);
  if (token_mask) {   // uniform over the launch
    const uint32_t *m = reinterpret_cast<const uint32_t *>(token_mask + tok * L.W + (e >> 6));
    load_to_lds4(m, &area[1][0]);
    load_to_lds4(m + 1, &area[2][0]);
  }
}

// 0 where the mask bit is clear, the token is past the chunk or the list entry was invalid
// One-token chunks on the many-chunk kernels (mid_one_token): of the 16 columns of the NB = 1
// layout only columns 0 (hi) and 8 (lo) hold anything, so xS keeps those two alone,
// [chunk][K-step][gg][hi, lo] of 8 bf16 (8 KiB per chunk at d = 2048 instead of 64), and the up
// kernel, which zeroes its LDS copy once, refills only them.  One thread per 16-byte entry.
__global__ __launch_bounds__(kThreads) void split_x1_kernel(const float *__restrict__ x, int64_t n_chunks, int d,
                                                            uint4 *__restrict__ xS) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t per_chunk = (int64_t)(d / 32) * 8;
  if (idx >= n_chunks * per_chunk) return;
  const int64_t c = idx / per_chunk;
  const int rem = (int)(idx - c * per_chunk);
  const int kstep = rem >> 3, gg = (rem >> 1) & 3;
  const bool want_lo = rem & 1;
  const float4 *p = reinterpret_cast<const float4 *>(x + c * d + kstep * 32 + gg * 8);
  const float4 a = p[0], b = p[1];
  const float xv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  uint32_t h[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    uint32_t hi, lo;
    split_bf16(xv[q], hi, lo);
    h[q] = want_lo ? lo : hi;
  }
  xS[idx] = make_uint4(h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16);
}

template <int NB>
__device__ __forceinline__ void read_scores(float (&f_tok)[acc_tiles(NB)], const uint32_t (&area)[3][64], bool has_mask,
                                            int e, bool valid, int k, int lane) {
  const int n = lane & 15;
#pragma unroll
  for (int q = 0; q < acc_tiles(NB); ++q) {
    const int t = NB == 1 ? (n & 7) : q * 16 + n;
    const uint32_t word = has_mask ? area[1 + ((e >> 5) & 1)][t] : ~0u;
    const bool on = valid && t < k && ((word >> (e & 31)) & 1);
    f_tok[q] = on ? __uint_as_float(area[0][t]) : 0.0f;
  }
}

// mid in memory, k <= 8 (NB = 1): mid_entry() in stream_common.hpp.
// k > 8 (NB = 2, 4): token-major, [chunk][slot][token][hi, lo][d_e] bf16, and only the rows of
// tokens whose mask bit for the slot's expert is set (and whose score is not zero) are written;
// tok_bits[chunk * E + slot] has bit t set for them.  At k = 32 about 60 % of the (token, slot)
// pairs of a union are such zeros, and what the stores of mid cost is their traffic to HBM (3 % of
// the up kernel's bytes took 11 % of its time); the down kernel stages the other tokens from a
// 16-byte block of zeros.

// Epilogue of one (chunk, slot), entirely inside the wave: lane (n = lane % 16, g) holds rows
// 4g .. 4g + 3 of each tile.  Swish / gating, router score and mask bit; mid is written split into
// bf16 hi/lo in the layout described above.
template <int NB, int NM, int RT>
__device__ __forceinline__ void up_epilogue_f(const f32x4 (&acc)[RT][NM][acc_tiles(NB)],
                                              const float (&f_tok)[acc_tiles(NB)], const LayerView &L, int64_t c,
                                              int s, int lane, int wave, uint16_t *__restrict__ midB,
                                              uint32_t *__restrict__ tok_bits, bool one_token = false) {
  constexpr int NA = acc_tiles(NB);
  const int E = L.E, d_e = L.d_e;
  const int g = lane >> 4;
  const int n = lane & 15;
  uint32_t bits = 0;
#pragma unroll
  for (int q = 0; q < NA; ++q) {
    const float f = f_tok[q];
    const bool on = f != 0.0f;   // a masked term, and one with a zero score, is +0 in mid
    if (NB > 1) bits |= ((uint32_t)__ballot(on) & 0xffffu) << (16 * q);   // lanes 0-15: g = 0, token 16 q + n
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
      if (NB == 1 && one_token) {
        // k = 1 (mid_one_token): columns 0 and 8 only, as rows [hi | lo][d_e] of the slot
        if ((n & 7) == 0)
          store_stream(reinterpret_cast<uint2 *>(midB + (((size_t)c * E + s) * 2 + (n >> 3)) * d_e +
                                                 (rr * 4 + wave) * 16 + 4 * g),
                       n < 8 ? vhi : vlo);
      } else if (NB == 1) {
        // fragment column n: hi for n < 8, lo of token n - 8 for n >= 8
        store_stream(mid_entry(midB, ((size_t)c * E + s) * (d_e / 32), rr * 4 + wave, g, n), n < 8 ? vhi : vlo);
      } else if (on) {
        uint16_t *row = midB + (((size_t)c * E + s) * (NB * 8) + q * 16 + n) * 2 * d_e + (rr * 4 + wave) * 16 + 4 * g;
        // plain stores here: a wave's 8-byte pieces land in 16 different token rows, and partial
        // lines written around the caches cost more than they save (tree_k32: up kernel + 5.6 %)
        *reinterpret_cast<uint2 *>(row) = vhi;
        *reinterpret_cast<uint2 *>(row + d_e) = vlo;
      }
    }
  }
  if (NB > 1 && wave == 0 && lane == 0) tok_bits[(size_t)c * E + s] = bits;
}

// NB: B fragments per K-step (see the top of the file); NM: 1 (Eq. 2) or 2 (gated); RT: 64-row
// groups of the expert (d_e = 64 * RT).  Wave w owns row tiles rr*4 + w.
template <int NB, int NM, int RT, bool ONE>
__global__ __launch_bounds__(kThreads, 2) void up_stream_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const uint4 *__restrict__ xS,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, const int32_t *__restrict__ items, const int32_t *__restrict__ total_ptr,
    int group, int k, uint16_t *__restrict__ midB, uint32_t *__restrict__ tok_bits) {
  static_assert(!ONE || NB == 1, "one-token chunks are k = 1");
  extern __shared__ uint4 xB[];   // [K-step][NB][64 lanes] of 8 bf16
  __shared__ uint32_t scoreS[2][4][3][64];   // [slot parity][wave]: see request_scores
  int spar = 0;
  constexpr int KC = 2048 / NB;   // contraction elements per LDS fill
  constexpr int NA = acc_tiles(NB);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lsrc = line_src(lane);
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int total = *total_ptr;
  const size_t row_bytes = (size_t)d * 2;
  const size_t rows8 = 8 * row_bytes;   // from the line of rows 0-7 to the line of rows 8-15

  // A list entry outside [0, E) (an invalid input) is an empty slot: the kernel streams a valid
  // expert in its place (the index is clamped) and writes zeros to mid, as if no token had it.
  // Returned: the clamped index, with bit 30 set when the entry was out of range.
  constexpr int kBad = 1 << 30;
  auto slot_expert = [&](int64_t c, int s) {
    const int e = active_idx ? active_idx[c * E + s] : s;
    return min(max(e, 0), E - 1) | ((unsigned)e >= (unsigned)E ? kBad : 0);
  };
  // an item is up to `group` consecutive slots of one chunk: the chunk's split x is written to
  // LDS once per item and serves all of them
  auto item_decode = [&](int item, int64_t &c, int &s, int &ns) {
    const int code = items[item];   // chunk * E + first slot
    c = code / E;
    s = code - (int)c * E;
    const int n_act = active_idx ? min(max(n_active[c], 0), E) : E;
    ns = max(1, min(group, n_act - s));
  };
  // per-lane byte pointer to the first fragment of (layer, expert, tile rr, matrix m)
  auto tile_ptr = [&](int layer, int e, int rr, int m) -> const char * {
    const char *w = static_cast<const char *>(m == 0 ? L.w_up : L.w_gate);
    const size_t row = ((size_t)layer * E + e) * d_e + (rr * 4 + wave) * 16 + line_row(lane);
    return w + row * row_bytes + line_byte(lane);
  };

  // One-token chunks (see split_x1_kernel): xS holds 8 entries per K-step, entry i of which belongs
  // at column 0 or 8 of its gg; the other columns of the LDS copy are zeroed here, once.
  constexpr bool one = ONE;   // mid_one_token
  auto x_entries = [&](int kc_len) { return one ? (kc_len / 32) * 8 : (kc_len / 32) * NB * 64; };
  auto x_src = [&](int64_t c, int kc0) { return xS + ((size_t)c * (d / 32) + kc0 / 32) * (one ? 8 : NB * 64); };
  auto x_dst = [&](int idx) { return one ? (idx >> 3) * 64 + ((idx >> 1) & 3) * 16 + (idx & 1) * 8 : idx; };
  if (one)
    for (int i = tid; i < kXBytes / 16; i += kThreads) xB[i] = make_uint4(0, 0, 0, 0);

  uint4 ring[kRing];
  // workgroup b runs on XCD b mod 8: consecutive items (slots of one chunk, same split x) go to
  // the workgroups of one XCD, which share an L2 (the launcher makes the grid a multiple of 8)
  int item = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (item >= total) return;
  int64_t c;
  int s, ns;        // current slot and slots left in the item (this one included)
  item_decode(item, c, s, ns);
  int e = slot_expert(c, s);
  bool e_ok = !(e & kBad);
  e &= ~kBad;
  int layer = clamp_layer(chunk_layer, c, L.n_layers);
  int64_t c_loaded = -1;   // chunk and K-chunk whose split x is in LDS
  int kc_loaded = -1;
  // The first PF entries per lane of the NEXT LDS fill are loaded during the last block of the
  // current K-chunk, ahead of that block's weight prefetches: loads return in issue order, so a
  // fill issued after them would wait for a full HBM round trip with the matrix cores idle.
  constexpr int PF = RT * NM * NA >= 16 ? 4 : (RT * NM * NA >= 8 ? 8 : 16);
  uint4 pf[PF];
  bool pf_valid = false;
  {
    const char *p = tile_ptr(layer, e, 0, 0);
#pragma unroll
    for (int i = 0; i < kRing; ++i) ring[i] = load_stream(p + (i & 1) * rows8 + (i >> 1) * 128);
  }

  while (true) {
    // what comes after this slot: the item's next slot, or the first slot of the next item
    bool has_next = true;
    int next_item = item;
    int64_t c_n = c;
    int s_n = s + 1, ns_n = ns - 1, e_n = 0, layer_n = layer;
    if (ns_n == 0) {
      next_item = item + gridDim.x;
      has_next = next_item < total;
      if (has_next) {
        item_decode(next_item, c_n, s_n, ns_n);
        layer_n = clamp_layer(chunk_layer, c_n, L.n_layers);
      }
    }
    if (has_next) e_n = slot_expert(c_n, s_n);
    const bool e_ok_n = !(e_n & kBad);
    e_n &= ~kBad;

    f32x4 acc[RT][NM][NA];
#pragma unroll
    for (int a = 0; a < RT; ++a)
#pragma unroll
      for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int q = 0; q < NA; ++q) acc[a][m][q] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the epilogue's scores are requested now: a load issued there would return behind the
    // ring's and stop the stream for a memory round trip
    request_scores(scoreS[spar][wave], L, scores, token_mask, c, e, k, lane);

    for (int kc0 = 0; kc0 < d; kc0 += KC) {
      const int kc_len = min(KC, d - kc0);
      const int nkb = kc_len / 512;
      const bool refill = c != c_loaded || kc0 != kc_loaded;   // uniform over the workgroup
      if (refill) __syncthreads();   // every wave is done with the previous contents of xB
      // copy the K-chunk's slice of the chunk's split x into LDS, 8 loads in flight per lane
      if (refill) {
        const int n16 = x_entries(kc_len);
        const uint4 *src = x_src(c, kc0);
        for (int base = 0; base < n16; base += PF * kThreads) {
          if (base > 0 || !pf_valid) {   // the first batch may have been loaded ahead
#pragma unroll
            for (int j = 0; j < PF; ++j) {
              const int idx = base + j * kThreads + tid;
              pf[j] = idx < n16 ? src[idx] : make_uint4(0, 0, 0, 0);
            }
          }
#pragma unroll
          for (int j = 0; j < PF; ++j) {
            const int idx = base + j * kThreads + tid;
            if (idx < n16) xB[x_dst(idx)] = pf[j];
          }
        }
      }
      if (refill) __syncthreads();
      c_loaded = c;
      kc_loaded = kc0;
      pf_valid = false;
      const bool last_kc = kc0 + KC >= d;
      // the LDS fill that follows this K-chunk: the slot's next K-chunk, else the next slot's first
      const int64_t c_f = last_kc ? c_n : c;
      const int k_f = last_kc ? 0 : kc0 + KC;
      const bool need_f = last_kc ? (has_next && (c_n != c || kc0 != 0)) : true;
      const int n16_f = x_entries(min(KC, d - k_f));
      const uint4 *src_f = x_src(c_f, k_f);
#pragma unroll
      for (int rr = 0; rr < RT; ++rr) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const char *cur = tile_ptr(layer, e, rr, m) + (size_t)kc0 * 2;
          // first block of the tile that follows this one in (K-chunk, rr, m) order
          const char *nxt_tile;
          if (m + 1 < NM) nxt_tile = tile_ptr(layer, e, rr, m + 1) + (size_t)kc0 * 2;
          else if (rr + 1 < RT) nxt_tile = tile_ptr(layer, e, rr + 1, 0) + (size_t)kc0 * 2;
          else if (!last_kc) nxt_tile = tile_ptr(layer, e, 0, 0) + (size_t)(kc0 + KC) * 2;
          else nxt_tile = tile_ptr(layer_n, e_n, 0, 0);   // nothing follows: expert 0's first tile, never used
          for (int kb = 0; kb < nkb; ++kb) {
            const bool tail = kb + 1 == nkb;
            const char *nxt = tail ? nxt_tile : cur + (size_t)(kb + 1) * 1024;
            if (rr == RT - 1 && m == NM - 1 && tail && need_f) {
#pragma unroll
              for (int j = 0; j < PF; ++j) {
                const int idx = j * kThreads + tid;
                pf[j] = idx < n16_f ? src_f[idx] : make_uint4(0, 0, 0, 0);
              }
              pf_valid = true;
            }
#pragma unroll
            for (int i = 0; i < kRing; i += 2) {   // a line: two K-steps
              uint4 f[2];
              line_operands(ring[i], ring[i + 1], lsrc, f[0], f[1]);
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int bf = 0; bf < NB; ++bf) {
                  const uint4 b = xB[(size_t)((kb * kRing + i + h) * NB + bf) * 64 + lane];
                  acc[rr][m][acc_of(NB, bf)] = mfma16(f[h], b, acc[rr][m][acc_of(NB, bf)]);
                }
              ring[i] = load_stream(nxt + (i >> 1) * 128);   // nxt is always a valid tile
              ring[i + 1] = load_stream(nxt + rows8 + (i >> 1) * 128);
            }
          }
        }
      }
    }

    float f_tok[NA];
    // everything older than the ring's 16 loads has arrived, the scores among it
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kRing) : "memory");
    read_scores<NB>(f_tok, scoreS[spar][wave], token_mask != nullptr, e, e_ok, k, lane);
    spar ^= 1;
    up_epilogue_f<NB, NM, RT>(acc, f_tok, L, c, s, lane, wave, midB, tok_bits, ONE);

    if (!has_next) break;
    item = next_item;
    c = c_n; s = s_n; ns = ns_n; e = e_n; e_ok = e_ok_n; layer = layer_n;
  }
}

// Up projection for k > 8 with the chunk's split x double buffered in LDS.  A refill of the
// single-buffer kernels costs two barriers at which the waves wait on memory while their weight
// rings drain (about 5 us per refill, four refills per slot at d = 2048, k = 32).  Here LDS
// holds two 32 KiB buffers of 1024 / NB contraction elements (FPT = 32 / NB K-steps); the buffer
// of the next K-chunk is filled by LDS-direct loads issued when the current K-chunk starts, so
// that at the K-chunk's end `s_waitcnt vmcnt(16)` (loads return in issue order, the 16 youngest
// are the ring's) finds it landed, one barrier publishes it, and the ring never stops.
// The weight stream's order is (item, K-chunk, slot, row tile, matrix, K-step); a cursor that
// runs exactly 16 fragments (the ring) ahead of the consumer produces the prefetch addresses, so
// it crosses tile, slot, K-chunk and item boundaries without special cases.  FPT is 8 or 16:
// the cursor then changes tile exactly when the consumer does.  An item is up to G * HW slots of
// one chunk: the workgroup is HW groups of four waves, group h takes slots h, h + HW, ... of the
// item (up to G, whose accumulators stay in registers across the K-chunks) and all of them share
// the buffers of x, the barriers and nothing else.
template <int NB, int NM, int RT, int G, int HW>
__global__ __launch_bounds__(kThreads * HW, 2 / HW) void up_stream_db_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const uint4 *__restrict__ xS,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, const int32_t *__restrict__ items, const int32_t *__restrict__ total_ptr,
    int k, uint16_t *__restrict__ midB, uint32_t *__restrict__ tok_bits) {
  static_assert(NB == 2 || NB == 4, "8 or 16 K-steps per buffer");
  static_assert(HW == 1 || HW == 2, "one or two groups of four waves");
  constexpr int FPT = 32 / NB;            // K-steps (fragments of one tile) per K-chunk
  constexpr int KB = 32 * FPT;            // contraction elements per buffer
  constexpr int kBuf = FPT * NB * 64;     // uint4 per buffer (2048 = 32 KiB)
  constexpr int TPS = RT * NM;            // tiles per slot and K-chunk
  static_assert(FPT == 16 || TPS % 2 == 0, "with 8 fragments per tile the ring half must follow from (rr, m)");
  constexpr int NA = acc_tiles(NB);
  extern __shared__ uint4 xB[];           // [2][K-step][NB][64 lanes]
  // wave = w4 of half `half`: the halves of a workgroup take every HW-th slot of the item each and
  // share the buffers of x
  const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, half = tid >> 8;
  const int lsrc = line_src(lane);
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int total = *total_ptr;
  const size_t row_bytes = (size_t)d * 2;
  const size_t rows8 = 8 * row_bytes;   // from the line of rows 0-7 to the line of rows 8-15
  const int nkc = d / KB;

  auto slot_expert = [&](int64_t c, int s) {
    const int e = active_idx ? active_idx[c * E + s] : s;
    return min(max(e, 0), E - 1);
  };
  auto item_decode = [&](int item, int64_t &c, int &s, int &ns) {
    const int code = items[item];   // chunk * E + first slot
    c = code / E;
    s = code - (int)c * E;
    const int n_act = active_idx ? min(max(n_active[c], 0), E) : E;
    ns = max(1, min(G * HW, n_act - s));   // slots of the item, this half's among them: s + half, s + half + HW, ...
  };
  // Slot sl of this half is slot s0 + sl * HW + half of the chunk; the half has (ns - half + HW - 1) / HW
  // of them.  A half without any (the chunk's last item, one slot left) streams the item's first
  // slot once more and writes nothing: the walk over the weights has no empty item.
  auto half_slots = [&](int ns) { return max(1, (ns - half + HW - 1) / HW); };
  auto half_slot = [&](int s0, int sl, int ns) { return half < ns ? s0 + sl * HW + half : s0; };
  // per-lane byte pointer to fragment 0 of tile t = rr * NM + m of (layer, expert)
  auto tile_ptr = [&](int layer, int e, int t) -> const char * {
    const int rr = t / NM, m = t % NM;
    const char *w = static_cast<const char *>(m == 0 ? L.w_up : L.w_gate);
    const size_t row = ((size_t)layer * E + e) * d_e + (rr * 4 + wave) * 16 + line_row(lane);
    return w + row * row_bytes + line_byte(lane);
  };
  // The experts of an item's slots are kept as bytes of one word (E <= 256): indexed by a run-time
  // slot, an array of them is moved to scratch memory by the compiler, and the load from there
  // waits for every outstanding weight load.
  static_assert(G <= 4 && kMaxExperts <= 256, "four expert ids in 32 bits");
  auto pick = [&](uint32_t v, int sl) { return (int)((v >> (8 * sl)) & 0xffu); };
  auto slots_experts = [&](int64_t c, int s0, int ns) {
    uint32_t v = 0;
#pragma unroll
    for (int sl = 0; sl < G; ++sl) v |= (uint32_t)slot_expert(c, half_slot(s0, min(sl, half_slots(ns) - 1), ns)) << (8 * sl);
    return v;   // slots past the half's last repeat it and are never used
  };
  // bit sl set: the list entry of slot sl is outside [0, E) (an invalid input): an empty slot, for
  // which a valid expert is streamed (the clamped index) and no row of mid is written
  auto slots_bad = [&](int64_t c, int s0, int ns) {
    uint32_t v = 0;
    if (active_idx) {
#pragma unroll
      for (int sl = 0; sl < G; ++sl)
        v |= ((unsigned)active_idx[c * E + half_slot(s0, min(sl, half_slots(ns) - 1), ns)] >= (unsigned)E ? 1u : 0u) << sl;
    }
    return half < ns ? v : ~0u;   // a half without a slot of its own writes nothing
  };
  // LDS-direct fill of one buffer: 32 KiB, 8 / HW loads per wave
  auto fill = [&](int64_t c, int kc, int buf) {
    constexpr int per_wave = kBuf / (4 * HW);
    const int fw = half * 4 + wave;
    const uint4 *src = xS + ((size_t)c * (d / 32) + (size_t)kc * FPT) * NB * 64 + fw * per_wave + lane;
    uint4 *dst = xB + buf * kBuf + fw * per_wave;
#pragma unroll
    for (int j = 0; j < per_wave / 64; ++j) load_to_lds16(src + j * 64, dst + j * 64);
  };

  // Router scores and mask words of the item's tokens, [item parity][slot][score, mask lo, mask
  // hi][token], also by LDS-direct loads: wave sl requests slot sl's when the item starts, the
  // K-chunks' barriers publish them, the epilogue reads them from LDS.  Loaded into registers they
  // made the epilogue start with a wait for "every load so far" (the compiler cannot count across
  // the K-chunk loop), i.e. for the ring's 16 loads of the next item; this way the kernel has no
  // such wait at all.
  __shared__ uint32_t scoreS[2][HW][G][3][64];
  auto request_scores = [&](int ipar, int64_t c, uint32_t es, int k) {
    if (wave < G) {   // uniform over the wave; a slot past ns repeats the last one
      const int e = pick(es, wave);
      const int64_t tok = c * k + min(lane & 31, k - 1);
      load_to_lds4(scores + tok * E + e, &scoreS[ipar][half][wave][0][0]);
      if (token_mask) {
        const uint32_t *m = reinterpret_cast<const uint32_t *>(token_mask + tok * L.W + (e >> 6));
        load_to_lds4(m, &scoreS[ipar][half][wave][1][0]);
        load_to_lds4(m + 1, &scoreS[ipar][half][wave][2][0]);
      }
    }
  };
  auto read_scores = [&](float (&f_tok)[NA], int ipar, int sl, int e, bool valid) {
    const int n = lane & 15;
#pragma unroll
    for (int q = 0; q < NA; ++q) {
      const int t = q * 16 + n;   // NB = 2: one accumulator tile, tokens 0-15
      const uint32_t word = token_mask ? scoreS[ipar][half][sl][1 + ((e >> 5) & 1)][t] : ~0u;
      const bool on = valid && t < k && ((word >> (e & 31)) & 1);
      f_tok[q] = on ? __uint_as_float(scoreS[ipar][half][sl][0][t]) : 0.0f;
    }
  };

  // Workgroup b runs on XCD b mod 8 and each XCD has its own L2.  The items of a chunk all read
  // the chunk's split x (256 KiB at k = 32), so consecutive items go to the workgroups of ONE XCD:
  // step j of workgroup (xcd, w) takes item ((j * 8 + xcd) * per_xcd + w), and x is served by that
  // L2 instead of crossing the fabric once per item.
  const int per_xcd = gridDim.x / 8;   // the launcher makes the grid a multiple of 8
  const int item_step = 8 * per_xcd;
  int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (item >= total) return;
  int64_t c;
  int s0, ns;
  item_decode(item, c, s0, ns);
  int layer = clamp_layer(chunk_layer, c, L.n_layers);
  uint32_t es = slots_experts(c, s0, ns), bad = slots_bad(c, s0, ns);

  // next item (valid while has_next) and the prefetch cursor
  bool has_next = false;
  int64_t c_n = c;
  int s0_n = 0, ns_n = 1, layer_n = layer;
  uint32_t esn = es, bad_n = bad;
  auto decode_next = [&](int next_item) {
    has_next = next_item < total;
    if (has_next) {
      item_decode(next_item, c_n, s0_n, ns_n);
      layer_n = clamp_layer(chunk_layer, c_n, L.n_layers);
      esn = slots_experts(c_n, s0_n, ns_n);
      bad_n = slots_bad(c_n, s0_n, ns_n);
    }
  };
  decode_next(item + item_step);

  bool cu_next = false;          // the cursor is in the next item
  int cu_kc = 0, cu_sl = 0, cu_t = 0;
  const char *cu_ptr = tile_ptr(layer, pick(es, 0), 0);
  // To the next tile of the stream.  All of this is uniform over the wave and written without
  // branches: control flow between two tiles makes the compiler's counted waits for the ring's
  // loads collapse to "wait for everything" at the join.
  auto cu_advance = [&]() {
    const int nsl = half_slots(cu_next ? ns_n : ns);
    const bool wrap_t = cu_t + 1 == TPS;
    const int t = wrap_t ? 0 : cu_t + 1;
    const bool wrap_s = wrap_t && cu_sl + 1 == nsl;
    const int sl = wrap_s ? 0 : cu_sl + (wrap_t ? 1 : 0);
    const bool wrap_k = wrap_s && cu_kc + 1 == nkc;
    const int kc = wrap_k ? 0 : cu_kc + (wrap_s ? 1 : 0);
    const bool to_next = wrap_k && !cu_next && has_next;
    const bool stay = wrap_k && !to_next;   // nothing follows: stay on the last tile (its loads are never used)
    cu_kc = stay ? nkc - 1 : kc;
    cu_sl = stay ? nsl - 1 : sl;
    cu_t = stay ? TPS - 1 : t;
    cu_next = cu_next || to_next;
    cu_ptr = tile_ptr(cu_next ? layer_n : layer, cu_next ? pick(esn, cu_sl) : pick(es, cu_sl), cu_t) +
             (size_t)cu_kc * (KB * 2);
  };

  // prologue: x of the first K-chunk, then the ring's first 16 fragments
  fill(c, 0, 0);
  uint4 ring[kRing];
#pragma unroll
  for (int h = 0; h < kRing / FPT; ++h) {
#pragma unroll
    for (int i = 0; i < FPT; ++i) ring[h * FPT + i] = load_stream(cu_ptr + (i & 1) * rows8 + (i >> 1) * 128);
    cu_advance();
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kRing) : "memory");   // the fill is older than the ring's loads
  __syncthreads();
  int par = 0;   // buffer of the current K-chunk
  int ipar = 0;  // half of scoreS of the current item

  while (true) {
    f32x4 acc[G][RT][NM][NA];
#pragma unroll
    for (int sl = 0; sl < G; ++sl)
#pragma unroll
      for (int a = 0; a < RT; ++a)
#pragma unroll
        for (int m = 0; m < NM; ++m)
#pragma unroll
          for (int q = 0; q < NA; ++q) acc[sl][a][m][q] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the epilogue's scores are requested now: a load issued there would return behind the
    // ring's and stop the stream for a memory round trip
    request_scores(ipar, c, es, k);

    for (int kc = 0; kc < nkc; ++kc) {
      // x of the K-chunk that follows goes into the other buffer (every wave left it at the last barrier)
      const bool last_kc = kc + 1 == nkc;
      if (!last_kc) fill(c, kc + 1, par ^ 1);
      else if (has_next) fill(c_n, 0, par ^ 1);
      const uint4 *xb = xB + par * kBuf;
#pragma unroll
      for (int sl = 0; sl < G; ++sl) {
        if (sl >= half_slots(ns)) break;   // uniform over the half
#pragma unroll
        for (int rr = 0; rr < RT; ++rr) {
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            constexpr int kHalves = kRing / FPT;   // tiles the ring holds
            const int r0 = kHalves == 1 ? 0 : ((rr * NM + m) % kHalves) * FPT;
#pragma unroll
            for (int i = 0; i < FPT; i += 2) {   // a line: two K-steps
              uint4 f[2];
              line_operands(ring[r0 + i], ring[r0 + i + 1], lsrc, f[0], f[1]);
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int bf = 0; bf < NB; ++bf) {
                  const uint4 b = xb[((i + h) * NB + bf) * 64 + lane];
                  acc[sl][rr][m][acc_of(NB, bf)] = mfma16(f[h], b, acc[sl][rr][m][acc_of(NB, bf)]);
                }
              ring[r0 + i] = load_stream(cu_ptr + (i >> 1) * 128);
              ring[r0 + i + 1] = load_stream(cu_ptr + rows8 + (i >> 1) * 128);
              // keep the refill here: left alone, the scheduler moves the loads of a tile together and
              // this kernel loses 10 % (the single-buffer kernel, oddly, is 1-5 % better left alone)
              __builtin_amdgcn_sched_barrier(0);
            }
            cu_advance();
          }
        }
      }
      // the next buffer has landed (it is older than the ring's 16 outstanding loads); publish it
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kRing) : "memory");
      __syncthreads();
      par ^= 1;
    }

    float f_tok[G][NA];
#pragma unroll
    for (int sl = 0; sl < G; ++sl) read_scores(f_tok[sl], ipar, sl, pick(es, sl), !((bad >> sl) & 1));
#pragma unroll
    for (int sl = 0; sl < G; ++sl)
      if (sl < half_slots(ns) && half < ns)   // a half without a slot of its own has nothing to write
        up_epilogue_f<NB, NM, RT>(acc[sl], f_tok[sl], L, c, half_slot(s0, sl, ns), lane, wave, midB, tok_bits);
    ipar ^= 1;   // the next item's scores go to the other half: a slower wave may still be reading this one

    if (!has_next) break;
    item += item_step;
    c = c_n; s0 = s0_n; ns = ns_n; layer = layer_n;
    es = esn;
    bad = bad_n;
    cu_next = false;   // the cursor was in this item already (an item is longer than the ring)
    decode_next(item + item_step);
  }
}

// ------------------------------------------------------------------------------------------------ up, few chunks

// The value lane (src_bytes / 4) holds (ds_bpermute; every lane names its source).
__device__ __forceinline__ uint4 lanes_from(uint4 v, int src_bytes) {
  return make_uint4((uint32_t)__builtin_amdgcn_ds_bpermute(src_bytes, (int)v.x),
                    (uint32_t)__builtin_amdgcn_ds_bpermute(src_bytes, (int)v.y),
                    (uint32_t)__builtin_amdgcn_ds_bpermute(src_bytes, (int)v.z),
                    (uint32_t)__builtin_amdgcn_ds_bpermute(src_bytes, (int)v.w));
}

struct RouteOut {
  const float *preact;            // A^0 [token][N_e]
  float *scores;                  // what blockffn_router and blockffn_chunk_union write
  uint64_t *token_mask, *union_mask;
  int32_t *active_idx, *n_active;
  unsigned long long *stats;      // or nullptr
};

// Small launches (e.g. a single chunk walking through a layer stack) do not have enough (chunk,
// slot) items to occupy the chip with one workgroup per item.  Here one workgroup takes one
// 16-row tile of one item; its four waves split the contraction, each keeps its quarter of the
// chunk's split x in registers (no LDS fill, no barrier before the stream starts) and the four
// partial tiles meet in LDS once at the end.  k <= 8 only; FW = d / 128 fragments per wave.
// ROUTE: the launch also stands in for the router's normalising pass and for the chunk union.  It
// is given the pre-activations A^0 (+ bias) of the chunk's tokens instead of scores, masks and
// lists; every workgroup redoes the chunk's routing from them (8 tokens x N_e values: masks,
// RMSNorm, union, the expert of its slot - the arithmetic of router_finish_kernel and
// chunk_union_kernel, so the same bits) and the workgroup of slot 0, tile 0 writes the outputs the
// two kernels would have written.  One round trip to memory for 2 KiB in place of the two loads
// of the list entry, and two launches fewer per layer.
// Items are (chunk, slot, tile) in that order and workgroup b takes items b, b + gridDim.x, ...: the
// grid covers every item, except for a single chunk, where it stops at the two workgroups per CU
// that can be resident (the hardware would run the rest after them anyway); the items of a
// workgroup then share the chunk, and with it the routing and the x registers.  Order of the
// requests: A^0 (or the list entry) first, then x, which depends on nothing and arrives while the
// routing is worked out, then the weights (loads return in the order they were issued, so
// nothing that is waited for early may stand behind a long burst).
template <int NM, int FW, bool ROUTE>
__global__ __launch_bounds__(kThreads) void up_split_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const float *__restrict__ x,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int k, uint16_t *__restrict__ midB, RouteOut ro, int total) {
  __shared__ float red[4][NM][4][64];
  __shared__ uint64_t tmask_s[8][kMaxMaskWords];   // ROUTE: the tokens' masks and RMS
  __shared__ float rms_s[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, n = lane & 15;
  const int E = L.E, d = L.d, d_e = L.d_e;
  const int tiles = d_e / 16;
  const int tok = n & 7, half = n >> 3;
  int item = blockIdx.x;   // below `total`: the grid is never larger
  const int64_t c = item / (E * tiles);
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int kq0 = wave * (d / 4);

  // ---- what the first item's expert depends on is requested first
  int n_act = E;
  int e_first = item / tiles - (int)c * E;
  [[maybe_unused]] float a0v[2][kMaxMaskWords];   // ROUTE: A^0 of tokens wave and wave + 4
  if constexpr (ROUTE) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int t = wave + 4 * it;
#pragma unroll
      for (int wd = 0; wd < kMaxMaskWords; ++wd) {
        const int i = wd * 64 + lane;
        a0v[it][wd] = (t < k && wd < L.W && i < E) ? ro.preact[(c * k + t) * E + i] : 0.0f;
      }
    }
  } else if (active_idx) {
    n_act = n_active[c];
    e_first = active_idx[c * E + e_first];
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- x of this wave's quarter of the contraction.  Fragment column n carries token n & 7, its
  // hi part for n < 8 and its lo part for n >= 8: lane (g, half, token) needs floats 8 g + 4 half
  // .. + 3 of the token's 32 per K-step, splits them, and lanes n and n + 8 exchange what the other
  // needs.  What bounds this launch is how fast a CU's memory pipeline takes requests in, and that
  // goes by groups of four consecutive lanes: four lanes reading 64 contiguous bytes are one
  // request where four lanes reading 16 bytes of four rows (the matrix core's operand order) are
  // four.  So every load is issued with the lanes in memory order (here lane = 8 token + piece, a
  // token's 128 bytes by eight neighbours) and the registers are put into operand order by a
  // cross-lane permutation once they are back (ds_bpermute).
  const float *xrow = x + (c * k + min(lane >> 3, k - 1)) * d + kq0 + (lane & 7) * 4;
  uint4 bfrag[FW];   // x as loaded, then (in place) the B operand of every K-step, kept for later items
#pragma unroll
  for (int i = 0; i < FW; ++i) bfrag[i] = *reinterpret_cast<const uint4 *>(xrow + i * 32);
  const int x_src = (8 * tok + 2 * g + half) * 4;   // byte address of the source lane
  __builtin_amdgcn_sched_barrier(0);

  [[maybe_unused]] uint64_t U[kMaxMaskWords];
  if constexpr (ROUTE) {
    const bool writer = blockIdx.x % (E * tiles) == 0;   // the workgroup of the chunk's slot 0, tile 0
    const int W = L.W;
#pragma unroll
    for (int it = 0; it < 2; ++it) {   // k <= 8: lanes run over the experts of one mask word at a time
      const int t = wave + 4 * it;
      if (t < k) {                     // uniform over the wave
        const int64_t tk = c * k + t;
        float a1[kMaxMaskWords];
        float sumsq = 0.0f;
#pragma unroll
        for (int wd = 0; wd < kMaxMaskWords; ++wd) {
          a1[wd] = 0.0f;
          if (wd < W) {
            const int i = wd * 64 + lane;
            const float a0 = a0v[it][wd];
            const bool active = (i < E) && (a0 > 0.0f);
            const uint64_t word = __ballot(active);
            if (lane == 0) {
              tmask_s[t][wd] = word;
              if (writer) ro.token_mask[tk * W + wd] = word;
            }
            a1[wd] = active ? a0 : 0.0f;
            sumsq = fmaf(a1[wd], a1[wd], sumsq);
          }
        }
        const float ms = wave_sum(sumsq) / (float)E;
        const float rms = sqrtf(ms + L.eps);
        if (lane == 0) rms_s[t] = rms;
        if (writer) {
#pragma unroll
          for (int wd = 0; wd < kMaxMaskWords; ++wd) {
            const int i = wd * 64 + lane;
            if (wd < W && i < E) {
              const float gn = L.g_rms ? L.g_rms[(size_t)layer * E + i] : 1.0f;
              ro.scores[tk * E + i] = a1[wd] > 0.0f ? gn * a1[wd] / rms : 0.0f;
            }
          }
        }
      }
    }
    __syncthreads();
    n_act = 0;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      U[wd] = 0;
      if (wd < W) {
        for (int t = 0; t < k; ++t) U[wd] |= tmask_s[t][wd];
        n_act += __popcll(U[wd]);
      }
    }
    if (writer && wave == 0) {   // Union(x), its ascending list, the counts (chunk_union_kernel's outputs)
      int base = 0;
#pragma unroll
      for (int wd = 0; wd < kMaxMaskWords; ++wd) {
        if (wd < W) {
          const uint64_t u = U[wd];
          if (lane == 0) ro.union_mask[c * W + wd] = u;
          const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(u >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)u, 0));
          if ((u >> lane) & 1) ro.active_idx[c * E + base + below] = wd * 64 + lane;
          base += __popcll(u);
        }
      }
      for (int sl = base + lane; sl < E; sl += kWave) ro.active_idx[c * E + sl] = -1;
      if (lane == 0) {
        ro.n_active[c] = base;
        if (ro.stats) {
          long long tok_active = 0;
          for (int t = 0; t < k; ++t)
            for (int wd = 0; wd < W; ++wd) tok_active += __popcll(tmask_s[t][wd]);
          atomicAdd(&ro.stats[0], (unsigned long long)((long long)k * E - tok_active));
          atomicAdd(&ro.stats[1], (unsigned long long)(E - base));
        }
      }
    }
  }   // tmask_s and rms_s are only read from here on

  const int lsrc = line_src(lane);
  for (bool first = true; item < total; item += gridDim.x, first = false) {
    const int code = item / tiles, rt = item - code * tiles;
    const int s = code - (int)c * E;   // a workgroup with several items has them all in chunk c
    if (s >= n_act) break;             // uniform over the workgroup; later items have later slots
    // score and mask word of this lane's token, for the epilogue (wave 0)
    float f = 0.0f;
    uint64_t mword = ~0ull;
    int e = s;
    if constexpr (ROUTE) {
      // the expert of slot s: the s-th set bit of the union
      int left = s;
#pragma unroll
      for (int wd = 0; wd < kMaxMaskWords; ++wd) {
        if (wd < L.W && left >= 0) {
          const int pc = __popcll(U[wd]);
          if (left < pc) {   // lane l asks whether bit l is the one with `left` set bits below it
            const uint64_t u = U[wd];
            const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(u >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)u, 0));
            e = wd * 64 + __builtin_ctzll(__ballot(((u >> lane) & 1) && below == left));
            left = -1;
          } else {
            left -= pc;
          }
        }
      }
      if (wave == 0 && tok < k) {
        const int64_t tk = c * k + tok;
        mword = tmask_s[tok][e >> 6];
        const float a0 = ro.preact[tk * E + e];
        const float a1v = a0 > 0.0f ? a0 : 0.0f;
        const float gn = L.g_rms ? L.g_rms[(size_t)layer * E + e] : 1.0f;
        f = a1v > 0.0f ? gn * a1v / rms_s[tok] : 0.0f;
      }
    } else if (active_idx) {
      e = first ? e_first : active_idx[c * E + s];
    }
    // a list entry outside [0, E) is an empty slot: zeros in mid (a valid expert is streamed in its place)
    const bool e_ok = (unsigned)e < (unsigned)E;
    e = min(max(e, 0), E - 1);
    // score and mask word for the epilogue: requested before the weights, so that they are back
    // before them instead of costing a round trip after them
    if (!ROUTE && wave == 0 && tok < k) {
      const int64_t t = c * k + tok;
      if (token_mask) mword = token_mask[t * L.W + (e >> 6)];
      f = scores[t * E + e];
    }

    // the weights: whole lines, non-temporal (load_stream): a[m][2 p] is line p of the tile's rows
    // 0-7, a[m][2 p + 1] of rows 8-15, lane = 8 row + piece
    uint4 a[NM][FW];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const char *w = static_cast<const char *>(m == 0 ? L.w_up : L.w_gate);
      const char *row = w + ((((size_t)layer * E + e) * d_e + rt * 16 + line_row(lane)) * d + kq0) * 2 + line_byte(lane);
#pragma unroll
      for (int i = 0; i < FW; ++i) a[m][i] = load_stream(row + (size_t)(i & 1) * 8 * d * 2 + (i >> 1) * 128);
    }
    // every load of this wave is in flight before anything waits
    __builtin_amdgcn_sched_barrier(0);
    if (first) {   // x came back long ago
#pragma unroll
      for (int i = 0; i < FW; ++i) {
        const uint4 xb = lanes_from(bfrag[i], x_src);
        const float v[4] = {__uint_as_float(xb.x), __uint_as_float(xb.y), __uint_as_float(xb.z), __uint_as_float(xb.w)};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          split_bf16(v[q], hi[q], lo[q]);
          if (tok >= k) hi[q] = lo[q] = 0u;
        }
        const uint32_t hw0 = hi[0] | hi[1] << 16, hw1 = hi[2] | hi[3] << 16;
        const uint32_t lw0 = lo[0] | lo[1] << 16, lw1 = lo[2] | lo[3] << 16;
        // lane n < 8 keeps its hi words and sends its lo words; lane n + 8 does the opposite
        const uint32_t r0 = __shfl_xor(half ? hw0 : lw0, 8, kWave);
        const uint32_t r1 = __shfl_xor(half ? hw1 : lw1, 8, kWave);
        bfrag[i] = half ? make_uint4(r0, r1, lw0, lw1) : make_uint4(hw0, hw1, r0, r1);
      }
    }
    f32x4 acc[NM];
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < FW; i += 2) {   // a line: two K-steps
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        uint4 f0, f1;
        line_operands(a[m][i], a[m][i + 1], lsrc, f0, f1);
        acc[m] = mfma16(f0, bfrag[i], acc[m]);
        acc[m] = mfma16(f1, bfrag[i + 1], acc[m]);
      }
    }
    if (!first) __syncthreads();   // wave 0 has read the previous item's partial tiles
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) red[wave][m][q][lane] = acc[m][q];
    __syncthreads();
    if (wave == 0) {
      const bool on = e_ok && tok < k && ((mword >> (e & 63)) & 1);
      uint32_t packed[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float u = (red[0][0][q][lane] + red[1][0][q][lane]) + (red[2][0][q][lane] + red[3][0][q][lane]);
        u += __shfl_xor(u, 8, kWave);
        float h;
        if (NM == 2) {
          float gt = (red[0][NM - 1][q][lane] + red[1][NM - 1][q][lane]) + (red[2][NM - 1][q][lane] + red[3][NM - 1][q][lane]);
          gt += __shfl_xor(gt, 8, kWave);
          h = swish(gt) * u;
        } else {
          h = swish(u);
        }
        uint32_t hi, lo;
        split_bf16(on ? f * h : 0.0f, hi, lo);
        packed[q] = n < 8 ? hi : lo;
      }
      store_stream(mid_entry(midB, ((size_t)c * E + s) * (d_e / 32), rt, g, n),
                   make_uint2(packed[0] | packed[1] << 16, packed[2] | packed[3] << 16));
    }
  }
}

// ------------------------------------------------------------------------------------------------ up, one chunk

// One chunk alone on the chip (a decode step walking through a layer stack).  What bounds its up
// projection is what the busiest CU has to take in: with one workgroup per (slot, 16-row tile)
// some CUs get two of them, each with its own copy of x.  Here one workgroup of eight waves per CU
// takes an equal share of the union's rows - `per` groups of four consecutive neurons, up to two
// 16-row tiles, wave = (tile, quarter of the contraction) - and reads x once: every wave loads
// half of its quarter and turns it into B operands in LDS, where all waves read them from.  The routing is
// redone by every workgroup as in up_split_kernel<.., ROUTE> (one token per wave), workgroup 0
// writes the router's and the union's outputs.  The partial sums of the four quarters are added in
// up_split_kernel's order: the same bits.
constexpr int kChipThreads = 512;
constexpr int kChipQuads = 8;   // groups of four rows per workgroup and round (two tiles)

template <int NM, int FW, bool ROUTE>
__global__ __launch_bounds__(kChipThreads) void up_chip_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const float *__restrict__ x,
    const float *__restrict__ scores, const uint64_t *__restrict__ token_mask, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int k, uint16_t *__restrict__ midB, RouteOut ro) {
  extern __shared__ uint4 xS[];   // [quarter][K-step][lane]: the B operands of the whole contraction
  __shared__ float red[8][NM][4][64];
  __shared__ float pre_s[8][kMaxExperts];            // A^0 of the chunk's tokens
  __shared__ uint64_t tmask_s[8][kMaxMaskWords];
  __shared__ float rms_s[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tile = wave >> 2, kq = wave & 3;
  const int g = lane >> 4, n = lane & 15;
  const int E = L.E, d = L.d, d_e = L.d_e, W = L.W;
  const int tok = n & 7, half = n >> 3;
  const int layer = clamp_layer(chunk_layer, 0, L.n_layers);
  const bool writer = blockIdx.x == 0;

  // ---- A^0 of token `wave`, then x: this wave's half of its quarter (both in memory order).
  // Up to the first matrix instruction no load stands under a branch (an index out of range is
  // clamped and the value dropped): where paths with different loads in flight join, the
  // compiler's counted waits turn into waits for nearly everything, x included, long before x is
  // needed.  What only workgroup 0 does for the chunk (the router's and the union's outputs)
  // comes at the very end for the same reason.
  // Without ROUTE the chunk's list takes the place of A^0: its count and its entries together
  // (lane l holds entries l, l + 64, ...); with no list (every expert, the dense pass) x stands in
  // as an address and the values are dropped.
  [[maybe_unused]] float a0v[kMaxMaskWords];   // values past the last expert are dropped where they are used
  [[maybe_unused]] int ent[kMaxMaskWords];
  [[maybe_unused]] int n_list = 0;
  if constexpr (ROUTE) {
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd)
      a0v[wd] = ro.preact[(size_t)min(wave, k - 1) * E + min(wd * 64 + lane, E - 1)];
  } else {
    const int32_t *lp = active_idx ? active_idx : reinterpret_cast<const int32_t *>(x);
    const int32_t *np = active_idx ? n_active : reinterpret_cast<const int32_t *>(x);
    const int span = active_idx ? E - 1 : 0;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) ent[wd] = lp[min(wd * 64 + lane, span)];
    n_list = np[0];
  }
  __builtin_amdgcn_sched_barrier(0);
  constexpr int FH = FW / 2;
  const float *xrow = x + (size_t)min(lane >> 3, k - 1) * d + kq * (d / 4) + (lane & 7) * 4;
  uint4 xraw[FH];
#pragma unroll
  for (int i = 0; i < FH; ++i) xraw[i] = *reinterpret_cast<const uint4 *>(xrow + (tile * FH + i) * 32);
  const int x_src = (8 * tok + 2 * g + half) * 4;
  __builtin_amdgcn_sched_barrier(0);

  // ---- routing of token `wave`
  if (ROUTE && wave < k) {   // uniform over the wave
    const int t = wave;
    float a1[kMaxMaskWords];
    float sumsq = 0.0f;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      a1[wd] = 0.0f;
      if (wd < W) {
        const int i = wd * 64 + lane;
        const float a0 = i < E ? a0v[wd] : 0.0f;
        const bool active = a0 > 0.0f;
        const uint64_t word = __ballot(active);
        if (i < E) pre_s[t][i] = a0;
        if (lane == 0) tmask_s[t][wd] = word;
        a1[wd] = active ? a0 : 0.0f;
        sumsq = fmaf(a1[wd], a1[wd], sumsq);
      }
    }
    const float ms = wave_sum(sumsq) / (float)E;
    const float rms = sqrtf(ms + L.eps);
    if (lane == 0) rms_s[t] = rms;
  }
  if constexpr (ROUTE) __syncthreads();   // the tokens' masks, RMS and A^0 are in LDS

  // ---- Union(x)
  [[maybe_unused]] uint64_t U[kMaxMaskWords];
  int n_act = 0;
  if constexpr (!ROUTE) {
    n_act = active_idx ? min(max(n_list, 0), E) : E;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd)
      if (!active_idx) ent[wd] = wd * 64 + lane;
  }
#pragma unroll
  for (int wd = 0; wd < kMaxMaskWords; ++wd) {
    U[wd] = 0;
    if (ROUTE && wd < W) {
#pragma unroll
      for (int t = 0; t < 8; ++t) U[wd] |= tmask_s[min(t, k - 1)][wd];   // eight reads in flight; a token past the end repeats the last
      n_act += __popcll(U[wd]);
    }
  }
  // the expert of slot sl: the sl-th set bit of the union (lane l asks whether bit l is that
  // one), or the list's entry as it stands (an entry outside [0, N_e) is an empty slot)
  auto slot_expert = [&](int sl) {
    int e = 0, left = sl;
    if constexpr (!ROUTE) {
#pragma unroll
      for (int wd = 0; wd < kMaxMaskWords; ++wd) {
        const int v = __builtin_amdgcn_readlane(ent[wd], sl & 63);
        e = (sl >> 6) == wd ? v : e;
      }
      return e;
    }
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      if (wd < W) {
        const uint64_t u = U[wd];
        const int pc = __popcll(u);
        const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(u >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)u, 0));
        const uint64_t hit = __ballot(((u >> lane) & 1) && below == left);
        if (left >= 0 && left < pc) e = wd * 64 + __builtin_ctzll(hit | (1ull << 63));
        left = left < pc ? -1 : left - pc;
      }
    }
    return e;
  };

  // Union(x), its ascending list and the counts (chunk_union_kernel's outputs), by one wave
  auto write_union = [&]() {
    int base = 0;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      if (wd < W) {
        const uint64_t u = U[wd];
        if (lane == 0) ro.union_mask[wd] = u;
        const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(u >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)u, 0));
        if ((u >> lane) & 1) ro.active_idx[base + below] = wd * 64 + lane;
        base += __popcll(u);
      }
    }
    for (int sl = base + lane; sl < E; sl += kWave) ro.active_idx[sl] = -1;
    if (lane == 0) {
      ro.n_active[0] = base;
      if (ro.stats) {
        long long tok_active = 0;
        for (int t = 0; t < k; ++t)
          for (int wd = 0; wd < W; ++wd) tok_active += __popcll(tmask_s[t][wd]);
        atomicAdd(&ro.stats[0], (unsigned long long)((long long)k * E - tok_active));
        atomicAdd(&ro.stats[1], (unsigned long long)(E - base));
      }
    }
  };

  // ---- this workgroup's share of the union's rows, in groups of four
  const int qshift = __builtin_ctz(d_e / 4);                 // groups per slot: 16, 32 or 64
  const int Q = n_act << qshift;
  // ceil(Q / workgroups) by a float division: exact for these sizes (Q <= 2^14, a quotient that
  // is not an integer is at least 1 / 1024 away from one) and a fifth of the integer sequence
  const int per = (int)ceilf((float)Q / (float)gridDim.x);
  const int q_lo = blockIdx.x * per, q_hi = min(Q, q_lo + per);
  const int lsrc = line_src(lane);
  // Rounds of up to kChipQuads groups (one round unless per > 8).  No branch stands around a load
  // or a matrix instruction (the compiler's counted waits would collapse at the join): a tile or a
  // group past the end asks for the last group's rows again and stores nothing.  In the first
  // round x is turned into B operands and exchanged while the weights are on their way, between
  // the two halves of the weight requests (all of them first would not leave the registers).
  for (int q0 = q_lo; q0 < q_hi; q0 += kChipQuads) {   // uniform over the workgroup
    const bool first = q0 == q_lo;
    // a round's groups lie in at most two slots
    const int sa = q0 >> qshift;
    const int ea = slot_expert(sa), eb = slot_expert(min(sa + 1, n_act - 1));
    // group `quad` of the round (a group past the end asks for the last one's rows again and stores
    // nothing): its slot, its first neuron there, its expert as listed
    auto group_of = [&](int quad, int &slot, int &j0, int &e_raw) {
      const int qc = min(q0 + quad, q_hi - 1);
      slot = qc >> qshift;
      j0 = (qc - (slot << qshift)) * 4;
      e_raw = slot == sa ? ea : eb;
    };
    // lane (n, g) of the epilogue sits in group g of the wave's tile
    const bool valid = q0 + 4 * tile + g < q_hi;
    int slot, j0, e_raw;
    group_of(4 * tile + g, slot, j0, e_raw);
    const bool e_ok = (unsigned)e_raw < (unsigned)E;   // always, with ROUTE
    const int e = min(max(e_raw, 0), E - 1);
    // what the epilogue needs of the lane's expert and token, asked for ahead of the weights: the
    // gain (ROUTE), or the score and the mask word; where a vector is absent x stands in as an
    // address and the value is dropped
    [[maybe_unused]] float gn_ld = 1.0f, f_ld = 0.0f;
    [[maybe_unused]] uint64_t m_ld = ~0ull;
    if constexpr (ROUTE) {
      const float *gp = L.g_rms ? L.g_rms + (size_t)layer * E + e : x;
      gn_ld = *gp;
    } else {
      const int tk = min(tok, k - 1);
      f_ld = scores[(size_t)tk * E + e];
      const uint64_t *mp = token_mask ? token_mask + (size_t)tk * W + (e >> 6) : reinterpret_cast<const uint64_t *>(x);
      m_ld = *mp;
    }
    // the weights: whole lines, non-temporal (load_stream): a[m][2 p] is line p of the tile's rows
    // 0-7 (groups 0 and 1), a[m][2 p + 1] of rows 8-15 (groups 2 and 3), lane = 8 row + piece
    const char *row[NM][2];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      int sl_l, j_l, e_l;
      group_of(4 * tile + 2 * hh + (lane >> 5), sl_l, j_l, e_l);
      e_l = min(max(e_l, 0), E - 1);
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const char *w = static_cast<const char *>(m == 0 ? L.w_up : L.w_gate);
        row[m][hh] = w + ((((size_t)layer * E + e_l) * d_e + j_l + ((lane >> 3) & 3)) * d + kq * (d / 4)) * 2 + line_byte(lane);
      }
    }
    uint4 a[NM][FW];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int i = 0; i < FH; ++i) a[m][i] = load_stream(row[m][i & 1] + (i >> 1) * 128);
    __builtin_amdgcn_sched_barrier(0);
    if (first) {
      // this wave's half of x as B operands, into LDS for the other tile's wave of the same quarter
#pragma unroll
      for (int i = 0; i < FH; ++i) {
        const uint4 xb = lanes_from(xraw[i], x_src);
        const float v[4] = {__uint_as_float(xb.x), __uint_as_float(xb.y), __uint_as_float(xb.z), __uint_as_float(xb.w)};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          split_bf16(v[q], hi[q], lo[q]);
          if (tok >= k) hi[q] = lo[q] = 0u;
        }
        const uint32_t hw0 = hi[0] | hi[1] << 16, hw1 = hi[2] | hi[3] << 16;
        const uint32_t lw0 = lo[0] | lo[1] << 16, lw1 = lo[2] | lo[3] << 16;
        // lane n < 8 keeps its hi words and sends its lo words; lane n + 8 does the opposite
        const uint32_t r0 = __shfl_xor(half ? hw0 : lw0, 8, kWave);
        const uint32_t r1 = __shfl_xor(half ? hw1 : lw1, 8, kWave);
        xS[(kq * FW + tile * FH + i) * 64 + lane] = half ? make_uint4(r0, r1, lw0, lw1) : make_uint4(hw0, hw1, r0, r1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int i = FH; i < FW; ++i) a[m][i] = load_stream(row[m][i & 1] + (i >> 1) * 128);
    __builtin_amdgcn_sched_barrier(0);
    if (first) __syncthreads();   // every B operand of the contraction is in LDS
    // score and mask bit of this lane's token, for the epilogue
    float f = 0.0f;
    bool on = false;
    if (kq == 0 && tok < k) {
      if constexpr (ROUTE) {
        const float a0 = pre_s[tok][e];
        const float a1v = a0 > 0.0f ? a0 : 0.0f;
        const float gn = L.g_rms ? gn_ld : 1.0f;
        f = a1v > 0.0f ? gn * a1v / rms_s[tok] : 0.0f;
        on = (tmask_s[tok][e >> 6] >> (e & 63)) & 1;
      } else {
        f = f_ld;
        on = e_ok && (token_mask ? (m_ld >> (e & 63)) & 1 : true);
      }
    }
    f32x4 acc[NM];
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < FW; i += 2) {   // a line: two K-steps
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        uint4 f0, f1;
        line_operands(a[m][i], a[m][i + 1], lsrc, f0, f1);
        acc[m] = mfma16(f0, xS[(kq * FW + i) * 64 + lane], acc[m]);
        acc[m] = mfma16(f1, xS[(kq * FW + i + 1) * 64 + lane], acc[m]);
      }
    }
    if (!first) __syncthreads();   // the epilogue waves have read the previous round's partial tiles
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) red[wave][m][q][lane] = acc[m][q];
    __syncthreads();
    if (kq == 0) {   // uniform over the wave
      const int w0 = tile * 4;
      uint32_t packed[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float u = (red[w0][0][q][lane] + red[w0 + 1][0][q][lane]) + (red[w0 + 2][0][q][lane] + red[w0 + 3][0][q][lane]);
        u += __shfl_xor(u, 8, kWave);
        float h;
        if (NM == 2) {
          float gt = (red[w0][NM - 1][q][lane] + red[w0 + 1][NM - 1][q][lane]) +
                     (red[w0 + 2][NM - 1][q][lane] + red[w0 + 3][NM - 1][q][lane]);
          gt += __shfl_xor(gt, 8, kWave);
          h = swish(gt) * u;
        } else {
          h = swish(u);
        }
        uint32_t hi, lo;
        split_bf16(on ? f * h : 0.0f, hi, lo);
        packed[q] = n < 8 ? hi : lo;
      }
      if (valid)
        store_stream(mid_entry(midB, (size_t)slot * (d_e / 32), j0 >> 4, (j0 >> 2) & 3, n),
                     make_uint2(packed[0] | packed[1] << 16, packed[2] | packed[3] << 16));
    }
  }
  if (ROUTE && writer) {   // the chunk's outputs of the router (wave t: token t) and of the union
    if (wave < k) {
      const int t = wave;
#pragma unroll
      for (int wd = 0; wd < kMaxMaskWords; ++wd) {
        const int i = wd * 64 + lane;
        if (wd < W) {
          if (lane == 0) ro.token_mask[(size_t)t * W + wd] = tmask_s[t][wd];
          if (i < E) {
            const float a0 = pre_s[t][i];
            const float a1v = a0 > 0.0f ? a0 : 0.0f;
            const float gn = L.g_rms ? L.g_rms[(size_t)layer * E + i] : 1.0f;
            ro.scores[(size_t)t * E + i] = a1v > 0.0f ? gn * a1v / rms_s[t] : 0.0f;
          }
        }
      }
    }
    if (wave == 0) write_union();
  }
}

// ------------------------------------------------------------------------------------------------ down

// KSD = d_e / 32 K-steps per slot, MW row tiles (16 output columns each) per wave, RING loads in
// flight per lane.  With splits > 1 the union's slots are divided among `splits` workgroups per
// (chunk, column block); each writes its partial sum to out + split * split_stride and a second
// kernel adds them in a fixed order (used when a launch has too few chunks to fill the chip).
__host__ __device__ inline bool down_by_xcd(int64_t n_chunks) { return n_chunks >= 64; }
__host__ __device__ inline int64_t down_grid_chunks(int64_t n_chunks) {
  return down_by_xcd(n_chunks) ? (n_chunks + 7) / 8 * 8 : n_chunks;
}

template <int NB, int KSD, int MW, int RING>
__global__ __launch_bounds__(kThreads, 2) void down_stream_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int64_t n_chunks, int k, int col_blocks, int splits,
    const uint16_t *__restrict__ midB, const uint32_t *__restrict__ tok_bits, const uint4 *__restrict__ zero16,
    float *__restrict__ out, size_t split_stride, int one_token) {
  constexpr int kFrag = KSD * MW;             // weight fragments per slot and wave
  static_assert(kFrag % RING == 0, "ring must divide the fragments of a slot");
  constexpr int kStage = KSD * NB * 64;       // uint4 of mid per slot
  constexpr int kPerThread = (kStage + kThreads - 1) / kThreads;
  constexpr int NA = acc_tiles(NB);
  __shared__ uint4 midS[2][kStage];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4;
  const int lsrc = line_src(lane);
  const int E = L.E, d = L.d;
  constexpr int d_e = KSD * 32;
  // Every workgroup of a chunk stages the chunk's whole mid (16 NB rows of d_e per slot): spread
  // over the XCDs, as consecutive block ids are, the col_blocks x splits workgroups of a chunk each
  // pulled it through the fabric (at k = 32, d_e = 128: 64 KiB of mid per 512 KiB of W_down, 12 %
  // on top of the weight bytes).  Block v runs on XCD v mod 8, so a chunk's workgroups get ids
  // that differ by multiples of 8 and share the mid in one L2.
  // A handful of chunks keep the plain order: their few workgroups must spread over all XCDs.
  const int per_chunk = col_blocks * splits;
  const bool by_xcd = down_by_xcd(n_chunks);
  const int64_t q = by_xcd ? blockIdx.x >> 3 : blockIdx.x;
  const int64_t c = by_xcd ? (q / per_chunk) * 8 + (blockIdx.x & 7) : q / per_chunk;
  if (c >= n_chunks) return;   // the grid is rounded up to 8 chunks
  const int within = (int)(q % per_chunk);
  const int sp = within % splits;
  const int col0 = (within / splits) * (4 * MW * 16) + wave * (MW * 16);
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  const int n_act = active_idx ? min(max(n_active[c], 0), E) : E;
  const int s_lo = (int)((int64_t)n_act * sp / splits), s_hi = (int)((int64_t)n_act * (sp + 1) / splits);
  float *y = out + (size_t)sp * split_stride;

  auto slot_expert = [&](int s) {
    int e = active_idx ? active_idx[c * E + s] : s;
    return min(max(e, 0), E - 1);
  };
  auto slot_ptr = [&](int e) -> const char * {
    const size_t row = ((size_t)layer * E + e) * d + col0 + line_row(lane);
    return static_cast<const char *>(L.w_down) + row * (d_e * 2) + line_byte(lane);
  };
  // Load f of a slot (two loads per 128-byte line, see load_stream): row tile f / KSD, line
  // (f % KSD) / 2 of its rows, rows 0-7 for even f and rows 8-15 for odd f; the pair holds the A
  // operands of K-steps f % KSD and f % KSD + 1.
  auto frag_off = [&](int f) {
    return (size_t)(f / KSD) * 16 * d_e * 2 + (size_t)((f % KSD) >> 1) * 128 + (size_t)(f & 1) * 8 * d_e * 2;
  };

  f32x4 acc[MW][NA];
#pragma unroll
  for (int a = 0; a < MW; ++a)
#pragma unroll
    for (int q = 0; q < NA; ++q) acc[a][q] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (s_hi > s_lo) {
    uint4 ring[RING];
    int e = slot_expert(s_lo);
    {
      const char *p = slot_ptr(e);
#pragma unroll
      for (int i = 0; i < RING; ++i) ring[i] = load_stream(p + frag_off(i));
    }
    const bool one = NB == 1 && one_token;   // mid_one_token: rows [hi | lo][d_e] per slot
    const uint4 *mid_c = reinterpret_cast<const uint4 *>(midB + (size_t)c * E * (one ? 2 : NB * 16) * d_e);
    // B-operand order in LDS is [K-step][NB][lane = gg * 16 + n] of 8 bf16.  k <= 8: mid is stored
    // like that.  k > 8: mid is token-major and holds only the rows of the tokens in `bits`; entry
    // (K-step, fragment bf, gg, n) is 16 bytes of row (token 16 (bf / 2) + n, hi or lo = bf & 1),
    // or of the block of zeros.
    auto slot_bits = [&](int s) { return NB == 1 ? 0u : tok_bits[c * E + min(s, s_hi - 1)]; };
    auto stage_src = [&](int s, int idx, uint32_t bits) -> const uint4 * {
      if (one) {   // column 0: the token's hi part, column 8: its lo part, the others zero
        const int ln = idx & 63, ks = idx >> 6, n = ln & 15, gg = ln >> 4;
        return (n & 7) == 0 ? mid_c + ((size_t)s * 2 + (n >> 3)) * (d_e / 8) + ks * 4 + gg : zero16;
      }
      if (NB == 1) return mid_c + (size_t)s * kStage + idx;
      const int ln = idx & 63, bf = (idx >> 6) % NB, ks = idx / (64 * NB);
      const int n = ln & 15, gg = ln >> 4, t = (bf >> 1) * 16 + n;
      const uint4 *row = mid_c + ((size_t)s * (NB * 16) + t * 2 + (bf & 1)) * (d_e / 8) + ks * 4 + gg;
      return (bits >> t) & 1 ? row : zero16;
    };
    {
      const uint32_t bits = slot_bits(s_lo);
#pragma unroll
      for (int q = 0; q < kPerThread; ++q) {
        const int idx = tid + q * kThreads;
        if (idx < kStage) midS[0][idx] = *stage_src(s_lo, idx, bits);
      }
    }
    __syncthreads();
    // the token bits of the slot staged in iteration s (slot s + 1) are fetched an iteration ahead
    uint32_t bits_stage = slot_bits(s_lo + 1), bits_after = slot_bits(s_lo + 2);

    for (int s = s_lo; s < s_hi; ++s) {
      const bool has_next = s + 1 < s_hi;
      const int e_n = has_next ? slot_expert(s + 1) : e;
      const char *nxt = slot_ptr(e_n);
      // mid of the next slot goes straight into the other LDS buffer (LDS-direct loads: lane j's
      // 16 bytes land at the wave's base + 16 j; no staging registers, no LDS stores).  The last
      // slot re-reads itself: harmless, and it keeps the number of loads in flight the same.
      const int s_stage = has_next ? s + 1 : s;
      uint4 *stage_dst = midS[(s - s_lo + 1) & 1];
#pragma unroll
      for (int q = 0; q < kPerThread; ++q) {
        const int idx = tid + q * kThreads;
        if (q * kThreads + wave * 64 < kStage)   // uniform over the wave (kStage is a multiple of 64)
          load_to_lds16(stage_src(s_stage, idx, bits_stage), stage_dst + q * kThreads + wave * 64);
      }
      bits_stage = bits_after;
      bits_after = slot_bits(s + 3);
      const char *cur = slot_ptr(e);
      const uint4 *bS = midS[(s - s_lo) & 1];
#pragma unroll
      for (int tile = 0; tile < MW; ++tile) {
#pragma unroll
        for (int ks = 0; ks < KSD; ks += 2) {   // a line: two K-steps
          const int f = tile * KSD + ks;
          uint4 fr[2];
          line_operands(ring[f % RING], ring[f % RING + 1], lsrc, fr[0], fr[1]);
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int bf = 0; bf < NB; ++bf)
              acc[tile][acc_of(NB, bf)] =
                  mfma16(fr[h], bS[((ks + h) * NB + bf) * 64 + lane], acc[tile][acc_of(NB, bf)]);
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int fn = f + h + RING;
            if (fn < kFrag) ring[(f + h) % RING] = load_stream(cur + frag_off(fn));
            else if (has_next) ring[(f + h) % RING] = load_stream(nxt + frag_off(fn - kFrag));
          }
        }
      }
      // loads return in issue order: everything older than the weight loads issued since (at
      // most RING are outstanding) has arrived, and with it the staged mid
      static_assert(kFrag >= RING, "the ring is refilled at least once per slot after the staging loads");
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(RING) : "memory");
      __syncthreads();
      e = e_n;
    }
  }

  const int n = lane & 15;
  // The unsplit launch writes y as whole 128-byte lines: the values of two column tiles (64 bytes
  // of a token's row each) are brought together so that the 64 lanes of a store cover 8 token rows
  // x 128 bytes, lane = 8 row + piece.  Piece p is element group p & 3 of the first (p < 4) or
  // second tile; it sits in lane (p & 3) * 16 + token.  k <= 8: lanes n and n + 8 hold the same
  // totals, so lane n sends the first tile's and lane n + 8 the second's.  k > 8: rows 0-7 and
  // rows 8-15 of a 16-token tile go out as two stores; for each, the lanes of the other eight
  // tokens pass on their partner's second-tile values (a rotation by 8 within 16 lanes).
  if (splits == 1 && MW % 2 == 0) {
    const int r = lane >> 3, p = lane & 7;
#pragma unroll
    for (int q = 0; q < NA; ++q) {
#pragma unroll
      for (int pair = 0; pair < MW / 2; ++pair) {
        float a[4], b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          a[j] = acc[2 * pair][q][j];
          b[j] = acc[2 * pair + 1][q][j];
          if (NB == 1) {
            a[j] += __shfl_xor(a[j], 8, kWave);
            b[j] += __shfl_xor(b[j], 8, kWave);
          }
        }
#pragma unroll
        for (int h = 0; h < (NB == 1 ? 1 : 2); ++h) {
          const bool first = NB == 1 ? n < 8 : (n >> 3) == h;   // this lane sends its first-tile values
          const int src = ((p & 3) * 16 + r + (NB == 1 ? (p >= 4 ? 8 : 0) : ((p >= 4) == (h == 0) ? 8 : 0))) * 4;
          float4 v;
          float *vp = reinterpret_cast<float *>(&v);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t other = NB == 1 ? __float_as_uint(b[j]) : ror8_into<0xf>(0u, __float_as_uint(b[j]));
            const uint32_t send = first ? __float_as_uint(a[j]) : other;
            vp[j] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)send));
          }
          const int t = NB == 1 ? r : q * 16 + 8 * h + r;
          if (t < k) store_stream(reinterpret_cast<float4 *>(y + (c * k + t) * d + col0 + pair * 32 + 4 * p), v);
        }
      }
    }
    return;
  }
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
      if (writer) {
        float4 *dst = reinterpret_cast<float4 *>(y + (c * k + t) * d + col0 + tile * 16 + 4 * g);
        if (splits > 1) *dst = v;          // partial sums: the reduce kernel reads them right away
        else store_stream(dst, v);
      }
    }
  }
}

// The same (chunk, column block, split of the slots) decomposition for a handful of chunks of at
// most 8 tokens, where a workgroup has three or four slots and the launch is over in a few
// microseconds: a ring that asks for one slot while it works on the one before pays a trip to
// memory per slot, one after the other.  Here everything a workgroup needs is asked for at once -
// the chunk's list (count and entries together, neither waiting for the other), then mid and the
// weights of up to kFewSlots slots (more than that in further rounds) - and waited for once.
// Weights are requested with the lanes in memory order (lane = 4 row + g: the 64 bytes a row
// gives to a fragment by four neighbouring lanes) and permuted into operand order in registers,
// as in up_split_kernel.  Slots and K-steps are added in the order of down_stream_kernel: the
// same bits.
constexpr int kFewSlots = 4;

// One round of NS slots starting at slot s0.  No branch around any load or matrix instruction: at
// a join the compiler's counted waits collapse to "wait for everything", which puts the slots'
// trips to memory back one after the other; hence one instantiation per number of slots.
template <int KSD, int MW, int NS>
__device__ __forceinline__ void down_few_round(const LayerView &L, int layer, const int (&ent)[kMaxMaskWords], int s0,
                                               int col0, const uint4 *__restrict__ mid_c,
                                               uint4 (&midS)[kFewSlots][KSD * 64], f32x4 (&acc)[MW]) {
  constexpr int kFrag = KSD * MW;        // weight fragments per slot and wave
  constexpr int kStage = KSD * 64;       // uint4 of mid per slot
  constexpr int kPerThread = (kStage + kThreads - 1) / kThreads;
  constexpr int d_e = KSD * 32;
  const int tid = threadIdx.x, lane = tid & 63;
  const int lsrc = line_src(lane);
  // mid first: it is waited for first, and loads come back in the order they were asked for
  uint4 m[NS][kPerThread];
#pragma unroll
  for (int j = 0; j < NS; ++j)
#pragma unroll
    for (int q = 0; q < kPerThread; ++q)
      m[j][q] = mid_c[(size_t)(s0 + j) * kStage + min(tid + q * kThreads, kStage - 1)];
  __builtin_amdgcn_sched_barrier(0);
  uint4 w[NS][kFrag];
#pragma unroll
  for (int j = 0; j < NS; ++j) {
    const int sl = s0 + j;
    int e = 0;
#pragma unroll
    for (int wd = 0; wd < kMaxMaskWords; ++wd) {
      const int v = __builtin_amdgcn_readlane(ent[wd], sl & 63);
      e = (sl >> 6) == wd ? v : e;
    }
    e = min(max(e, 0), L.E - 1);
    // whole lines, non-temporal (load_stream): load f = row tile f / KSD, line (f % KSD) / 2, rows
    // 0-7 for even f and rows 8-15 for odd f, lane = 8 row + piece
    const size_t row = ((size_t)layer * L.E + e) * L.d + col0 + line_row(lane);
    const char *p = static_cast<const char *>(L.w_down) + row * (d_e * 2) + line_byte(lane);
#pragma unroll
    for (int f = 0; f < kFrag; ++f)
      w[j][f] = load_stream(p + (size_t)(f / KSD) * 16 * d_e * 2 + (size_t)((f % KSD) >> 1) * 128 +
                            (size_t)(f & 1) * 8 * d_e * 2);
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < NS; ++j)
#pragma unroll
    for (int q = 0; q < kPerThread; ++q) {
      const int idx = tid + q * kThreads;
      if (idx < kStage) midS[j][idx] = m[j][q];
    }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < NS; ++j)
#pragma unroll
    for (int f = 0; f < kFrag; f += 2) {   // a line: two K-steps
      uint4 f0, f1;
      line_operands(w[j][f], w[j][f + 1], lsrc, f0, f1);
      acc[f / KSD] = mfma16(f0, midS[j][(f % KSD) * 64 + lane], acc[f / KSD]);
      acc[f / KSD] = mfma16(f1, midS[j][(f % KSD + 1) * 64 + lane], acc[f / KSD]);
    }
}

template <int KSD, int MW>
__global__ __launch_bounds__(kThreads, 2) void down_few_kernel(
    LayerView L, const int32_t *__restrict__ chunk_layer, const int32_t *__restrict__ active_idx,
    const int32_t *__restrict__ n_active, int64_t n_chunks, int k, int col_blocks, int splits,
    const uint16_t *__restrict__ midB, float *__restrict__ out, size_t split_stride) {
  constexpr int d_e = KSD * 32;
  __shared__ uint4 midS[kFewSlots][KSD * 64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4;
  const int E = L.E, d = L.d;
  const int per_chunk = col_blocks * splits;
  const int64_t c = blockIdx.x / per_chunk;
  if (c >= n_chunks) return;
  const int within = (int)(blockIdx.x % per_chunk);
  const int sp = within % splits;
  const int col0 = (within / splits) * (4 * MW * 16) + wave * (MW * 16);
  const int layer = clamp_layer(chunk_layer, c, L.n_layers);
  // the chunk's list: lane l holds entries l, l + 64, ...
  int n_act = E;
  int ent[kMaxMaskWords];
#pragma unroll
  for (int wd = 0; wd < kMaxMaskWords; ++wd) {
    const int i = wd * 64 + lane;
    ent[wd] = i;
    if (active_idx && i < E) ent[wd] = active_idx[c * E + i];
  }
  if (active_idx) n_act = min(max(n_active[c], 0), E);
  const int s_lo = (int)((int64_t)n_act * sp / splits), s_hi = (int)((int64_t)n_act * (sp + 1) / splits);
  float *y = out + (size_t)sp * split_stride;
  const uint4 *mid_c = reinterpret_cast<const uint4 *>(midB + (size_t)c * E * 16 * d_e);

  f32x4 acc[MW];
#pragma unroll
  for (int a = 0; a < MW; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int s0 = s_lo; s0 < s_hi; s0 += kFewSlots) {   // uniform over the workgroup
    if (s0 != s_lo) __syncthreads();                  // every wave has read the round before out of midS
    switch (min(kFewSlots, s_hi - s0)) {
      case 1: down_few_round<KSD, MW, 1>(L, layer, ent, s0, col0, mid_c, midS, acc); break;
      case 2: down_few_round<KSD, MW, 2>(L, layer, ent, s0, col0, mid_c, midS, acc); break;
      case 3: down_few_round<KSD, MW, 3>(L, layer, ent, s0, col0, mid_c, midS, acc); break;
      default: down_few_round<KSD, MW, 4>(L, layer, ent, s0, col0, mid_c, midS, acc); break;
    }
  }

  const int n = lane & 15, t = n & 7;
  const bool writer = n < 8 && t < k;
#pragma unroll
  for (int tile = 0; tile < MW; ++tile) {
    float4 v;
    float *vp = reinterpret_cast<float *>(&v);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float a = acc[tile][j];
      vp[j] = a + __shfl_xor(a, 8, kWave);
    }
    if (writer) *reinterpret_cast<float4 *>(y + (c * k + t) * d + col0 + tile * 16 + 4 * g) = v;
  }
}

template <int NB, int NM, int RT>
hipError_t launch_up(const LayerView &L, const int32_t *chunk_layer, const uint4 *xS, const float *scores,
                     const uint64_t *token_mask, const int32_t *active_idx, const int32_t *n_active,
                     const int32_t *items, const int32_t *total, int group, int64_t max_items, int k, uint16_t *midB,
                     uint32_t *tok_bits, bool one_token, hipStream_t s) {
  static PerDeviceOnce lds_limit, lds_limit_one;   // one per instantiation
  const int64_t grid = (std::min<int64_t>(max_items, (int64_t)num_cus() * 2) + 7) / 8 * 8;
  if constexpr (NB == 1) {
    if (one_token) {
      auto kern = up_stream_kernel<NB, NM, RT, true>;
      const hipError_t e = lds_limit_one.run([&] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kXBytes);
      });
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), kXBytes, s, L, chunk_layer, xS, scores, token_mask,
                         active_idx, n_active, items, total, group, k, midB, tok_bits);
      return hipGetLastError();
    }
  }
  auto kern = up_stream_kernel<NB, NM, RT, false>;
  const hipError_t e = lds_limit.run([&] {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kXBytes);
  });
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), kXBytes, s, L, chunk_layer, xS, scores, token_mask,
                     active_idx, n_active, items, total, group, k, midB, tok_bits);
  return hipGetLastError();
}

template <int NB, int NM, int RT, int G, int HW>
hipError_t launch_up_db(const LayerView &L, const int32_t *chunk_layer, const uint4 *xS, const float *scores,
                        const uint64_t *token_mask, const int32_t *active_idx, const int32_t *n_active,
                        const int32_t *items, const int32_t *total, int64_t max_items, int k, uint16_t *midB,
                        uint32_t *tok_bits, hipStream_t s) {
  static PerDeviceOnce lds_limit;   // one per instantiation
  auto kern = up_stream_db_kernel<NB, NM, RT, G, HW>;
  const hipError_t e = lds_limit.run([&] {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kXBytes);
  });
  if (e != hipSuccess) return e;
  const int64_t grid = (std::min<int64_t>(max_items, (int64_t)num_cus() * 2 / HW) + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads * HW), kXBytes, s, L, chunk_layer, xS, scores, token_mask,
                     active_idx, n_active, items, total, k, midB, tok_bits);
  return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const float *__restrict__ part, int splits,
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

template <int NB, int KSD>
hipError_t launch_down(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                       const int32_t *n_active, int64_t n_chunks, int k, const uint16_t *midB, const uint32_t *tok_bits,
                       const uint4 *zero16, float *part, float *y, hipStream_t s) {
  const int splits = down_splits(L, n_chunks);
  const size_t stride = (size_t)n_chunks * k * L.d;
  const int one_token = NB == 1 && mid_one_token(L, n_chunks, k) ? 1 : 0;
  if (splits == 0) {
    constexpr int MW = (NB == 4 && KSD >= 8) ? 4 : 8;   // 8 row tiles x 2 accumulator tiles do not fit beside 64 fragments of addresses
    const int col_blocks = L.d / (4 * MW * 16);
    const int64_t grid = down_grid_chunks(n_chunks) * col_blocks;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((down_stream_kernel<NB, KSD, MW, kRing>), dim3((unsigned)grid), dim3(kThreads), 0, s, L,
                       chunk_layer, active_idx, n_active, n_chunks, k, col_blocks, 1, midB, tok_bits, zero16, y, stride,
                       one_token);
    return hipGetLastError();
  }
  constexpr int MW = 8 / KSD;
  const int col_blocks = L.d / (4 * MW * 16);
  if (NB == 1 && splits > 1 && !down_by_xcd(n_chunks)) {   // a handful of short chunks: everything asked for at once
    const int64_t grid = n_chunks * col_blocks * splits;
    hipLaunchKernelGGL((down_few_kernel<KSD, MW>), dim3((unsigned)grid), dim3(kThreads), 0, s, L, chunk_layer, active_idx,
                       n_active, n_chunks, k, col_blocks, splits, midB, part, stride);
  } else {
    const int64_t grid = down_grid_chunks(n_chunks) * col_blocks * splits;
    hipLaunchKernelGGL((down_stream_kernel<NB, KSD, MW, 8>), dim3((unsigned)grid), dim3(kThreads), 0, s, L, chunk_layer,
                       active_idx, n_active, n_chunks, k, col_blocks, splits, midB, tok_bits, zero16,
                       splits > 1 ? part : y, stride, one_token);
  }
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || splits == 1) return err;
  const size_t n4 = stride / 4;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)std::min<size_t>((n4 + kThreads - 1) / kThreads, 1024)),
                     dim3(kThreads), 0, s, part, splits, stride, n4, y);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_worklist(const int32_t *n_active, int64_t n_chunks, int E, int group, int32_t *items,
                           int32_t *total, hipStream_t s) {
  if (group < 1 || group > kMaxGroup) return hipErrorInvalidValue;
  const int64_t blocks = (n_chunks + kListChunks - 1) / kListChunks;
  if (blocks < 1 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(worklist_kernel, dim3((unsigned)blocks), dim3(kListChunks), 0, s, n_active, n_chunks, E, group,
                     items, total);
  return hipGetLastError();
}

// Workgroups of up_split_kernel: one per item; for a single chunk no more than the two per CU
// that can be resident (its workgroups then loop over their items, all of the one chunk).
static int split_grid(int64_t n_chunks, int total) { return n_chunks == 1 ? std::min(total, 2 * num_cus()) : total; }

bool stream_supported(const LayerView &L, int wdtype, int k) {
  return wdtype == BLOCKFFN_BF16 && k <= 32 && L.d % 512 == 0 &&
         (L.d_e == 64 || L.d_e == 128 || L.d_e == 256);
}

size_t stream_workspace_bytes(const LayerView &L, int64_t n_chunks, int k) {
  // mid as bf16 hi/lo fragments [chunk][slot][NB][16][d_e], then the item count and the item list
  size_t b = mid_bytes(L, n_chunks, k) + item_bytes(L, n_chunks) + xs_bytes(L, n_chunks, k);
  const int splits = down_splits(L, n_chunks);
  if (splits > 1) b += ((size_t)splits * n_chunks * k * L.d * sizeof(float) + 255) & ~(size_t)255;
  return b;
}

hipError_t launch_up_stream(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                            const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, void *ws, hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  if (n_chunks * L.E > 0x7fffffffLL) return hipErrorInvalidValue;
  StreamWs w = carve_stream(L, n_chunks, k, ws);
  const int NB = b_frags(k), RT = L.d_e / 64;
  const int64_t max_items = n_chunks * L.E;
  if (few_chunks(L, n_chunks, k)) {
    if (n_chunks == 1) {   // one workgroup per CU, equal shares of the listed experts' rows
      const int fw = L.d / 128;
      const size_t lds = (size_t)4 * fw * 64 * sizeof(uint4);
#define BLOCKFFN_CHIP(nm, fw_)                                                                                  \
  {                                                                                                             \
    static PerDeviceOnce lds_limit;                                                                             \
    auto kern = up_chip_kernel<nm, fw_, false>;                                                                 \
    const hipError_t e = lds_limit.run([&] {                                                                    \
      return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                 (int)lds);                                                                     \
    });                                                                                                         \
    if (e != hipSuccess) return e;                                                                              \
    hipLaunchKernelGGL(kern, dim3((unsigned)num_cus()), dim3(kChipThreads), lds, s, L, chunk_layer, x, scores,  \
                       token_mask, active_idx, n_active, k, w.midB, RouteOut{});                                \
  }
      if (fw == 16) { if (gated) BLOCKFFN_CHIP(2, 16) else BLOCKFFN_CHIP(1, 16) }
      else { if (gated) BLOCKFFN_CHIP(2, 8) else BLOCKFFN_CHIP(1, 8) }
#undef BLOCKFFN_CHIP
      return hipGetLastError();
    }
    // few chunks: one workgroup per (item, 16-row tile)
    const int total = (int)(max_items * (L.d_e / 16));
    const dim3 grid((unsigned)split_grid(n_chunks, total));
#define BLOCKFFN_SPLIT(nm, fw)                                                                             \
  hipLaunchKernelGGL((up_split_kernel<nm, fw, false>), grid, dim3(kThreads), 0, s, L, chunk_layer, x, scores, token_mask, \
                     active_idx, n_active, k, w.midB, RouteOut{}, total)
    if (L.d == 2048) { if (gated) BLOCKFFN_SPLIT(2, 16); else BLOCKFFN_SPLIT(1, 16); }
    else { if (gated) BLOCKFFN_SPLIT(2, 8); else BLOCKFFN_SPLIT(1, 8); }
#undef BLOCKFFN_SPLIT
    return hipGetLastError();
  }
  // Two slots per item when the whole contraction of x fits in LDS: the 64 KiB of x are then
  // fetched and split once per 2 experts.  (With more K-chunks LDS is refilled per K-chunk anyway.)
  // k > 8 with more than one LDS fill per slot: the double-buffered kernel, where the accumulators
  // of more than one slot fit in registers (otherwise it has nothing over the single buffer).
  // 8 fragments per tile (k > 16) need an even number of tiles per slot.
  const int nm = gated ? 2 : 1;
  const bool use_db = L.d > 2048 / NB && up_db_shape(NB, RT, nm);
  const int group = use_db ? up_group(NB, RT, nm) * up_halves(NB, RT, nm) : (L.d <= 2048 / NB ? 2 : 1);
  hipError_t err = launch_worklist(n_active, n_chunks, L.E, group, w.items, w.total, s);
  if (err != hipSuccess) return err;
  {
    const int64_t entries = n_chunks * (int64_t)(L.d / 32) * NB * 64;
    const int64_t blocks = (entries + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (NB == 1 && mid_one_token(L, n_chunks, k))
      hipLaunchKernelGGL(split_x1_kernel, dim3((unsigned)((n_chunks * (L.d / 32) * 8 + kThreads - 1) / kThreads)),
                         dim3(kThreads), 0, s, x, n_chunks, L.d, w.xS);
    else if (NB == 1)
      hipLaunchKernelGGL(split_x_kernel<1>, dim3((unsigned)blocks), dim3(kThreads), 0, s, x, n_chunks, k, L.d, w.xS);
    else if (NB == 2)
      hipLaunchKernelGGL(split_x_kernel<2>, dim3((unsigned)blocks), dim3(kThreads), 0, s, x, n_chunks, k, L.d, w.xS);
    else
      hipLaunchKernelGGL(split_x_kernel<4>, dim3((unsigned)blocks), dim3(kThreads), 0, s, x, n_chunks, k, L.d, w.xS);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
#define BLOCKFFN_CASE(nb, nm, rt)                                                                         \
  if (NB == nb && (gated ? 2 : 1) == nm && RT == rt) {                                                    \
    if constexpr (up_db_shape(nb, rt, nm))                                                                \
      if (use_db)                                                                                         \
        return launch_up_db<nb, nm, rt, up_group(nb, rt, nm), up_halves(nb, rt, nm)>(                   \
            L, chunk_layer, w.xS, scores, token_mask, active_idx, n_active, w.items, w.total, max_items, k, \
            w.midB, w.tok_bits, s);                                                                       \
    return launch_up<nb, nm, rt>(L, chunk_layer, w.xS, scores, token_mask, active_idx, n_active, w.items, w.total, \
                                 group, max_items, k, w.midB, w.tok_bits, mid_one_token(L, n_chunks, k), s);  \
  }
  BLOCKFFN_CASE(1, 1, 1) BLOCKFFN_CASE(1, 1, 2) BLOCKFFN_CASE(1, 1, 4)
  BLOCKFFN_CASE(1, 2, 1) BLOCKFFN_CASE(1, 2, 2) BLOCKFFN_CASE(1, 2, 4)
  BLOCKFFN_CASE(2, 1, 1) BLOCKFFN_CASE(2, 1, 2) BLOCKFFN_CASE(2, 1, 4)
  BLOCKFFN_CASE(2, 2, 1) BLOCKFFN_CASE(2, 2, 2) BLOCKFFN_CASE(2, 2, 4)
  BLOCKFFN_CASE(4, 1, 1) BLOCKFFN_CASE(4, 1, 2) BLOCKFFN_CASE(4, 1, 4)
  BLOCKFFN_CASE(4, 2, 1) BLOCKFFN_CASE(4, 2, 2) BLOCKFFN_CASE(4, 2, 4)
#undef BLOCKFFN_CASE
  return hipErrorInvalidValue;
}

bool few_routed_supported(const LayerView &L, int wdtype, int64_t n_chunks, int k) {
  return stream_supported(L, wdtype, k) && few_chunks(L, n_chunks, k) && router_few(L, n_chunks, k) &&
         (size_t)n_chunks * k * L.E * sizeof(float) <= xs_bytes(L, n_chunks, k);
}

float *few_preact_buffer(const LayerView &L, int64_t n_chunks, int k, void *ws) {
  return reinterpret_cast<float *>(carve_stream(L, n_chunks, k, ws).xS);   // the split x of larger launches lives here
}

hipError_t launch_up_few_routed(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                                int64_t n_chunks, int k, void *ws, float *scores, uint64_t *token_mask,
                                uint64_t *union_mask, int32_t *active_idx, int32_t *n_active, int64_t *stats,
                                hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  if (!few_chunks(L, n_chunks, k) || (size_t)n_chunks * k * L.E * sizeof(float) > xs_bytes(L, n_chunks, k))
    return hipErrorInvalidValue;
  StreamWs w = carve_stream(L, n_chunks, k, ws);
  RouteOut ro{reinterpret_cast<const float *>(w.xS), scores, token_mask, union_mask, active_idx, n_active,
              reinterpret_cast<unsigned long long *>(stats)};
  if (n_chunks == 1) {   // one workgroup per CU, equal shares of the union's rows
    const int fw = L.d / 128;
    const size_t lds = (size_t)4 * fw * 64 * sizeof(uint4);
#define BLOCKFFN_CHIP(nm, fw_)                                                                                  \
  {                                                                                                             \
    static PerDeviceOnce lds_limit;                                                                             \
    auto kern = up_chip_kernel<nm, fw_, true>;                                                                  \
    const hipError_t e = lds_limit.run([&] {                                                                    \
      return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                 (int)lds);                                                                     \
    });                                                                                                         \
    if (e != hipSuccess) return e;                                                                              \
    hipLaunchKernelGGL(kern, dim3((unsigned)num_cus()), dim3(kChipThreads), lds, s, L, chunk_layer, x, nullptr, nullptr, \
                       nullptr, nullptr, k, w.midB, ro);                                                        \
  }
    if (fw == 16) { if (gated) BLOCKFFN_CHIP(2, 16) else BLOCKFFN_CHIP(1, 16) }
    else { if (gated) BLOCKFFN_CHIP(2, 8) else BLOCKFFN_CHIP(1, 8) }
#undef BLOCKFFN_CHIP
    return hipGetLastError();
  }
  const int total = (int)(n_chunks * L.E * (L.d_e / 16));
  const dim3 grid((unsigned)split_grid(n_chunks, total));
#define BLOCKFFN_SPLIT(nm, fw)                                                                                 \
  hipLaunchKernelGGL((up_split_kernel<nm, fw, true>), grid, dim3(kThreads), 0, s, L, chunk_layer, x, nullptr, nullptr, \
                     nullptr, nullptr, k, w.midB, ro, total)
  if (L.d == 2048) { if (gated) BLOCKFFN_SPLIT(2, 16); else BLOCKFFN_SPLIT(1, 16); }
  else { if (gated) BLOCKFFN_SPLIT(2, 8); else BLOCKFFN_SPLIT(1, 8); }
#undef BLOCKFFN_SPLIT
  return hipGetLastError();
}

hipError_t launch_down_stream(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                              const int32_t *n_active, int64_t n_chunks, int k, const void *ws, float *y,
                              hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  StreamWs w = carve_stream(L, n_chunks, k, const_cast<void *>(ws));
  const int NB = b_frags(k), KSD = L.d_e / 32;
#define BLOCKFFN_CASE(nb, ksd) \
  if (NB == nb && KSD == ksd) \
    return launch_down<nb, ksd>(L, chunk_layer, active_idx, n_active, n_chunks, k, w.midB, w.tok_bits, w.zero16, \
                                w.part, y, s);
  BLOCKFFN_CASE(1, 2) BLOCKFFN_CASE(1, 4) BLOCKFFN_CASE(1, 8)
  BLOCKFFN_CASE(2, 2) BLOCKFFN_CASE(2, 4) BLOCKFFN_CASE(2, 8)
  BLOCKFFN_CASE(4, 2) BLOCKFFN_CASE(4, 4) BLOCKFFN_CASE(4, 8)
#undef BLOCKFFN_CASE
  return hipErrorInvalidValue;
}

}  // namespace blockffn
