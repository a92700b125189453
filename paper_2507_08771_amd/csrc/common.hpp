// Shared device helpers of the gfx950 kernels: weight widening, 128-bit loads, wave64
// reductions, and the POD view of a layer that kernels take by value.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/blockffn.h"

namespace blockffn {

constexpr int kWave = 64;
constexpr int kMaxExperts = 256;
constexpr int kMaxMaskWords = kMaxExperts / 64;
constexpr int kMaxK = 512;
constexpr int kMaxDe = 1024;
constexpr int kMaxD = 16384;

// What a kernel needs to know about the layer; filled from blockffn_layer after validation.
struct LayerView {
  int d, E, d_e, n_layers, W;
  float eps;
  const void *w_router;
  const float *b_router;
  const float *g_rms;
  const void *w_up;
  const void *w_gate;
  const void *w_down;
};

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// Eight consecutive weights starting at element index `idx` (a multiple of 8), widened to fp32.
template <typename WT>
__device__ __forceinline__ void load8(const void *base, size_t idx, float (&w)[8]);

template <>
__device__ __forceinline__ void load8<float>(const void *base, size_t idx, float (&w)[8]) {
  const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + idx);
  float4 a = p[0], b = p[1];
  w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
  w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
}

template <>
__device__ __forceinline__ void load8<bf16_t>(const void *base, size_t idx, float (&w)[8]) {
  const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + idx);
  w[0] = bf16_lo(v.x); w[1] = bf16_hi(v.x);
  w[2] = bf16_lo(v.y); w[3] = bf16_hi(v.y);
  w[4] = bf16_lo(v.z); w[5] = bf16_hi(v.z);
  w[6] = bf16_lo(v.w); w[7] = bf16_hi(v.w);
}

// v of another lane of the same row of 16, chosen by a DPP control word (a VALU operand modifier:
// no trip through the LDS pipeline as a shuffle takes).
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the wave, the same bits in every lane: within a row of 16 by four DPP steps (lane ^ 1,
// lane ^ 2, the mirror lane of the half row, the mirror lane of the row: after each step the lanes
// that were combined hold the same value, a + b and b + a being the same), then the four rows in a
// fixed order.  A dozen VALU instructions where six shuffles cost six LDS round trips one after
// the other, which is what the short, latency-bound launches spend their time on.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_lane<0xB1>(v);    // quad_perm [1, 0, 3, 2]
  v += dpp_lane<0x4E>(v);    // quad_perm [2, 3, 0, 1]
  v += dpp_lane<0x141>(v);   // row_half_mirror
  v += dpp_lane<0x140>(v);   // row_mirror
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ uint64_t wave_or(uint64_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v |= __shfl_xor(v, off, kWave);
  return v;
}

__device__ __forceinline__ long long wave_sum_i64(long long v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// LDS-direct load: lane j's 16 bytes at `src` land in LDS at `dst` + 16 j (dst is uniform over
// the wave; it goes through M0).  Written as inline assembly on purpose: the compiler's wait
// insertion treats the builtin form as a store to LDS that any later LDS read may alias and puts
// `s_waitcnt vmcnt(0)` in front of that read, which serialises the very loads this is meant to
// keep in flight under the matrix work.  Issued this way the compiler does not count the load, so
// the caller must wait for it itself (`s_waitcnt vmcnt(n)`: loads return in issue order) and put
// a barrier between the wait and reads by other waves.
__device__ __forceinline__ void load_to_lds16(const void *src, void *dst) {
  typedef __attribute__((address_space(3))) void lds_void;
  const uint32_t lds_addr =
      __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void *)dst);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr), "v"(src)
               : "memory", "m0");
}

// The same with 4 bytes per lane: lane j's dword lands at dst + 4 j.
__device__ __forceinline__ void load_to_lds4(const void *src, void *dst) {
  typedef __attribute__((address_space(3))) void lds_void;
  const uint32_t lds_addr =
      __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void *)dst);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
               :
               : "s"(lds_addr), "v"(src)
               : "memory", "m0");
}

// Swish with beta = 1 (SiLU), full-precision exponential.
__device__ __forceinline__ float swish(float u) { return u / (1.0f + expf(-u)); }

__device__ __forceinline__ int clamp_layer(const int32_t *chunk_layer, int64_t c, int n_layers) {
  if (chunk_layer == nullptr) return 0;
  int l = chunk_layer[c];
  return l < 0 ? 0 : (l >= n_layers ? n_layers - 1 : l);
}

// ------------------------------------------------------------------------------------------------ host: per device
// The library keeps nothing per process that depends on the device: what it caches (the number
// of compute units, "this kernel's LDS limit has been raised") is kept per device ordinal, in
// atomics, so that threads driving different GPUs - or the same one - need no lock.
constexpr int kMaxDevices = 64;

// Ordinal of the calling thread's current device, or -1 (unknown, or beyond kMaxDevices: nothing is cached then).
inline int current_device() {
  int dev = -1;
  return hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices ? dev : -1;
}

// Compute units of the current device (256 if the runtime will not say).
inline int num_cus() {
  static std::atomic<int> cus[kMaxDevices];
  const int dev = current_device();
  if (dev >= 0) {
    const int known = cus[dev].load(std::memory_order_relaxed);
    if (known > 0) return known;
  }
  int n = 0;
  if (dev < 0 || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  cus[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Runs `f` (a set-up step that is idempotent, e.g. hipFuncSetAttribute) until it has succeeded
// once on the current device.  Two threads may both run it the first time; neither skips it.
struct PerDeviceOnce {
  std::atomic<uint64_t> done{0};
  static_assert(kMaxDevices <= 64, "one bit per device");
  template <typename F>
  hipError_t run(F f) {
    const int dev = current_device();
    if (dev >= 0 && ((done.load(std::memory_order_acquire) >> dev) & 1)) return hipSuccess;
    const hipError_t e = f();
    if (e == hipSuccess && dev >= 0) done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
    return e;
  }
};

// Launchers implemented in the .hip files (host side).  Each returns a hipError_t.
hipError_t launch_router(const LayerView &L, int wdtype, const int32_t *chunk_layer, const float *x,
                         int64_t n_chunks, int k, float *scores, uint64_t *token_mask, float *preact,
                         hipStream_t s);   // preact: A^0 [n_tok][E] as well, or nullptr
hipError_t launch_chunk_union(const uint64_t *token_mask, int64_t n_chunks, int k, int E,
                              uint64_t *union_mask, int32_t *active_idx, int32_t *n_active,
                              int64_t *stats, hipStream_t s);

// CLS_L for L = 1 .. L_max over disjoint (row 0) and sliding (row 1) windows that stay inside
// sequences of seq_len tokens; inactive / windows / cls are [2][L_max].  L_max <= stats_max_window().
int stats_max_window();
hipError_t launch_cls_sweep(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int E, int L_max,
                            int64_t *inactive, int64_t *windows, double *cls, hipStream_t s);
// Eq. 4 / Eq. 5 forward values: losses[0] = L_al, losses[1] = L_cs for chunks of L tokens.
// workspace: losses_workspace_bytes() bytes, 8-byte aligned.
size_t losses_workspace_bytes();
hipError_t launch_router_losses(const float *a0, int64_t n_tok, int64_t seq_len, int E, int L, float alpha,
                                double *losses, void *workspace, hipStream_t s);
// LRU expert-cache simulation on HOST lists; returns a BLOCKFFN_* code.
int offload_sim(const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks, int E, int capacity,
                int64_t *loads_per_chunk, int64_t *totals);
// Reuse ratio of neighbouring tokens: num / cnt are [E + 1] (indexed by |S_i|), ratio is [1].
hipError_t launch_reuse_ratio(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int E, int64_t *num,
                              int64_t *cnt, double *ratio, hipStream_t s);
// Shape-generic FFN kernels.  active_idx == nullptr selects the dense path (every expert, no
// masking).  mid is fp32 [chunk][slot][token][neuron] with E slots per chunk.
hipError_t launch_up_generic(const LayerView &L, int wdtype, bool gated, const int32_t *chunk_layer, const float *x,
                             const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                             const int32_t *n_active, int64_t n_chunks, int k, float *mid, hipStream_t s);
hipError_t launch_down_generic(const LayerView &L, int wdtype, const int32_t *chunk_layer, const int32_t *active_idx,
                               const int32_t *n_active, int64_t n_chunks, int k, const float *mid, float *y,
                               hipStream_t s);

// Weight-streaming matrix-core kernels (bf16 weights, k <= 32, d % 512 == 0, d_e in {64,128,256}).
// The workspace layout differs from the generic kernels': mid is stored as bf16 hi/lo planes.
bool stream_supported(const LayerView &L, int wdtype, int k);
size_t stream_workspace_bytes(const LayerView &L, int64_t n_chunks, int k);
hipError_t launch_up_stream(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                            const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, void *ws, hipStream_t s);
hipError_t launch_down_stream(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                              const int32_t *n_active, int64_t n_chunks, int k, const void *ws, float *y,
                              hipStream_t s);

// A few chunks of up to 8 tokens as three launches instead of six (blockffn_forward_chunks): the
// router's per-expert kernel writes A^0 into the workspace, the up projection redoes the routing
// from it in every workgroup and writes the router's and the union's outputs, the down projection
// follows as usual.
bool router_few(const LayerView &L, int64_t n_chunks, int k);
hipError_t launch_router_preact_few(const LayerView &L, int wdtype, const int32_t *chunk_layer, const float *x,
                                    int64_t n_chunks, int k, float *preact, hipStream_t s);
float *few_preact_buffer(const LayerView &L, int64_t n_chunks, int k, void *ws);
hipError_t launch_up_few_routed(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                                int64_t n_chunks, int k, void *ws, float *scores, uint64_t *token_mask,
                                uint64_t *union_mask, int32_t *active_idx, int32_t *n_active, int64_t *stats,
                                hipStream_t s);
bool few_routed_supported(const LayerView &L, int wdtype, int64_t n_chunks, int k);

// Flat list of the active experts in groups of `group` consecutive slots: items[i] = chunk * E +
// first slot of the group, full groups first, then the chunks' shorter last groups, longest first;
// total[0] = its length (n_active == nullptr: every chunk has E slots), total[16 .. 19] = 0 (a
// 16-byte block of zeros for the kernels that follow).  items needs n_chunks * E entries, total 20.
hipError_t launch_worklist(const int32_t *n_active, int64_t n_chunks, int E, int group, int32_t *items,
                           int32_t *total, hipStream_t s);

// Matrix-core grouped contraction for large chunks (bf16 weights, 32 < k <= 512).
bool gemm_supported(const LayerView &L, int wdtype, int k, bool gated);
size_t gemm_workspace_bytes(const LayerView &L, int64_t n_chunks, int k);
hipError_t launch_up_gemm(const LayerView &L, bool gated, const int32_t *chunk_layer, const float *x,
                          const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                          const int32_t *n_active, int64_t n_chunks, int k, void *ws, hipStream_t s);
hipError_t launch_down_gemm(const LayerView &L, const int32_t *chunk_layer, const int32_t *active_idx,
                            const int32_t *n_active, int64_t n_chunks, int k, const void *ws, float *y,
                            hipStream_t s);

// Plain read stream over `bytes` bytes (measurement helper): variant 0..3 selects the tile per
// workgroup (1 MiB, 256 KiB, 256 KiB, 64 KiB) and the loads in flight per lane (8, 8, 16, 16).
hipError_t launch_stream_read(const void *buf, size_t bytes, int variant, uint32_t *sink, hipStream_t s);

}  // namespace blockffn
