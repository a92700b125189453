// C ABI of the library: argument checking and dispatch.  No kernel lives here.
#include <algorithm>
#include <cstdlib>
#include <mutex>

#include "common.hpp"

using namespace blockffn;

// Scratch of blockffn_sparse_ffn_static: one copy per device, held from the moment the library's
// code is loaded on that device until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress(); the device address it yields (static_scratch() below) is what the
// kernels, like any workspace pointer, are given.
static __device__ __align__(256) unsigned char scratch[BLOCKFFN_STATIC_SCRATCH_BYTES];

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Returns BLOCKFFN_OK and fills `v`, or the error code.
int check_layer(const blockffn_layer *l, LayerView &v) {
  if (l == nullptr) return BLOCKFFN_ERR_INVALID;
  if (l->d < 8 || l->d % 8 != 0 || l->d_e < 8 || l->d_e % 8 != 0) return BLOCKFFN_ERR_INVALID;
  if (l->n_experts < 1 || l->n_layers < 1) return BLOCKFFN_ERR_INVALID;
  if (!(l->rms_eps >= 0.0f)) return BLOCKFFN_ERR_INVALID;
  if (l->expert_kind != BLOCKFFN_EXPERT_SWISH && l->expert_kind != BLOCKFFN_EXPERT_GATED)
    return BLOCKFFN_ERR_INVALID;
  if (l->w_router == nullptr || l->w_up == nullptr || l->w_down == nullptr) return BLOCKFFN_ERR_INVALID;
  if ((l->expert_kind == BLOCKFFN_EXPERT_GATED) != (l->w_gate != nullptr)) return BLOCKFFN_ERR_INVALID;
  if (!aligned(l->w_router, 16) || !aligned(l->w_up, 16) || !aligned(l->w_down, 16) || !aligned(l->w_gate, 16))
    return BLOCKFFN_ERR_INVALID;
  if (!aligned(l->b_router, 4) || !aligned(l->g_rms, 4)) return BLOCKFFN_ERR_INVALID;
  if (l->wdtype != BLOCKFFN_F32 && l->wdtype != BLOCKFFN_BF16) return BLOCKFFN_ERR_UNSUPPORTED;
  if (l->n_experts > kMaxExperts || l->d_e > kMaxDe || l->d > kMaxD) return BLOCKFFN_ERR_UNSUPPORTED;
  v.d = l->d;
  v.E = l->n_experts;
  v.d_e = l->d_e;
  v.n_layers = l->n_layers;
  v.W = (l->n_experts + 63) / 64;
  v.eps = l->rms_eps;
  v.w_router = l->w_router;
  v.b_router = l->b_router;
  v.g_rms = l->g_rms;
  v.w_up = l->w_up;
  v.w_gate = l->w_gate;
  v.w_down = l->w_down;
  return BLOCKFFN_OK;
}

int check_chunks(int64_t n_chunks, int32_t k) {
  if (n_chunks < 0 || k < 1) return BLOCKFFN_ERR_INVALID;
  if (k > kMaxK) return BLOCKFFN_ERR_UNSUPPORTED;
  if (n_chunks * k > 0x7fffffffLL) return BLOCKFFN_ERR_UNSUPPORTED;   // tokens per call
  return BLOCKFFN_OK;
}

// BLOCKFFN_FORCE_GENERIC=1 in the environment keeps every shape on the shape-generic kernels
// (used to compare the two implementations on the same inputs).  Read once, when the first FFN
// call of the process arrives: later changes of the environment are not seen; a process that
// wants to switch at run time calls blockffn_force_generic().
std::atomic<int> g_force_generic{-1};   // -1: as the environment said; 0 / 1: set by blockffn_force_generic()
bool force_generic() {
  static const bool from_env = [] {
    const char *e = std::getenv("BLOCKFFN_FORCE_GENERIC");
    return e != nullptr && e[0] == '1';
  }();
  const int set = g_force_generic.load(std::memory_order_relaxed);
  return set < 0 ? from_env : set != 0;
}

// Device address of `scratch` on the current device; looked up once per device.
int static_scratch(void **out) {
  static std::mutex mu;
  static void *ptr[kMaxDevices];   // zero-initialised
  const int dev = current_device();
  if (dev < 0) return BLOCKFFN_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return BLOCKFFN_ERR_LAUNCH;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return BLOCKFFN_OK;
}
bool use_stream(const LayerView &v, int wdtype, int32_t k) { return !force_generic() && stream_supported(v, wdtype, k); }
bool use_gemm(const LayerView &v, int wdtype, int32_t k, bool gated) {
  return !force_generic() && gemm_supported(v, wdtype, k, gated);
}

size_t workspace_need(const LayerView &v, int wdtype, bool gated, int64_t n_chunks, int32_t k) {
  // generic kernels: mid[chunk][slot][token][neuron] fp32, slots sized for the worst case
  size_t bytes = (size_t)n_chunks * v.E * (size_t)k * v.d_e * sizeof(float);
  bytes = (bytes + 255) & ~(size_t)255;
  if (stream_supported(v, wdtype, k)) bytes = std::max(bytes, stream_workspace_bytes(v, n_chunks, k));
  if (gemm_supported(v, wdtype, k, gated)) bytes = std::max(bytes, gemm_workspace_bytes(v, n_chunks, k));
  return bytes;
}

enum { kPhaseUp = 1, kPhaseDown = 2, kStaticScratch = 4 };   // kStaticScratch: the workspace is the static array

int ffn_common(int phases, const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
               const float *scores, const uint64_t *token_mask, const int32_t *active_idx, const int32_t *n_active,
               int64_t n_chunks, int32_t k, float *y, void *workspace, size_t workspace_bytes, void *stream) {
  LayerView v;
  int rc = check_layer(layer, v);
  if (rc != BLOCKFFN_OK) return rc;
  rc = check_chunks(n_chunks, k);
  if (rc != BLOCKFFN_OK) return rc;
  // the dense path is selected by passing no list at all; a partial set of list arguments is an error
  const bool dense = active_idx == nullptr;
  if (dense ? (n_active != nullptr || token_mask != nullptr) : (n_active == nullptr)) return BLOCKFFN_ERR_INVALID;
  if (phases & kPhaseUp) {
    if (x == nullptr || scores == nullptr || (!dense && token_mask == nullptr)) return BLOCKFFN_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(scores, 4) || !aligned(token_mask, 8)) return BLOCKFFN_ERR_INVALID;
  }
  if (phases & kPhaseDown) {
    if (y == nullptr || !aligned(y, 16)) return BLOCKFFN_ERR_INVALID;
  }
  if (!aligned(active_idx, 4) || !aligned(n_active, 4) || !aligned(chunk_layer, 4)) return BLOCKFFN_ERR_INVALID;
  if (n_chunks == 0) return BLOCKFFN_OK;
  if (n_chunks * v.E > 0x7fffffffLL) return BLOCKFFN_ERR_UNSUPPORTED;   // (chunk, slot) pairs are indexed in 32 bits
  const bool gated = layer->expert_kind == BLOCKFFN_EXPERT_GATED;
  const size_t need = workspace_need(v, layer->wdtype, gated, n_chunks, k);
  if (phases & kStaticScratch) {
    if (need > (size_t)BLOCKFFN_STATIC_SCRATCH_BYTES) return BLOCKFFN_ERR_SCRATCH;
    rc = static_scratch(&workspace);
    if (rc != BLOCKFFN_OK) return rc;
    workspace_bytes = (size_t)BLOCKFFN_STATIC_SCRATCH_BYTES;
  }
  if (workspace == nullptr || !aligned(workspace, 256)) return BLOCKFFN_ERR_INVALID;
  if (workspace_bytes < need) return BLOCKFFN_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t err = hipSuccess;
  if (use_stream(v, layer->wdtype, k)) {
    if (phases & kPhaseUp)
      err = launch_up_stream(v, gated, chunk_layer, x, scores, token_mask, active_idx, n_active, n_chunks, k,
                             workspace, s);
    if (err == hipSuccess && (phases & kPhaseDown))
      err = launch_down_stream(v, chunk_layer, active_idx, n_active, n_chunks, k, workspace, y, s);
  } else if (use_gemm(v, layer->wdtype, k, gated)) {
    if (phases & kPhaseUp)
      err = launch_up_gemm(v, gated, chunk_layer, x, scores, token_mask, active_idx, n_active, n_chunks, k,
                           workspace, s);
    if (err == hipSuccess && (phases & kPhaseDown))
      err = launch_down_gemm(v, chunk_layer, active_idx, n_active, n_chunks, k, workspace, y, s);
  } else {
    float *mid = static_cast<float *>(workspace);
    if (phases & kPhaseUp)
      err = launch_up_generic(v, layer->wdtype, gated, chunk_layer, x, scores, token_mask, active_idx, n_active,
                              n_chunks, k, mid, s);
    if (err == hipSuccess && (phases & kPhaseDown))
      err = launch_down_generic(v, layer->wdtype, chunk_layer, active_idx, n_active, n_chunks, k, mid, y, s);
  }
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}


// a stream of n_tok token masks cut into sequences of seq_len tokens
int check_stream_of_masks(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int32_t n_experts) {
  if (n_experts < 1 || n_tok < 0 || seq_len < 1) return BLOCKFFN_ERR_INVALID;
  if (n_tok % seq_len != 0) return BLOCKFFN_ERR_INVALID;
  if (n_experts > kMaxExperts) return BLOCKFFN_ERR_UNSUPPORTED;
  if (token_mask == nullptr && n_tok > 0) return BLOCKFFN_ERR_INVALID;
  if (!aligned(token_mask, 8)) return BLOCKFFN_ERR_INVALID;
  return BLOCKFFN_OK;
}

}  // namespace

extern "C" {

int blockffn_router_preact(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x, int64_t n_chunks,
                           int32_t k, float *scores, uint64_t *token_mask, float *preact, void *stream) {
  LayerView v;
  int rc = check_layer(layer, v);
  if (rc != BLOCKFFN_OK) return rc;
  rc = check_chunks(n_chunks, k);
  if (rc != BLOCKFFN_OK) return rc;
  if (x == nullptr || scores == nullptr || token_mask == nullptr) return BLOCKFFN_ERR_INVALID;
  if (!aligned(x, 16) || !aligned(scores, 4) || !aligned(token_mask, 8) || !aligned(preact, 4))
    return BLOCKFFN_ERR_INVALID;
  if (n_chunks == 0) return BLOCKFFN_OK;
  hipError_t err = launch_router(v, layer->wdtype, chunk_layer, x, n_chunks, k, scores, token_mask, preact,
                                 static_cast<hipStream_t>(stream));
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

int blockffn_router(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x, int64_t n_chunks,
                    int32_t k, float *scores, uint64_t *token_mask, void *stream) {
  return blockffn_router_preact(layer, chunk_layer, x, n_chunks, k, scores, token_mask, nullptr, stream);
}

int blockffn_offload_sim(const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks, int32_t n_experts,
                         int32_t capacity, int64_t *loads_per_chunk, int64_t *totals) {
  if (n_experts < 1 || n_chunks < 0 || capacity < 0) return BLOCKFFN_ERR_INVALID;
  if (n_experts > kMaxExperts) return BLOCKFFN_ERR_UNSUPPORTED;
  if (totals == nullptr) return BLOCKFFN_ERR_INVALID;
  if (n_chunks > 0 && (active_idx == nullptr || n_active == nullptr)) return BLOCKFFN_ERR_INVALID;
  return offload_sim(active_idx, n_active, n_chunks, n_experts, capacity, loads_per_chunk, totals);
}

size_t blockffn_losses_workspace_bytes(void) { return losses_workspace_bytes(); }

int blockffn_router_losses(const float *preact, int64_t n_tok, int64_t seq_len, int32_t n_experts, int32_t chunk_len,
                           float alpha, double *losses, void *workspace, size_t workspace_bytes, void *stream) {
  if (n_experts < 1 || n_tok < 0 || seq_len < 1 || chunk_len < 1) return BLOCKFFN_ERR_INVALID;
  if (n_tok % seq_len != 0) return BLOCKFFN_ERR_INVALID;
  if (!(alpha >= 0.0f) || !(alpha <= 3.0e38f)) return BLOCKFFN_ERR_INVALID;   // NaN and inf fail too
  if (n_experts > kMaxExperts) return BLOCKFFN_ERR_UNSUPPORTED;
  if (preact == nullptr && n_tok > 0) return BLOCKFFN_ERR_INVALID;
  if (losses == nullptr || workspace == nullptr) return BLOCKFFN_ERR_INVALID;
  if (!aligned(preact, 4) || !aligned(losses, 8) || !aligned(workspace, 8)) return BLOCKFFN_ERR_INVALID;
  if (workspace_bytes < losses_workspace_bytes()) return BLOCKFFN_ERR_WORKSPACE;
  hipError_t err = launch_router_losses(preact, n_tok, seq_len, n_experts, chunk_len, alpha, losses, workspace,
                                        static_cast<hipStream_t>(stream));
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

int blockffn_chunk_union(const uint64_t *token_mask, int64_t n_chunks, int32_t k, int32_t n_experts,
                         uint64_t *union_mask, int32_t *active_idx, int32_t *n_active, int64_t *stats,
                         void *stream) {
  if (n_experts < 1) return BLOCKFFN_ERR_INVALID;
  int rc = check_chunks(n_chunks, k);
  if (rc != BLOCKFFN_OK) return rc;
  if (n_experts > kMaxExperts) return BLOCKFFN_ERR_UNSUPPORTED;
  if (token_mask == nullptr || union_mask == nullptr || active_idx == nullptr || n_active == nullptr)
    return BLOCKFFN_ERR_INVALID;
  if (!aligned(token_mask, 8) || !aligned(union_mask, 8) || !aligned(active_idx, 4) || !aligned(n_active, 4) ||
      !aligned(stats, 8))
    return BLOCKFFN_ERR_INVALID;
  if (n_chunks == 0) return BLOCKFFN_OK;
  hipError_t err = launch_chunk_union(token_mask, n_chunks, k, n_experts, union_mask, active_idx, n_active, stats,
                                      static_cast<hipStream_t>(stream));
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

int blockffn_cls_sweep(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int32_t n_experts, int32_t l_max,
                       int64_t *inactive, int64_t *windows, double *cls, void *stream) {
  int rc = check_stream_of_masks(token_mask, n_tok, seq_len, n_experts);
  if (rc != BLOCKFFN_OK) return rc;
  if (l_max < 1) return BLOCKFFN_ERR_INVALID;
  if (l_max > stats_max_window()) return BLOCKFFN_ERR_UNSUPPORTED;
  if (inactive == nullptr || windows == nullptr || cls == nullptr) return BLOCKFFN_ERR_INVALID;
  if (!aligned(inactive, 8) || !aligned(windows, 8) || !aligned(cls, 8)) return BLOCKFFN_ERR_INVALID;
  hipError_t err = launch_cls_sweep(token_mask, n_tok, seq_len, n_experts, l_max, inactive, windows, cls,
                                    static_cast<hipStream_t>(stream));
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

int blockffn_reuse_ratio(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int32_t n_experts, int64_t *num,
                         int64_t *cnt, double *ratio, void *stream) {
  int rc = check_stream_of_masks(token_mask, n_tok, seq_len, n_experts);
  if (rc != BLOCKFFN_OK) return rc;
  if (num == nullptr || cnt == nullptr || ratio == nullptr) return BLOCKFFN_ERR_INVALID;
  if (!aligned(num, 8) || !aligned(cnt, 8) || !aligned(ratio, 8)) return BLOCKFFN_ERR_INVALID;
  hipError_t err = launch_reuse_ratio(token_mask, n_tok, seq_len, n_experts, num, cnt, ratio,
                                      static_cast<hipStream_t>(stream));
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

int blockffn_sparse_ffn(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x, const float *scores,
                        const uint64_t *token_mask, const int32_t *active_idx, const int32_t *n_active,
                        int64_t n_chunks, int32_t k, float *y, void *workspace, size_t workspace_bytes,
                        void *stream) {
  if (active_idx == nullptr || n_active == nullptr || token_mask == nullptr) return BLOCKFFN_ERR_INVALID;
  return ffn_common(kPhaseUp | kPhaseDown, layer, chunk_layer, x, scores, token_mask, active_idx, n_active, n_chunks,
                    k, y, workspace, workspace_bytes, stream);
}

int blockffn_forward_chunks(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x, int64_t n_chunks,
                            int32_t k, float *scores, uint64_t *token_mask, uint64_t *union_mask, int32_t *active_idx,
                            int32_t *n_active, int64_t *stats, float *y, void *workspace, size_t workspace_bytes,
                            void *stream) {
  LayerView v;
  int rc = check_layer(layer, v);
  if (rc != BLOCKFFN_OK) return rc;
  rc = check_chunks(n_chunks, k);
  if (rc != BLOCKFFN_OK) return rc;
  const bool fused = n_chunks > 0 && !force_generic() && few_routed_supported(v, layer->wdtype, n_chunks, k);
  if (!fused) {   // the three stages one after the other; each checks its own arguments
    rc = blockffn_router(layer, chunk_layer, x, n_chunks, k, scores, token_mask, stream);
    if (rc != BLOCKFFN_OK) return rc;
    rc = blockffn_chunk_union(token_mask, n_chunks, k, layer->n_experts, union_mask, active_idx, n_active, stats, stream);
    if (rc != BLOCKFFN_OK) return rc;
    return blockffn_sparse_ffn(layer, chunk_layer, x, scores, token_mask, active_idx, n_active, n_chunks, k, y, workspace,
                               workspace_bytes, stream);
  }
  if (x == nullptr || scores == nullptr || token_mask == nullptr || union_mask == nullptr || active_idx == nullptr ||
      n_active == nullptr || y == nullptr)
    return BLOCKFFN_ERR_INVALID;
  if (!aligned(x, 16) || !aligned(scores, 4) || !aligned(token_mask, 8) || !aligned(union_mask, 8) ||
      !aligned(active_idx, 4) || !aligned(n_active, 4) || !aligned(stats, 8) || !aligned(y, 16) ||
      !aligned(chunk_layer, 4))
    return BLOCKFFN_ERR_INVALID;
  const bool gated = layer->expert_kind == BLOCKFFN_EXPERT_GATED;
  if (workspace == nullptr || !aligned(workspace, 256)) return BLOCKFFN_ERR_INVALID;
  if (workspace_bytes < workspace_need(v, layer->wdtype, gated, n_chunks, k)) return BLOCKFFN_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t err = launch_router_preact_few(v, layer->wdtype, chunk_layer, x, n_chunks, k,
                                            few_preact_buffer(v, n_chunks, k, workspace), s);
  if (err == hipSuccess)
    err = launch_up_few_routed(v, gated, chunk_layer, x, n_chunks, k, workspace, scores, token_mask, union_mask,
                               active_idx, n_active, stats, s);
  if (err == hipSuccess) err = launch_down_stream(v, chunk_layer, active_idx, n_active, n_chunks, k, workspace, y, s);
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

int blockffn_sparse_ffn_static(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                               const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                               const int32_t *n_active, int64_t n_chunks, int32_t k, float *y, void *stream) {
  if (active_idx == nullptr || n_active == nullptr || token_mask == nullptr) return BLOCKFFN_ERR_INVALID;
  return ffn_common(kPhaseUp | kPhaseDown | kStaticScratch, layer, chunk_layer, x, scores, token_mask, active_idx,
                    n_active, n_chunks, k, y, nullptr, 0, stream);
}

int blockffn_sparse_ffn_up(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                           const float *scores, const uint64_t *token_mask, const int32_t *active_idx,
                           const int32_t *n_active, int64_t n_chunks, int32_t k, void *workspace,
                           size_t workspace_bytes, void *stream) {
  return ffn_common(kPhaseUp, layer, chunk_layer, x, scores, token_mask, active_idx, n_active, n_chunks, k, nullptr,
                    workspace, workspace_bytes, stream);
}

int blockffn_sparse_ffn_down(const blockffn_layer *layer, const int32_t *chunk_layer, const int32_t *active_idx,
                             const int32_t *n_active, int64_t n_chunks, int32_t k, float *y, void *workspace,
                             size_t workspace_bytes, void *stream) {
  return ffn_common(kPhaseDown, layer, chunk_layer, nullptr, nullptr, nullptr, active_idx, n_active, n_chunks, k, y,
                    workspace, workspace_bytes, stream);
}

int blockffn_dense_ffn(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x, const float *scores,
                       int64_t n_chunks, int32_t k, float *y, void *workspace, size_t workspace_bytes,
                       void *stream) {
  return ffn_common(kPhaseUp | kPhaseDown, layer, chunk_layer, x, scores, nullptr, nullptr, nullptr, n_chunks, k, y,
                    workspace, workspace_bytes, stream);
}

int blockffn_force_generic(int mode) {
  if (mode < -1 || mode > 1) return BLOCKFFN_ERR_INVALID;
  g_force_generic.store(mode, std::memory_order_relaxed);
  return BLOCKFFN_OK;
}

int blockffn_stream_read(const void *buf, size_t bytes, int32_t variant, uint32_t *sink, void *stream) {
  if (buf == nullptr || sink == nullptr || !aligned(buf, 16) || !aligned(sink, 4)) return BLOCKFFN_ERR_INVALID;
  if (variant < 0 || variant > 7) return BLOCKFFN_ERR_INVALID;
  hipError_t err = launch_stream_read(buf, bytes, variant, sink, static_cast<hipStream_t>(stream));
  return err == hipSuccess ? BLOCKFFN_OK : BLOCKFFN_ERR_LAUNCH;
}

size_t blockffn_workspace_bytes(const blockffn_layer *layer, int64_t n_chunks, int32_t k) {
  LayerView v;
  if (check_layer(layer, v) != BLOCKFFN_OK) return 0;
  if (check_chunks(n_chunks, k) != BLOCKFFN_OK) return 0;
  return workspace_need(v, layer->wdtype, layer->expert_kind == BLOCKFFN_EXPERT_GATED, n_chunks, k);
}

const char *blockffn_strerror(int code) {
  switch (code) {
    case BLOCKFFN_OK: return "ok";
    case BLOCKFFN_ERR_INVALID: return "invalid argument";
    case BLOCKFFN_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case BLOCKFFN_ERR_WORKSPACE: return "workspace too small";
    case BLOCKFFN_ERR_LAUNCH: return "HIP launch error";
    case BLOCKFFN_ERR_SCRATCH: return "shape needs more than the static scratch holds (BLOCKFFN_STATIC_SCRATCH_BYTES)";
    default: return "unknown error code";
  }
}

int blockffn_version(void) { return 102; }

}  // extern "C"
