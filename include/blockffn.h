/*
 * blockffn.h - C ABI of the MI355X (gfx950) chunk-sparse expert FFN.
 *
 * The library runs the inference hot path of a BlockFFN layer for chunks of k consecutive
 * tokens (the n draft tokens verified together in speculative decoding, Sec. 3.3):
 *
 *   router        A^0 = W_router^T x (+ b),  A^1 = ReLU(A^0),  A = RMSNorm(A^1)        (Eq. 3)
 *   chunk union   Union(x): experts activated by at least one token of the chunk        (Sec. 3.3)
 *   sparse FFN    FFN(x_t) = sum_{i in Union} [A_i(x_t) > 0] A_i(x_t) E_i(x_t)           (Eq. 1, Sec. 3.3)
 *   dense FFN     FFN(x_t) = sum_{i=1..N_e} A_i(x_t) E_i(x_t), every expert evaluated   (Eq. 1)
 *
 *   E_i(x) = W_down^(i)T Swish(W_up^(i)T x)                         (Eq. 2, the paper's expert)
 *   E_i(x) = W_down^(i)T [Swish(W_gate^(i)T x) . W_up^(i)T x]       (gated variant, Table 1)
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * - Every pointer is a DEVICE pointer owned by the caller, except `layer` (host struct, read
 *   during the call only), `stream`, and the arguments of blockffn_offload_sim (host memory).  The library never allocates, frees or keeps them.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *   work on it: no synchronisation, no host read-back.  Outputs of one call are valid inputs
 *   of the next call on the same stream.
 * - Chunk c is the token range [c*k, (c+1)*k); token t of the batch is row t of x / scores / y.
 * - W = ceil(N_e / 64) mask words per token or chunk; expert i is bit (i % 64) of word (i / 64);
 *   bits at or above N_e are zero.
 * - Weights hold `n_layers` layers stacked in their leading dimension.  `chunk_layer`
 *   (device int32 [n_chunks], or NULL = layer 0 for all) says which layer's weights chunk c
 *   reads; values are clamped into [0, n_layers).  This is how a batch of chunks walks through
 *   distinct weight sets in one launch.
 * - Every matrix is stored one row per OUTPUT feature with the contraction index contiguous
 *   (the transposes written in Eq. 2-3): w_router [L][E][d], w_up / w_gate [L][E][d_e][d],
 *   w_down [L][E][d][d_e].  dtype per `wdtype`: fp32 or bf16.  Weight pointers must be 16-byte
 *   aligned.  Activations (x, scores, y) are fp32; accumulation is fp32.
 * - Return value: BLOCKFFN_OK or a negative code; nothing is enqueued when a code is returned
 *   by argument checking.  No exceptions, no exit, no output to stdout/stderr.
 * - Inputs are assumed finite.  A NaN pre-activation counts as inactive.
 *
 * - An entry of active_idx below n_active that lies outside [0, N_e) is an empty slot: it
 *   contributes nothing to y, on every kernel path (n_active itself is clamped into [0, N_e]).
 *
 * Limits: 1 <= N_e <= 256, 1 <= k <= 512, d % 8 == 0, d_e % 8 == 0, d_e <= 1024, d <= 16384,
 * n_chunks * k < 2^31 and n_chunks * N_e < 2^31 per call (beyond: BLOCKFFN_ERR_UNSUPPORTED).
 */
#ifndef BLOCKFFN_H
#define BLOCKFFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { BLOCKFFN_F32 = 0, BLOCKFFN_BF16 = 1 };
enum { BLOCKFFN_EXPERT_SWISH = 0, /* Eq. 2 */
       BLOCKFFN_EXPERT_GATED = 1  /* Table 1, gated row */ };
enum {
  BLOCKFFN_OK = 0,
  BLOCKFFN_ERR_INVALID = -1,     /* NULL pointer, size < 1, d or d_e not a multiple of 8, misaligned weights */
  BLOCKFFN_ERR_UNSUPPORTED = -2, /* shape or dtype outside the limits above */
  BLOCKFFN_ERR_WORKSPACE = -3,   /* workspace smaller than blockffn_workspace_bytes() */
  BLOCKFFN_ERR_LAUNCH = -4,      /* the HIP runtime refused a launch */
  BLOCKFFN_ERR_SCRATCH = -5      /* blockffn_sparse_ffn_static: the shape needs more than BLOCKFFN_STATIC_SCRATCH_BYTES */
};

/* Size of the per-device static scratch array behind blockffn_sparse_ffn_static. */
#define BLOCKFFN_STATIC_SCRATCH_BYTES (128u << 20)

typedef struct blockffn_layer {
  int32_t d;           /* d_h: hidden size */
  int32_t n_experts;   /* N_e */
  int32_t d_e;         /* expert intermediate size */
  int32_t wdtype;      /* BLOCKFFN_F32 | BLOCKFFN_BF16, for all four weight tensors */
  int32_t expert_kind; /* BLOCKFFN_EXPERT_SWISH | BLOCKFFN_EXPERT_GATED */
  int32_t n_layers;    /* L >= 1 layers stacked in each tensor below */
  float rms_eps;       /* RMSNorm epsilon (inside the root), >= 0 */
  int32_t reserved;    /* 0 */
  const void *w_router;  /* [L][E][d] */
  const float *b_router; /* [L][E] fp32, or NULL (the paper's router has no bias) */
  const float *g_rms;    /* [L][E] fp32 RMSNorm gain, or NULL (all ones) */
  const void *w_up;      /* [L][E][d_e][d] */
  const void *w_gate;    /* [L][E][d_e][d]; NULL iff expert_kind == SWISH */
  const void *w_down;    /* [L][E][d][d_e] */
} blockffn_layer;

/* Eq. 3.  scores [n_chunks*k][E] fp32 (A, exact zeros where inactive); token_mask
 * [n_chunks*k][W] uint64, bit set iff A^0 > 0 (strictly; follows the ReLU pattern A^1, so a
 * zero gain leaves the bit set).  RMSNorm: mean of squares over all N_e entries, eps inside
 * the root, then the gain.  An all-inactive token gets an all-zero row. */
int blockffn_router(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                    int64_t n_chunks, int32_t k, float *scores, uint64_t *token_mask,
                    void *stream);

/* Sec. 3.3 Union(x) and Sec. 2.1 TLS / CLS counts.  union_mask [n_chunks][W] = OR of the
 * chunk's token masks; active_idx [n_chunks][E] = set bits in ascending order, tail filled
 * with -1; n_active [n_chunks] = popcount.  stats (int64[2], or NULL) is ADDED to:
 * stats[0] += inactive (token, expert) pairs, stats[1] += inactive (chunk, expert) pairs, so
 * TLS = stats[0] / (tokens * E) and CLS_k = stats[1] / (chunks * E). */
int blockffn_chunk_union(const uint64_t *token_mask, int64_t n_chunks, int32_t k,
                         int32_t n_experts, uint64_t *union_mask, int32_t *active_idx,
                         int32_t *n_active, int64_t *stats, void *stream);

/* Sec. 3.3: streams only the weights of the experts in active_idx[c][0 .. n_active[c]) once
 * per chunk, applies them to all k tokens, and drops the terms of tokens whose mask bit for
 * that expert is clear.  Overwrites y [n_chunks*k][d] completely (zeros for an empty union).
 * scores / token_mask / active_idx / n_active as produced by the two calls above.
 * workspace: at least blockffn_workspace_bytes() bytes, 256-byte aligned; contents undefined
 * before and after. */
int blockffn_sparse_ffn(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                        const float *scores, const uint64_t *token_mask,
                        const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks,
                        int32_t k, float *y, void *workspace, size_t workspace_bytes,
                        void *stream);

/* Eq. 1 with no sparsity used (the paper's sparsity-ablation setting, App. H): all N_e experts
 * are streamed for every chunk and weighted by `scores` with no masking.  Same kernels and
 * workspace as the sparse path. */
int blockffn_dense_ffn(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                       const float *scores, int64_t n_chunks, int32_t k, float *y,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Router, chunk union and chunk-sparse FFN in one call (Eq. 3 and Sec. 3.3, the whole path of a
 * layer): exactly what blockffn_router, blockffn_chunk_union and blockffn_sparse_ffn compute when
 * called in that order on one stream with these arguments - every output (scores, token_mask,
 * union_mask, active_idx, n_active, stats added to, y) has the same bits.  For a handful of chunks
 * of up to 8 tokens (one chunk walking through a model's layers, where the time goes to launches
 * and their round trips to memory) the layer is three launches instead of six; every other shape
 * runs the three stages as they are.  Arguments, workspace and error codes as for those calls. */
int blockffn_forward_chunks(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                            int64_t n_chunks, int32_t k, float *scores, uint64_t *token_mask,
                            uint64_t *union_mask, int32_t *active_idx, int32_t *n_active,
                            int64_t *stats, float *y, void *workspace, size_t workspace_bytes,
                            void *stream);

/* blockffn_sparse_ffn for callers that cannot allocate device memory and so have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as blockffn_sparse_ffn; the workspace is a static device array of
 * BLOCKFFN_STATIC_SCRATCH_BYTES (128 MiB) that every GPU the library runs on holds until the
 * process ends.  The call allocates and frees nothing.  A shape whose blockffn_workspace_bytes()
 * exceeds that size returns BLOCKFFN_ERR_SCRATCH and enqueues nothing (at N_e = 64, d_e = 256,
 * d = 2048 the array holds 200 chunks of 8 tokens, 56 chunks of 32 tokens, or one 512-token
 * prefill chunk).  All calls on one GPU share the array: calls
 * that overlap in time on one GPU (two streams, two threads) race; calls on one stream, and calls
 * on different GPUs, do not.  Nothing in the array needs clearing between calls: every word a
 * kernel reads is written earlier in the same call. */
int blockffn_sparse_ffn_static(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                               const float *scores, const uint64_t *token_mask,
                               const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks,
                               int32_t k, float *y, void *stream);

/* The two halves of blockffn_sparse_ffn as separate enqueues (Sec. 3.3 describes the up and
 * the down projection as two sparse matrix products with the intermediate `mid` between
 * them).  `up` fills the workspace with mid = mask . A . Swish-or-gated(W_up^T x) for the
 * experts of the union; `down` reduces it through W_down into y.  Calling up then down with
 * the same arguments on one stream equals blockffn_sparse_ffn.  active_idx == NULL (with
 * token_mask and n_active NULL too) selects the dense path in both. */
int blockffn_sparse_ffn_up(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                           const float *scores, const uint64_t *token_mask,
                           const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks,
                           int32_t k, void *workspace, size_t workspace_bytes, void *stream);
int blockffn_sparse_ffn_down(const blockffn_layer *layer, const int32_t *chunk_layer,
                             const int32_t *active_idx, const int32_t *n_active,
                             int64_t n_chunks, int32_t k, float *y, void *workspace,
                             size_t workspace_bytes, void *stream);

/* blockffn_router that also writes the pre-activations A^0 = W_router^T x (+ b) of Eq. 3 to
 * preact [n_chunks*k][E] fp32 (NULL: not written).  scores and token_mask exactly as
 * blockffn_router writes them; preact holds the values whose sign decided the mask bits. */
int blockffn_router_preact(const blockffn_layer *layer, const int32_t *chunk_layer, const float *x,
                           int64_t n_chunks, int32_t k, float *scores, uint64_t *token_mask,
                           float *preact, void *stream);

/* Forward values of the CLS-aware training objectives (Sec. 3.2) on the pre-activations of a
 * stream of n_tok tokens cut into sequences of seq_len tokens (n_tok a multiple of seq_len),
 * evaluated in fp64:
 *   losses[0] = L_al, Eq. 4: binary cross entropy with input sigmoid(alpha * A^0[t, i]) and
 *     target sigmoid(alpha * A^0[t+1, i]) (the sequence shifted left by one token), averaged
 *     over all (t, i) whose token has a successor in its sequence; the logarithms are the exact
 *     log-sigmoids (no clamping).  0 when seq_len = 1.
 *   losses[1] = L_cs, Eq. 5, for chunks of chunk_len consecutive tokens: p_ik = the L1
 *     normalisation over experts of ReLU(A^0) for token k (all zero for a token with no active
 *     expert), P^i_act = 1 - exp(sum_k ln(1 - p_ik)), averaged over experts and over the
 *     disjoint chunks [j*chunk_len, (j+1)*chunk_len) of every sequence (a shorter tail is left
 *     out).  0 when there is no chunk.
 * alpha >= 0 finite.  workspace: blockffn_losses_workspace_bytes() bytes, 8-byte aligned,
 * contents undefined on entry and on return.  The result does not depend on scheduling: partial
 * sums are combined in a fixed order. */
size_t blockffn_losses_workspace_bytes(void);
int blockffn_router_losses(const float *preact, int64_t n_tok, int64_t seq_len, int32_t n_experts,
                           int32_t chunk_len, float alpha, double *losses, void *workspace,
                           size_t workspace_bytes, void *stream);

/* Expert-cache simulation for offloading (Sec. 1 and Sec. 4.1.2 name the saving of expert IO as
 * the second use of chunk-level sparsity and of a high reuse ratio; no mechanism is given, this
 * is the textbook one).  HOST code on HOST pointers, nothing is launched: active_idx
 * [n_chunks][N_e] and n_active [n_chunks] are one layer's union lists copied back from
 * blockffn_chunk_union.  A cache of `capacity` experts with least-recently-used replacement,
 * empty at the start, is driven by the lists: the experts of a chunk are touched in list order;
 * touching a resident expert is a hit and makes it the most recently used; touching any other
 * is a load, which first evicts the least recently used resident expert when the cache is full.
 *   loads_per_chunk [n_chunks] int64, or NULL   loads caused by each chunk
 *   totals [3] int64                            touches, loads, evictions
 * Bytes moved = loads * bytes of one expert.  An entry of a list outside [0, N_e), or an
 * n_active outside [0, N_e], returns BLOCKFFN_ERR_INVALID (outputs then undefined). */
int blockffn_offload_sim(const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks,
                         int32_t n_experts, int32_t capacity, int64_t *loads_per_chunk,
                         int64_t *totals);

/* Sec. 2.1, the curve of Fig. 1(a): CLS_L for every window length L = 1 .. l_max at once, from
 * the token masks blockffn_router wrote.  The n_tok tokens are n_tok / seq_len sequences of
 * seq_len tokens (n_tok must be a multiple of seq_len); no window crosses a sequence boundary.
 * Row 0 of each output is for disjoint windows [j*L, (j+1)*L) (floor(seq_len / L) per sequence,
 * a shorter tail is left out), row 1 for sliding windows (every start s with s + L <= seq_len).
 *   inactive [2][l_max] int64   sum over the windows of (N_e - experts active in the window)
 *   windows  [2][l_max] int64   number of windows
 *   cls      [2][l_max] double  inactive / (windows * N_e); 0 where there is no window
 * All three are overwritten.  CLS_1 is TLS; disjoint L = k gives the CLS_k of
 * blockffn_chunk_union.  1 <= l_max <= 64 (larger: BLOCKFFN_ERR_UNSUPPORTED). */
int blockffn_cls_sweep(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int32_t n_experts,
                       int32_t l_max, int64_t *inactive, int64_t *windows, double *cls, void *stream);

/* Sec. 4.1.2 (Table 4), expert selection stability: with S_i the experts token i activates,
 * the mean of |S_i & S_{i+1}| / |S_i| over neighbouring tokens of the same sequence.  A pair
 * whose S_i is empty has no ratio and is left out of the mean; all pairs of all sequences are
 * pooled.  Outputs (overwritten), indexed by c = |S_i|:
 *   num [N_e + 1] int64   sum of |S_i & S_{i+1}| over the pairs with |S_i| = c
 *   cnt [N_e + 1] int64   number of such pairs (entry 0 stays 0)
 *   ratio [1] double      (sum_c num[c] / c) / sum_c cnt[c], added in ascending c; 0 with no pair
 * The integer outputs are exact; ratio is their fp64 evaluation. */
int blockffn_reuse_ratio(const uint64_t *token_mask, int64_t n_tok, int64_t seq_len, int32_t n_experts,
                         int64_t *num, int64_t *cnt, double *ratio, void *stream);

/* Kernel selection for cross-checks (no step of the layer): the FFN entry points pick the
 * weight-streaming or the matrix-core kernels where the shape allows and the shape-generic fp32
 * ALU kernels otherwise.  mode 1 keeps every later call of the process on the shape-generic
 * kernels, mode 0 on the automatic choice, mode -1 (the initial state) follows the environment
 * variable BLOCKFFN_FORCE_GENERIC (=1: generic), which is read once per process.  Workspace sizes
 * do not depend on it.  Returns BLOCKFFN_ERR_INVALID for any other mode. */
int blockffn_force_generic(int mode);

/* Measurement helper (no step of the layer): reads `bytes` bytes (rounded down to 16) at buf with
 * 128-bit loads and nothing else, so that a benchmark can time what a pure read stream reaches
 * on this device and report the weight-streaming kernels against that measured ceiling as well
 * as against the nominal HBM peak.  buf: device memory, 16-byte aligned.  variant 0..7: variant % 4
 * selects the tile a workgroup reads (1 MiB, 256 KiB, 256 KiB, 64 KiB) and the loads in flight per
 * lane (8, 8, 16, 16); 0..3 use plain loads, 4..7 non-temporal loads (what the weight streams
 * use).  sink: 4 writable device bytes (written to in practice never). */
int blockffn_stream_read(const void *buf, size_t bytes, int32_t variant, uint32_t *sink, void *stream);

/* Bytes of workspace the two FFN entry points need for this shape (0 on invalid arguments). */
size_t blockffn_workspace_bytes(const blockffn_layer *layer, int64_t n_chunks, int32_t k);

/* Static description of a return code. */
const char *blockffn_strerror(int code);

/* ABI version of this header (major * 100 + minor). */
int blockffn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BLOCKFFN_H */
