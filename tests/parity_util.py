"""Helpers shared by the GPU parity tests: run the oracle and the HIP path on the same
seeded inputs and compare them to the stated bars.

Bars: masks, union words, active lists, counts and TLS/CLS statistics bit-exact; router
scores and FFN outputs per token row  max_j |v - ref| <= rtol * rms_j(ref)  with
rtol = 1e-5 for fp32 weights and 2e-2 for bf16 weights (the oracle widens the same stored
bf16 weights exactly, so the HIP path is in practice far inside the bf16 bar; the tests
also hold it to `tight`, a bound derived from fp32 accumulation).
"""

from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2507_08771_amd import binding as B
from paper_2507_08771_amd import workloads as wl

RTOL = {"f32": 1e-5, "bf16": 2e-2}
# fp32 accumulation with activations carried as two bf16 halves (16 significant bits) on the
# matrix-core path: error is a few 1e-6 of the row rms; 1e-4 leaves a wide margin.
TIGHT = {"f32": 1e-5, "bf16": 1e-4}
# Large chunks (k > 32) run as a bf16 x bf16 grouped contraction on the matrix cores.  x enters as
# two bf16 halves (16 significant bits, as on the streaming path); mid is rounded to bf16 once
# (relative error at most 2^-9 per element, about 1.1e-3 rms).  That one rounding leaves 1.6e-3 of
# the row's norm at the median and up to 2.7e-3 on rows made of a single 64-neuron expert (measured,
# and reproduced by rounding the oracle's own mid to bf16 on the CPU); the largest of a row's elements
# sits at 4 to 5 sigma of that.  Held: the stated 2e-2 on the row maximum, 1.5e-2 on the pinned
# few-term rows, 3.5e-3 on every row's L2-relative error.
GEMM_BAR = 2e-2
GEMM_FEW_TERMS_BAR = 1.5e-2
GEMM_L2_BAR = 3.5e-3


def oracle_layer(layers, l, eps=1e-6, use_gain=True, use_bias=True):
    g = lambda n: None if layers.get(n) is None else wl.to_numpy(layers[n][l])
    return oracle.Layer(g("w_router"), g("w_up"), g("w_down"), w_gate=g("w_gate"),
                        b_router=g("b_router") if use_bias else None,
                        g_rms=g("g_rms") if use_gain else None, eps=eps)


def run_oracle(layers, x, k, chunk_layer=None, eps=1e-6, dense=False, use_gain=True, use_bias=True, chunks=None):
    """Oracle outputs for all chunks (or the listed ones), honouring the per-chunk layer."""
    xn = wl.to_numpy(x)
    T, d = xn.shape
    C = T // k
    E = layers["w_router"].shape[1]
    W = (E + 63) // 64
    cl = np.zeros(C, np.int64) if chunk_layer is None else wl.to_numpy(chunk_layer).astype(np.int64)
    sel = np.arange(C) if chunks is None else np.asarray(chunks)
    out = dict(scores=np.zeros((T, E), np.float32), token_mask=np.zeros((T, W), np.uint64),
               union_mask=np.zeros((C, W), np.uint64), active_idx=np.full((C, E), -1, np.int32),
               n_active=np.zeros(C, np.int32), stats=np.zeros(2, np.int64), y=np.zeros((T, d), np.float64),
               y_dense=np.zeros((T, d), np.float64) if dense else None)
    for l in np.unique(cl[sel]):
        L = oracle_layer(layers, int(l), eps, use_gain, use_bias)
        cs = sel[cl[sel] == l]
        tok = (cs[:, None] * k + np.arange(k)[None, :]).reshape(-1)
        xs = xn[tok]
        r = oracle.forward(L, xs, k)
        out["scores"][tok] = r["scores"]
        out["token_mask"][tok] = r["token_mask"]
        out["union_mask"][cs] = r["union_mask"]
        out["active_idx"][cs] = r["active_idx"]
        out["n_active"][cs] = r["n_active"]
        out["stats"] += r["stats"]
        out["y"][tok] = r["y"]
        if dense:
            out["y_dense"][tok] = oracle.dense_ffn(L, xs, r["scores"])
    return out


def to_device(layers, device="cuda"):
    return {n: (None if t is None else t.to(device)) for n, t in layers.items()}


def run_gpu(layers_dev, x_dev, k, chunk_layer=None, eps=1e-6, dense=False, use_gain=True, use_bias=True):
    L = B.Layer(layers_dev["w_router"], layers_dev["w_up"], layers_dev["w_down"], layers_dev.get("w_gate"),
                layers_dev["b_router"] if use_bias else None, layers_dev["g_rms"] if use_gain else None, eps)
    C = x_dev.shape[0] // k
    buf = B.Buffers(L, C, k)
    cl = None if chunk_layer is None else chunk_layer.to(x_dev.device).to(torch.int32).contiguous()
    B.forward_chunks(L, x_dev, buf, cl)
    out = dict(scores=buf.scores, token_mask=buf.token_mask, union_mask=buf.union_mask, active_idx=buf.active_idx,
               n_active=buf.n_active, stats=buf.stats, y=buf.y)
    if dense:
        yd = torch.empty_like(buf.y)
        B.blockffn_dense_ffn(L, x_dev, buf.scores, C, k, yd, buf.workspace, cl)
        out["y_dense"] = yd
    torch.cuda.synchronize()
    res = {}
    for n, t in out.items():
        a = t.cpu().numpy()
        if n in ("token_mask", "union_mask"):
            a = a.view(np.uint64)
        res[n] = a
    res["_layer"], res["_buf"] = L, buf
    return res


def row_rel_err(v, ref):
    """max_j |v - ref| / rms_j(ref) per row (rows with a zero reference must match exactly)."""
    ref = ref.astype(np.float64)
    err = np.abs(v.astype(np.float64) - ref).max(axis=1)
    rms = np.sqrt((ref * ref).mean(axis=1))
    zero = rms == 0
    assert np.all(err[zero] == 0), "non-zero output where the reference row is exactly zero"
    return np.where(zero, 0.0, err / np.where(zero, 1.0, rms))


def preact_roundings(d):
    """Number of fp32 roundings on the longest chain of additions behind one pre-activation A^0 in
    the router kernels (products are exact: fused multiply-adds on the vector ALUs, bf16 x bf16
    on the matrix cores).
      matrix cores: a wave accumulates every fourth pair of K-steps of 32 elements,
        2 ceil(ceil(d / 64) / 4) accumulator updates, each taking in a 32-term dot product (a tree
        of depth 5); then the h / m / l sums (2), the four waves pairwise (2), the bias (1);
      vector ALUs: chains of 8 fused multiply-adds per 2048 columns, a 6-level reduction across
        the wave, one addition per 2048-column block, the four waves (2), the bias (1).
    Each rounding moves the sum by at most 2^-24 of its magnitude, which is bounded by
    mag = |b| + sum_j |x_j| |W_ij|; so |A^0 - exact| <= preact_roundings(d) * 2^-24 * mag to first
    order, whatever the order of the additions inside those chains."""
    pairs = -(-d // 64)
    mfma = 2 * -(-pairs // 4) + 5 + 2 + 2 + 1
    blocks = -(-d // 2048)
    valu = 8 * blocks + 6 + blocks + 2 + 1
    return max(mfma, valu)


def preact_error_allowed(layers, l, xs, use_bias=True):
    """Per (token, expert) bound on |A^0_fp32 - A^0_exact| for layer l: see preact_roundings()."""
    mag = np.abs(xs).astype(np.float64) @ np.abs(layers["w_router"][int(l)].double().numpy()).T
    if use_bias and layers.get("b_router") is not None:
        mag = mag + np.abs(layers["b_router"][int(l)].double().numpy())[None, :]
    return preact_roundings(xs.shape[1]) * 2.0 ** -24 * mag


def score_error_from_preact(a0, delta, ref_scores, eps, gmax):
    """Per-token bound on max_i |score_i - reference| given the bound `delta` on the pre-activations.
    score_i = g_i a1_i / s with s = sqrt(mean_j a1_j^2 + eps).  To first order
      |d score_i| <= g_i (|d a1_i| / s + a1_i |d s| / s^2),   |d s| = |sum_j a1_j d a1_j| / (E s) <= dmax
    (Cauchy-Schwarz: sum_j a1_j <= sqrt(E) sqrt(sum_j a1_j^2) <= E s), hence
      |d score_i| <= gmax dmax / s * (1 + max_i a1_i / s).
    A token whose only active expert is barely active has s close to sqrt(eps), which is what makes
    the plain "1e-5 of the row's rms" bar unreachable for it in any fp32 order of additions.  That
    plain bar (for the arithmetic after A^0: the sum of squares, the root, the division) is added."""
    a1 = np.maximum(a0, 0.0)
    s = np.sqrt((a1 * a1).mean(axis=1) + eps)
    dmax = delta.max(axis=1)
    rms = np.sqrt((ref_scores.astype(np.float64) ** 2).mean(axis=1))
    return 1e-5 * np.maximum(rms, 1e-30) + gmax * dmax / s * (1.0 + a1.max(axis=1) / s)


def score_error_allowed(layers, x, k, chunk_layer, ref_scores, eps=1e-6, use_gain=True, use_bias=True):
    """Per-token bound on |score - reference| for a whole batch (chunks may use different layers)."""
    xn = wl.to_numpy(x)
    T = xn.shape[0]
    cl = np.zeros(T // k, np.int64) if chunk_layer is None else wl.to_numpy(chunk_layer).astype(np.int64)
    allowed = np.zeros(T)
    for l in np.unique(cl):
        tok = np.nonzero(np.repeat(cl == l, k))[0]
        _, _, a0 = oracle.router(oracle_layer(layers, int(l), eps=eps, use_gain=use_gain, use_bias=use_bias),
                                 xn[tok], return_a0=True)
        delta = preact_error_allowed(layers, l, xn[tok], use_bias)
        gmax = float(layers["g_rms"][int(l)].max()) if use_gain and layers.get("g_rms") is not None else 1.0
        allowed[tok] = score_error_from_preact(a0, delta, ref_scores[tok], eps, gmax)
    return allowed


def assert_scores_within_allowance(gpu_scores, ref_scores, allowed, what=""):
    """Scores against the derived bound; prints how much of the allowance the worst row uses."""
    err = np.abs(gpu_scores.astype(np.float64) - ref_scores).max(axis=1)
    used = float((err / allowed).max(initial=0.0))
    print("score error: worst row uses %.3f of its allowance %s" % (used, what), flush=True)
    assert used <= 1.0, "router score beyond the derived fp32 bound (%.3f of it) %s" % (used, what)
    return used


def oracle_ffn_on_gpu_routing(layers, x, k, chunk_layer, gpu, eps=1e-6, use_gain=True, use_bias=True):
    """The oracle's chunk-sparse FFN driven by the scores, masks and lists the HIP path produced:
    judges the FFN kernels on every row, independently of the router's rounding."""
    xn = wl.to_numpy(x)
    T, d = xn.shape
    C = T // k
    cl = np.zeros(C, np.int64) if chunk_layer is None else wl.to_numpy(chunk_layer).astype(np.int64)
    y = np.zeros((T, d), np.float64)
    for l in np.unique(cl):
        L = oracle_layer(layers, int(l), eps, use_gain, use_bias)
        cs = np.nonzero(cl == l)[0]
        tok = (cs[:, None] * k + np.arange(k)[None, :]).reshape(-1)
        y[tok] = oracle.sparse_ffn(L, xn[tok], gpu["scores"][tok], gpu["token_mask"][tok], gpu["active_idx"][cs],
                                   gpu["n_active"][cs], k)
    return y


def assert_integers_equal(gpu, ref, chunks=None, k=None):
    if chunks is None:
        for n in ("token_mask", "union_mask", "active_idx", "n_active", "stats"):
            np.testing.assert_array_equal(gpu[n], ref[n], err_msg=n)
    else:
        cs = np.asarray(chunks)
        tok = (cs[:, None] * k + np.arange(k)[None, :]).reshape(-1)
        np.testing.assert_array_equal(gpu["token_mask"][tok], ref["token_mask"][tok])
        for n in ("union_mask", "active_idx", "n_active"):
            np.testing.assert_array_equal(gpu[n][cs], ref[n][cs], err_msg=n)


def assert_floats_close(gpu, ref, wdtype, rows=None, dense=False, tight=True, bar=None, l2_bar=None):
    sl = slice(None) if rows is None else rows
    if bar is None:
        bar = TIGHT[wdtype] if tight else RTOL[wdtype]
    e_scores = row_rel_err(gpu["scores"][sl], ref["scores"][sl]).max(initial=0.0)
    assert e_scores <= 1e-5, "router scores off by %.3g" % e_scores
    # zero pattern of the scores is part of the integer bar
    np.testing.assert_array_equal(gpu["scores"][sl] == 0, ref["scores"][sl] == 0)
    e_y = row_rel_err(gpu["y"][sl], ref["y"][sl]).max(initial=0.0)
    assert e_y <= bar, "sparse FFN output off by %.3g (bar %.1g)" % (e_y, bar)
    if l2_bar is not None:
        num = ((gpu["y"][sl] - ref["y"][sl]) ** 2).sum(axis=1)
        den = (ref["y"][sl] ** 2).sum(axis=1)
        l2 = np.sqrt(num[den > 0] / den[den > 0]).max(initial=0.0)
        assert l2 <= l2_bar, "sparse FFN output L2-relative error %.3g (bar %.1g)" % (l2, l2_bar)
    e_d = 0.0
    if dense:
        e_d = row_rel_err(gpu["y_dense"][sl], ref["y_dense"][sl]).max(initial=0.0)
        assert e_d <= bar, "dense FFN output off by %.3g (bar %.1g)" % (e_d, bar)
    return dict(scores=e_scores, y=e_y, y_dense=e_d)
