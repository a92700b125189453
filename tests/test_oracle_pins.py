"""Pins of the CPU oracle against what the paper's definitions and plain mathematics fix.

None of these tests touches the HIP path.  Each targets a mistake the oracle could
plausibly hold: a transposed operand, a dropped bias / gain / eps, RMSNorm averaged over
the wrong set, Swish on the wrong branch of the gated expert, a wrong mask bit or list
order, an expert skipped or double counted.
"""

import itertools
import json
import math
import os

import numpy as np
import pytest
import torch
from scipy.special import expit

HERE = os.path.dirname(os.path.abspath(__file__))


def bf16_bits(a):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_round(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def mask_to_sets(mask, E):
    out = []
    for row in mask:
        s = set()
        for i in range(E):
            if (int(row[i // 64]) >> (i % 64)) & 1:
                s.add(i)
        out.append(s)
    return out


def sets_to_mask(sets, E):
    W = (E + 63) // 64
    m = np.zeros((len(sets), W), np.uint64)
    for t, s in enumerate(sets):
        for i in s:
            m[t, i // 64] |= np.uint64(1) << np.uint64(i % 64)
    return m


def dummy_ffn_weights(E, d, d_e, rng):
    return (rng.standard_normal((E, d_e, d)).astype(np.float32),
            rng.standard_normal((E, d, d_e)).astype(np.float32))


# ----------------------------------------------------------------------------- router (Eq. 3)

def test_router_hand_worked_golden(oracle):
    with open(os.path.join(HERE, "golden", "router_worked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        wr = np.array(c["w_router"], np.float32)
        E, d = wr.shape
        up, down = dummy_ffn_weights(E, d, 2, np.random.default_rng(0))
        b = None if c["b_router"] is None else np.array(c["b_router"], np.float32)
        g = None if c["g_rms"] is None else np.array(c["g_rms"], np.float32)
        L = oracle.Layer(wr, up, down, b_router=b, g_rms=g, eps=c["eps"])
        scores, mask, a0 = oracle.router(L, np.array(c["x"], np.float32), return_a0=True)
        np.testing.assert_allclose(a0, np.array(c["a0"]), rtol=0, atol=1e-12, err_msg=c["name"])
        np.testing.assert_allclose(scores, np.array(c["scores"]), rtol=2e-7, atol=0, err_msg=c["name"])
        assert mask_to_sets(mask, E) == [set(s) for s in c["mask_bits"]], c["name"]


def test_router_bf16_weights_widen_exactly(oracle):
    # 0x3F81 = 1.0078125, 0xC040 = -3.0, 0x3E80 = 0.25 : bf16 patterns widened by a 16-bit shift
    wr = np.array([[0x3F81, 0xC040], [0x3E80, 0x3F80]], np.uint16)
    up = np.zeros((2, 1, 2), np.uint16)
    down = np.zeros((2, 2, 1), np.uint16)
    L = oracle.Layer(wr, up, down, eps=0.0)
    _, _, a0 = oracle.router(L, np.array([[2.0, 1.0]], np.float32), return_a0=True)
    np.testing.assert_array_equal(a0, [[2 * 1.0078125 - 3.0, 0.5 + 1.0]])


@pytest.mark.parametrize("E,d", [(1, 8), (5, 16), (16, 24), (63, 8), (64, 8), (65, 8), (130, 16)])
def test_router_invariants(oracle, E, d):
    rng = np.random.default_rng(E * 1000 + d)
    wr = rng.standard_normal((E, d)).astype(np.float32)
    up, down = dummy_ffn_weights(E, d, 2, rng)
    x = rng.standard_normal((40, d)).astype(np.float32)
    # (i) RMSNorm identity: sum_i A_i^2 = E * ms / (ms + eps), ms = mean_i ReLU(A0_i)^2
    for eps in (0.0, 1e-6, 0.5):
        L = oracle.Layer(wr, up, down, eps=eps)
        A, mask, a0 = oracle.router(L, x, return_a0=True)
        ms = (np.maximum(a0, 0) ** 2).mean(axis=1)
        has = ms > 0
        np.testing.assert_allclose((A.astype(np.float64) ** 2).sum(1)[has], E * ms[has] / (ms[has] + eps), rtol=1e-5)
        assert np.all(A[~has] == 0)
        # (ii) non-negative; zero pattern of A = zero pattern of ReLU(A0) = complement of the mask
        assert np.all(A >= 0)
        sets = mask_to_sets(mask, E)
        for t in range(x.shape[0]):
            assert sets[t] == set(np.nonzero(a0[t] > 0)[0].tolist())
            assert sets[t] == set(np.nonzero(A[t] > 0)[0].tolist())
    # (iii) no bias, eps = 0: positive rescaling of x leaves A unchanged
    L = oracle.Layer(wr, up, down, eps=0.0)
    A1, m1 = oracle.router(L, x)
    A2, m2 = oracle.router(L, (4.0 * x).astype(np.float32))   # power of two: exact rescale
    np.testing.assert_array_equal(m1, m2)
    np.testing.assert_allclose(A1, A2, rtol=1e-6)
    # (iv) permuting experts permutes scores and mask bits
    perm = rng.permutation(E)
    Lp = oracle.Layer(wr[perm], up[perm], down[perm], eps=0.0)
    Ap, mp = oracle.router(Lp, x)
    np.testing.assert_array_equal(Ap, A1[:, perm])
    assert mask_to_sets(mp, E) == [set(int(np.nonzero(perm == i)[0][0]) for i in s) for s in mask_to_sets(m1, E)]


def test_router_single_expert_closed_form(oracle):
    # E = 1: A = 0 for a0 <= 0, else g / sqrt(1 + eps / a0^2)
    wr = np.array([[2.0, 0.0, 0.0]], np.float32)
    up, down = dummy_ffn_weights(1, 3, 2, np.random.default_rng(1))
    g = np.array([3.0], np.float32)
    eps = 0.25
    L = oracle.Layer(wr, up, down, g_rms=g, eps=eps)
    x = np.array([[0.5, 9, 9], [-0.5, 9, 9], [4.0, 0, 0]], np.float32)
    A, mask = oracle.router(L, x)
    a0 = np.array([1.0, -1.0, 8.0])
    want = np.where(a0 > 0, 3.0 / np.sqrt(1 + eps / a0 ** 2), 0.0)
    np.testing.assert_allclose(A[:, 0], want, rtol=2e-7)
    assert mask[:, 0].tolist() == [1, 0, 1]


def test_router_matches_matmul_library(oracle):
    # special case served by a library routine: A0 is one fp64 matrix product
    rng = np.random.default_rng(5)
    E, d, T = 24, 96, 33
    wr = bf16_round(rng.standard_normal((E, d)) * 0.02)
    b = (rng.standard_normal(E) * 0.1).astype(np.float32)
    up, down = dummy_ffn_weights(E, d, 2, rng)
    x = rng.standard_normal((T, d)).astype(np.float32)
    L = oracle.Layer(bf16_bits(wr), bf16_bits(up), bf16_bits(down), b_router=b, eps=1e-6)
    A, mask, a0 = oracle.router(L, x, return_a0=True)
    ref = x.astype(np.float64) @ wr.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(a0, ref, rtol=0, atol=1e-13)


def test_router_exact_arithmetic_fixture_any_order(oracle):
    # x in {-4..4}/4, W_r in {-8..8}/64, b multiples of 2^-8: every partial sum is an exact
    # multiple of 2^-8 below 2^24 ulps, so integer arithmetic gives A0 with no rounding at all.
    rng = np.random.default_rng(11)
    E, d, T = 70, 512, 64
    xi = rng.integers(-4, 5, (T, d))
    wi = rng.integers(-8, 9, (E, d))
    bi = rng.integers(-300, 300, E)
    x = (xi / 4.0).astype(np.float32)
    wr = (wi / 64.0).astype(np.float32)
    b = (bi / 256.0).astype(np.float32)
    up, down = dummy_ffn_weights(E, d, 2, rng)
    L = oracle.Layer(wr, up, down, b_router=b, eps=0.0)
    A, mask, a0 = oracle.router(L, x, return_a0=True)
    exact = xi @ wi.T + bi            # integers: A0 * 256
    np.testing.assert_array_equal(a0 * 256.0, exact.astype(np.float64))
    assert mask_to_sets(mask, E) == [set(np.nonzero(r > 0)[0].tolist()) for r in exact]
    # the same in fp32 with a reversed summation order is still exact
    a0_f32_rev = (x[:, ::-1].astype(np.float32)[:, None, :] * wr[:, ::-1][None, :, :]).astype(np.float32)
    acc = np.zeros((T, E), np.float32)
    for j in range(d):
        acc = (acc + a0_f32_rev[:, :, j]).astype(np.float32)
    np.testing.assert_array_equal((acc + b).astype(np.float64) * 256.0, exact.astype(np.float64))


def test_router_sign_patterns_bruteforce(oracle):
    # identity router on signed unit vectors: the mask must be exactly the set of +1 coordinates
    E = d = 6
    wr = np.eye(E, dtype=np.float32)
    up, down = dummy_ffn_weights(E, d, 2, np.random.default_rng(2))
    L = oracle.Layer(wr, up, down, eps=0.0)
    pats = np.array(list(itertools.product([-1.0, 0.0, 1.0], repeat=d)), np.float32)
    A, mask = oracle.router(L, pats)
    want = [set(np.nonzero(p > 0)[0].tolist()) for p in pats]
    assert mask_to_sets(mask, E) == want
    # and with n active experts of equal A1, each score is sqrt(E / n)
    for p, a in zip(pats, A):
        n = int((p > 0).sum())
        if n:
            np.testing.assert_allclose(a[p > 0], math.sqrt(E / n), rtol=2e-7)


# ----------------------------------------------------------------------------- union / counts (Sec. 2.1, 3.3)

@pytest.mark.parametrize("E", [1, 16, 63, 64, 65, 128, 200])
@pytest.mark.parametrize("k", [1, 3, 4, 8, 32])
def test_union_bruteforce_sets(oracle, E, k):
    rng = np.random.default_rng(E * 100 + k)
    C = 9
    sets = []
    for c in range(C):
        base = set(np.nonzero(rng.random(E) < 0.25)[0].tolist())
        for t in range(k):
            if c == 0:
                sets.append(set())                       # an all-inactive chunk
            elif c == 1:
                sets.append(set(range(E)))               # an all-active chunk
            else:
                flip = set(np.nonzero(rng.random(E) < 0.05)[0].tolist())
                sets.append(base ^ flip)
    mask = sets_to_mask(sets, E)
    stats = np.array([5, 7], np.int64)                   # counts are ADDED to what is there
    union, idx, n = oracle.chunk_union(mask, k, E, stats)
    tls_inactive = sum(E - len(s) for s in sets)
    cls_inactive = 0
    for c in range(C):
        u = set().union(*sets[c * k:(c + 1) * k])
        assert mask_to_sets(union[c:c + 1], E)[0] == u
        assert n[c] == len(u)
        assert idx[c, :len(u)].tolist() == sorted(u)
        assert np.all(idx[c, len(u):] == -1)
        cls_inactive += E - len(u)
    assert stats.tolist() == [5 + tls_inactive, 7 + cls_inactive]
    assert n[0] == 0 and n[1] == E
    # unused high bits of the last word stay clear
    if E % 64:
        assert np.all(union[:, -1] >> np.uint64(E % 64) == 0)


def test_union_k1_and_repeated_tokens_and_monotonicity(oracle):
    rng = np.random.default_rng(3)
    E, T = 48, 64
    sets = [set(np.nonzero(rng.random(E) < 0.2)[0].tolist()) for _ in range(T)]
    mask = sets_to_mask(sets, E)
    # k = 1: union = token mask, CLS_1 count = TLS count
    st = np.zeros(2, np.int64)
    union, idx, n = oracle.chunk_union(mask, 1, E, st)
    np.testing.assert_array_equal(union, mask)
    assert st[0] == st[1]
    # k identical tokens: same union as one of them
    rep = np.repeat(mask[:8], 4, axis=0)
    u4, _, n4 = oracle.chunk_union(rep, 4, E)
    np.testing.assert_array_equal(u4, mask[:8])
    # CLS_k <= TLS and CLS_2k <= CLS_k for nested chunks
    prev = None
    for k in (1, 2, 4, 8, 16):
        st = np.zeros(2, np.int64)
        oracle.chunk_union(mask, k, E, st)
        tls = st[0] / (T * E)
        cls = st[1] / ((T // k) * E)
        assert cls <= tls + 1e-12
        if prev is not None:
            assert cls <= prev + 1e-12
        prev = cls


# ----------------------------------------------------------------------------- expert FFN (Eq. 1-2, Table 1)

def full_lists(T, k, E):
    C = T // k
    idx = np.tile(np.arange(E, dtype=np.int32), (C, 1))
    n = np.full((C,), E, np.int32)
    mask = sets_to_mask([set(range(E))] * T, E)
    return mask, idx, n


def test_ffn_hand_worked_golden(oracle):
    with open(os.path.join(HERE, "golden", "ffn_worked.json")) as f:
        gold = json.load(f)
    ln3 = math.log(3.0)
    assert abs(ln3 - gold["ln3"]) < 1e-15
    for c in gold["cases"]:
        up = np.array(c["w_up"], np.float32)
        down = np.array(c["w_down"], np.float32)
        gate = None if c["w_gate"] is None else np.array(c["w_gate"], np.float32)
        E, d_e, d = up.shape
        x = (np.array(c["x_ln3_units"]) * ln3 + np.array(c["x_plain"])).astype(np.float32)
        scores = np.array(c["scores"], np.float32)
        L = oracle.Layer(np.zeros((E, d), np.float32), up, down, w_gate=gate)
        want = np.array(c["y_ln3_units"]) * ln3
        y_dense = oracle.dense_ffn(L, x, scores)
        np.testing.assert_allclose(y_dense, want, rtol=3e-7, atol=1e-7, err_msg=c["name"])  # x is fp32-rounded ln 3
        mask, idx, n = full_lists(1, 1, E)
        y_sparse = oracle.sparse_ffn(L, x, scores, mask, idx, n, 1)
        np.testing.assert_array_equal(y_sparse, y_dense)


@pytest.mark.parametrize("wdtype", ["f32", "bf16"])
def test_ffn_single_expert_is_a_two_matmul_mlp(oracle, wdtype):
    rng = np.random.default_rng(21)
    d, d_e, T = 40, 24, 7
    up = (rng.standard_normal((1, d_e, d)) * 0.3).astype(np.float32)
    gate = (rng.standard_normal((1, d_e, d)) * 0.3).astype(np.float32)
    down = (rng.standard_normal((1, d, d_e)) * 0.3).astype(np.float32)
    if wdtype == "bf16":
        up, gate, down = bf16_round(up), bf16_round(gate), bf16_round(down)
        enc = bf16_bits
    else:
        enc = lambda a: a
    x = rng.standard_normal((T, d)).astype(np.float32)
    a = rng.random((T, 1)).astype(np.float32) + 0.5
    xd = x.astype(np.float64)
    # Eq. 2 through library matmuls and the library logistic function
    u = xd @ up[0].astype(np.float64).T
    want = a.astype(np.float64) * ((u * expit(u)) @ down[0].astype(np.float64).T)
    L = oracle.Layer(enc(np.zeros((1, d), np.float32)), enc(up), enc(down))
    np.testing.assert_allclose(oracle.dense_ffn(L, x, a), want, rtol=1e-12, atol=1e-13)
    # gated variant: Swish on the gate branch, plain product with the up branch
    g = xd @ gate[0].astype(np.float64).T
    want_g = a.astype(np.float64) * (((g * expit(g)) * u) @ down[0].astype(np.float64).T)
    Lg = oracle.Layer(enc(np.zeros((1, d), np.float32)), enc(up), enc(down), w_gate=enc(gate))
    np.testing.assert_allclose(oracle.dense_ffn(Lg, x, a), want_g, rtol=1e-12, atol=1e-13)


def test_ffn_one_hot_weights_closed_form(oracle):
    # W_up rows pick single coordinates of x, W_down has a single non-zero per (expert, neuron):
    # y[c] = sum over (i, j) hitting column c of A_i * Swish(x[p(i,j)]) * v(i,j)
    E, d, d_e = 3, 5, 2
    pick = {(0, 0): 4, (0, 1): 1, (1, 0): 0, (1, 1): 0, (2, 0): 3, (2, 1): 2}
    dest = {(0, 0): (2, 1.5), (0, 1): (0, -2.0), (1, 0): (4, 0.5), (1, 1): (2, 3.0), (2, 0): (1, 1.0), (2, 1): (1, -1.0)}
    up = np.zeros((E, d_e, d), np.float32)
    down = np.zeros((E, d, d_e), np.float32)
    for (i, j), p in pick.items():
        up[i, j, p] = 1.0
    for (i, j), (c, v) in dest.items():
        down[i, c, j] = v
    x = np.array([[0.5, -1.0, 2.0, -3.0, 1.25]], np.float32)
    A = np.array([[2.0, 0.5, 1.0]], np.float32)
    want = np.zeros(d)
    for (i, j), p in pick.items():
        c, v = dest[(i, j)]
        u = float(x[0, p])
        want[c] += float(A[0, i]) * (u / (1.0 + math.exp(-u))) * v
    L = oracle.Layer(np.zeros((E, d), np.float32), up, down)
    np.testing.assert_allclose(oracle.dense_ffn(L, x, A)[0], want, rtol=1e-14)


def test_ffn_multi_expert_is_weighted_sum_of_single_experts(oracle):
    rng = np.random.default_rng(8)
    E, d, d_e, T = 5, 16, 8, 6
    up = (rng.standard_normal((E, d_e, d)) * 0.3).astype(np.float32)
    gate = (rng.standard_normal((E, d_e, d)) * 0.3).astype(np.float32)
    down = (rng.standard_normal((E, d, d_e)) * 0.3).astype(np.float32)
    x = rng.standard_normal((T, d)).astype(np.float32)
    A = rng.random((T, E)).astype(np.float32)
    for gated in (False, True):
        L = oracle.Layer(np.zeros((E, d), np.float32), up, down, w_gate=gate if gated else None)
        y = oracle.dense_ffn(L, x, A)
        xd = x.astype(np.float64)
        want = np.zeros((T, d))
        for i in range(E):
            u = xd @ up[i].astype(np.float64).T
            h = (xd @ gate[i].astype(np.float64).T)
            h = (h * expit(h)) * u if gated else u * expit(u)
            want += A[:, i:i + 1].astype(np.float64) * (h @ down[i].astype(np.float64).T)
        np.testing.assert_allclose(y, want, rtol=1e-11, atol=1e-13)


def test_gated_with_gate_equal_up_reduces_to_nongated(oracle):
    # W_gate = W_up gives h_gated = u * Swish(u): the non-gated expert with W_down' = W_down diag(u)
    rng = np.random.default_rng(9)
    d, d_e = 12, 6
    up = (rng.standard_normal((1, d_e, d)) * 0.4).astype(np.float32)
    down64 = rng.standard_normal((d, d_e)) * 0.4
    x = rng.standard_normal((1, d)).astype(np.float32)
    u = (x.astype(np.float64) @ up[0].astype(np.float64).T)[0]
    u32 = u.astype(np.float32)                      # W_down' must be representable: round u once ...
    down_scaled = (down64.astype(np.float32) * u32[None, :]).astype(np.float32)
    # ... and compare against the gated oracle in a tolerance that covers that one rounding
    Lg = oracle.Layer(np.zeros((1, d), np.float32), up, down64.astype(np.float32)[None], w_gate=up)
    Ln = oracle.Layer(np.zeros((1, d), np.float32), up, down_scaled[None])
    a = np.ones((1, 1), np.float32)
    np.testing.assert_allclose(oracle.dense_ffn(Lg, x, a), oracle.dense_ffn(Ln, x, a), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("gated", [False, True])
def test_sparse_equals_dense_bitwise_and_skips(oracle, gated):
    rng = np.random.default_rng(13)
    E, d, d_e, k, C = 10, 24, 8, 4, 5
    T = k * C
    wr = (rng.standard_normal((E, d)) * 0.2).astype(np.float32)
    b = np.full(E, -1.0, np.float32)
    up = (rng.standard_normal((E, d_e, d)) * 0.3).astype(np.float32)
    gate = (rng.standard_normal((E, d_e, d)) * 0.3).astype(np.float32) if gated else None
    down = (rng.standard_normal((E, d, d_e)) * 0.3).astype(np.float32)
    x = rng.standard_normal((T, d)).astype(np.float32)
    x[:k] = -np.abs(x[:k]) * 0                      # chunk 0: zero input, bias negative: empty union
    L = oracle.Layer(wr, up, down, w_gate=gate, b_router=b)
    out = oracle.forward(L, x, k)
    assert out["n_active"][0] == 0
    cc = next(c for c in range(1, C) if 1 < out["n_active"][c] < E)   # a chunk that really skips experts
    y_dense = oracle.dense_ffn(L, x, out["scores"])
    np.testing.assert_array_equal(out["y"], y_dense)          # Sec. 3.3 premise: only exact zeros are left out
    assert np.all(out["y"][:k] == 0)                           # empty union: zero output
    # linearity in W_down and in the scores (powers of two: exact)
    L2 = oracle.Layer(wr, up, (2 * down).astype(np.float32), w_gate=gate, b_router=b)
    np.testing.assert_array_equal(oracle.dense_ffn(L2, x, out["scores"]), 2 * y_dense)
    np.testing.assert_array_equal(oracle.dense_ffn(L, x, (0.5 * out["scores"]).astype(np.float32)), 0.5 * y_dense)
    # a cleared mask bit removes the term even though the score is non-zero (skip, not multiply)
    mask2 = out["token_mask"].copy()
    i = int(out["active_idx"][cc, 0])
    first_tok_with_i = next(tt for tt in range(cc * k, (cc + 1) * k) if (int(mask2[tt, 0]) >> i) & 1)
    mask2[first_tok_with_i, 0] &= ~(np.uint64(1) << np.uint64(i))
    y_skip = oracle.sparse_ffn(L, x, out["scores"], mask2, out["active_idx"], out["n_active"], k)
    scores_zeroed = out["scores"].copy()
    scores_zeroed[first_tok_with_i, i] = 0.0
    np.testing.assert_array_equal(y_skip, oracle.dense_ffn(L, x, scores_zeroed))
    assert not np.array_equal(y_skip, y_dense)
    # an expert left out of the union list is not visited for any token of that chunk
    idx2, n2 = out["active_idx"].copy(), out["n_active"].copy()
    idx2[cc, :n2[cc] - 1] = idx2[cc, 1:n2[cc]]
    idx2[cc, n2[cc] - 1] = -1
    n2[cc] -= 1
    y_drop = oracle.sparse_ffn(L, x, out["scores"], out["token_mask"], idx2, n2, k)
    sc = out["scores"].copy()
    sc[cc * k:(cc + 1) * k, i] = 0.0
    np.testing.assert_array_equal(y_drop, oracle.dense_ffn(L, x, sc))


# ----------------------------------------------------------------------------- generator statistics

@pytest.mark.parametrize("k,sigma,indep", [(8, 0.3, False), (4, 0.3, False), (32, 0.5, False), (1, 0.0, True)])
def test_generator_sparsity_matches_closed_form(oracle, k, sigma, indep):
    from paper_2507_08771_amd import workloads as wl

    w = wl.Workload("t", d=512, E=64, d_e=8, wdtype="bf16", gated=False, k=k, n_chunks=4096 // k,
                    sigma=sigma, independent=indep, seed=3)
    layers = wl.make_layers(w, 1)
    x = wl.make_tokens(w, layers)
    L = oracle.Layer(wl.to_numpy(layers["w_router"][0]), wl.to_numpy(layers["w_up"][0]),
                     wl.to_numpy(layers["w_down"][0]), b_router=wl.to_numpy(layers["b_router"][0]))
    scores, mask, a0 = oracle.router(L, wl.to_numpy(x), return_a0=True)
    st = np.zeros(2, np.int64)
    oracle.chunk_union(mask, k, w.E, st)
    tls = st[0] / (w.n_tok * w.E)
    cls = st[1] / (w.n_chunks * w.E)
    e_tls, e_cls = wl.expected_sparsity(k, sigma, independent=indep)
    assert abs(tls - e_tls) < 0.01
    assert abs(cls - e_cls) < 0.03
    # the guard band holds
    mag = np.abs(wl.to_numpy(x)).astype(np.float64) @ np.abs(layers["w_router"][0].double().numpy()).T \
        + np.abs(layers["b_router"][0].double().numpy())
    assert np.all(np.abs(a0) > wl.GUARD_REL * mag)


def test_expected_sparsity_reference_values():
    from paper_2507_08771_amd import workloads as wl

    # independent tokens: an expert is idle for a whole chunk with probability 0.8^k
    assert wl.expected_sparsity(8, 0.0, independent=True)[1] == pytest.approx(0.8 ** 8)
    # sigma -> infinity behaves like independent tokens; sigma -> 0 like one token
    assert wl.expected_sparsity(8, 200.0)[1] == pytest.approx(0.8 ** 8, abs=2e-3)
    assert wl.expected_sparsity(8, 1e-3)[1] == pytest.approx(0.8, abs=2e-3)
    # the levels the workloads aim at (about 70 % for 8 correlated tokens, lower for 32 noisier ones)
    assert wl.expected_sparsity(8, 0.3)[1] == pytest.approx(0.672, abs=2e-3)
    assert wl.expected_sparsity(32, 0.5)[1] == pytest.approx(0.464, abs=2e-3)
