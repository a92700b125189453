"""Pins for the sparsity-statistics oracle (CLS_L sweep of Sec. 2.1 / Fig. 1(a) and the reuse
ratio of Sec. 4.1.2): closed forms on constructed masks, exact rational brute force with Python
sets, and cross-checks against the chunk-union oracle, which is separate code."""

from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import sparsity_stats as ss


def masks_from_sets(sets, E):
    W = (E + 63) // 64
    m = np.zeros((len(sets), W), dtype=np.uint64)
    for t, s in enumerate(sets):
        for i in s:
            m[t, i // 64] |= np.uint64(1) << np.uint64(i % 64)
    return m


def random_sets(rng, n, E, p):
    return [set(np.nonzero(rng.random(E) < p)[0].tolist()) for _ in range(n)]


def brute_cls(sets, E, seq_len, L, sliding):
    """(inactive, windows) by set unions over explicitly listed windows."""
    inactive = windows = 0
    for base in range(0, len(sets), seq_len):
        if sliding:
            starts = range(0, seq_len - L + 1)
        else:
            starts = range(0, (seq_len // L) * L, L)
        for s in starts:
            u = set()
            for t in range(base + s, base + s + L):
                u |= sets[t]
            inactive += E - len(u)
            windows += 1
    return inactive, windows


@pytest.mark.parametrize("E,seq_len,n_seq,p", [(5, 7, 3, 0.3), (64, 16, 2, 0.1), (70, 12, 4, 0.05), (130, 9, 2, 0.2)])
def test_cls_sweep_brute_force_with_sets(E, seq_len, n_seq, p):
    rng = np.random.default_rng(E * 1000 + seq_len)
    sets = random_sets(rng, seq_len * n_seq, E, p)
    L_max = seq_len + 2   # includes lengths with no window at all
    inactive, windows, cls = ss.cls_sweep(masks_from_sets(sets, E), E, seq_len, L_max)
    for L in range(1, L_max + 1):
        for mode, sliding in ((0, False), (1, True)):
            if L <= seq_len:
                bi, bw = brute_cls(sets, E, seq_len, L, sliding)
            else:
                bi, bw = 0, 0
            assert (inactive[mode, L - 1], windows[mode, L - 1]) == (bi, bw), (L, mode)
            want = float(Fraction(bi, bw * E)) if bw else 0.0
            assert cls[mode, L - 1] == pytest.approx(want, rel=1e-15, abs=0)


def test_cls_window_counts_closed_form():
    E, seq_len, n_seq, L_max = 8, 11, 3, 13
    m = np.zeros((seq_len * n_seq, 1), dtype=np.uint64)
    inactive, windows, cls = ss.cls_sweep(m, E, seq_len, L_max)
    for L in range(1, L_max + 1):
        assert windows[0, L - 1] == n_seq * (seq_len // L)
        assert windows[1, L - 1] == n_seq * max(0, seq_len - L + 1)
    # no expert ever active: every window is fully sparse
    assert np.all(inactive == windows * E)
    assert np.all(cls[windows > 0] == 1.0) and np.all(cls[windows == 0] == 0.0)


def test_cls_rotating_single_expert_closed_form():
    """Token t activates expert t mod E only: a window of L tokens holds min(L, E) distinct
    experts, so CLS_L = 1 - min(L, E) / E for both window families."""
    E, seq_len = 6, 24
    sets = [{t % E} for t in range(seq_len)]
    inactive, windows, cls = ss.cls_sweep(masks_from_sets(sets, E), E, seq_len, 10)
    for L in range(1, 11):
        want = 1.0 - min(L, E) / E
        assert cls[0, L - 1] == pytest.approx(want, abs=1e-15)
        assert cls[1, L - 1] == pytest.approx(want, abs=1e-15)


def test_cls_identical_tokens_equal_tls_for_every_length():
    E, seq_len = 70, 16
    s = {1, 5, 64, 69}
    inactive, windows, cls = ss.cls_sweep(masks_from_sets([s] * seq_len, E), E, seq_len, 16)
    assert np.allclose(cls, 1.0 - len(s) / E, rtol=0, atol=1e-15)


def test_cls_matches_chunk_union_counts():
    """L = 1 is TLS and disjoint windows of L = k are the chunks of the union step: the two
    inactive-pair counters of the chunk-union oracle (separate C code) must be reproduced."""
    rng = np.random.default_rng(3)
    E, k, C = 40, 4, 12
    sets = random_sets(rng, k * C, E, 0.2)
    m = masks_from_sets(sets, E)
    stats = np.zeros(2, dtype=np.int64)
    oracle.chunk_union(m, k, E, stats)
    inactive, windows, _ = ss.cls_sweep(m, E, k * C, k)
    assert inactive[0, 0] == inactive[1, 0] == stats[0]
    assert inactive[0, k - 1] == stats[1] and windows[0, k - 1] == C


def test_cls_nested_chunks_are_monotone():
    """A window of 2L tokens is inactive only where both of its halves are: CLS_2L <= CLS_L on
    disjoint windows when the sequence length is a multiple of 2L (Sec. 2.1, Fig. 1(a))."""
    rng = np.random.default_rng(5)
    E, seq_len = 32, 64
    m = masks_from_sets(random_sets(rng, seq_len * 2, E, 0.1), E)
    _, _, cls = ss.cls_sweep(m, E, seq_len, 32)
    for L in (1, 2, 4, 8, 16):
        assert cls[0, 2 * L - 1] <= cls[0, L - 1]
    # sliding windows: a longer window starting at the same token can only be less sparse
    assert cls[1, 0] >= cls[1, 31]


def test_cls_ignores_bits_at_or_above_E():
    E = 10
    m = np.array([[0b1 | (1 << 12)], [0b10 | (1 << 63)]], dtype=np.uint64)
    inactive, _, _ = ss.cls_sweep(m, E, 2, 2)
    assert inactive[0, 0] == 2 * E - 2 and inactive[0, 1] == E - 2


def test_cls_independent_masks_statistics():
    """Experts drawn independently with probability p: E[CLS_L] = (1 - p)^L."""
    rng = np.random.default_rng(11)
    E, seq_len, p = 64, 512, 0.2
    m = masks_from_sets(random_sets(rng, seq_len, E, p), E)
    _, windows, cls = ss.cls_sweep(m, E, seq_len, 8)
    for L in range(1, 9):
        q = (1 - p) ** L
        for mode in (0, 1):
            n_indep = E * (seq_len // L)   # sliding windows overlap: no more independent ones
            assert abs(cls[mode, L - 1] - q) < 5 * np.sqrt(q * (1 - q) / n_indep) + 1e-12


# ------------------------------------------------------------------------------------ reuse ratio

def brute_reuse(sets, seq_len):
    total, pairs = Fraction(0), 0
    for base in range(0, len(sets), seq_len):
        for i in range(base, base + seq_len - 1):
            if sets[i]:
                total += Fraction(len(sets[i] & sets[i + 1]), len(sets[i]))
                pairs += 1
    return total, pairs


@pytest.mark.parametrize("E,seq_len,n_seq,p", [(5, 6, 3, 0.4), (64, 20, 2, 0.15), (130, 10, 3, 0.1)])
def test_reuse_ratio_exact_rational_brute_force(E, seq_len, n_seq, p):
    rng = np.random.default_rng(E + seq_len)
    sets = random_sets(rng, seq_len * n_seq, E, p)
    sets[2] = set()          # an empty S_i: its pair is left out
    sets[seq_len - 1] = set(range(E))   # last token of a sequence: never a first element
    num, cnt, ratio = ss.reuse_ratio(masks_from_sets(sets, E), E, seq_len)
    total, pairs = brute_reuse(sets, seq_len)
    assert cnt.sum() == pairs and cnt[0] == 0 and num[0] == 0
    assert sum(Fraction(int(num[c]), c) for c in range(1, E + 1)) == total
    assert ratio == pytest.approx(float(total / pairs), rel=1e-14)


def test_reuse_ratio_closed_forms():
    E = 8
    f = lambda sets, L: ss.reuse_ratio(masks_from_sets(sets, E), E, L)[2]
    assert f([{1, 2, 3}] * 5, 5) == 1.0                         # identical neighbours
    assert f([{0, 1}, {2, 3}] * 3, 6) == 0.0                    # disjoint neighbours
    assert f([{t % E, (t + 1) % E} for t in range(12)], 12) == 0.5   # one of two kept
    assert f([set(range(i + 1)) for i in range(E)], E) == 1.0   # growing sets: S_i inside S_{i+1}
    shrink = [set(range(E - i)) for i in range(E)]              # S_{i+1} = S_i minus one expert
    want = sum(Fraction(E - i - 1, E - i) for i in range(E - 1)) / (E - 1)
    assert f(shrink, E) == pytest.approx(float(want), rel=1e-15)
    # asymmetric: the ratio divides by |S_i|, not |S_{i+1}|
    assert f([{0, 1, 2, 3}, {0}], 2) == 0.25 and f([{0}, {0, 1, 2, 3}], 2) == 1.0


def test_reuse_ratio_pairs_do_not_cross_sequences():
    E = 4
    sets = [{0}, {0}, {1}, {1}]
    assert ss.reuse_ratio(masks_from_sets(sets, E), E, 2)[2] == 1.0   # pairs (0,1) and (2,3)
    assert ss.reuse_ratio(masks_from_sets(sets, E), E, 4)[2] == pytest.approx(2 / 3)
    # no pair at all (length-1 sequences, or every first token empty) reports 0
    assert ss.reuse_ratio(masks_from_sets(sets, E), E, 1)[2] == 0.0
    assert ss.reuse_ratio(masks_from_sets([set(), {1}], E), E, 2) [2] == 0.0


def test_reuse_ratio_independent_masks_statistics():
    """Independent draws with probability p: E[|S_i & S_{i+1}| / |S_i|] = p."""
    rng = np.random.default_rng(2)
    E, n, p = 64, 2000, 0.2
    ratio = ss.reuse_ratio(masks_from_sets(random_sets(rng, n, E, p), E), E, n)[2]
    assert abs(ratio - p) < 5 * np.sqrt(p * (1 - p) / (n * E * p))
