"""Pins for the oracle of the CLS-aware objectives (Eq. 4 and Eq. 5): a library routine on the
range where it applies, closed forms, exact rational brute force, and the link between the
chunk sparsification loss and the chunk's expert union."""

import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import router_losses as rl


def test_locality_loss_equals_library_bce_on_moderate_values():
    rng = np.random.default_rng(0)
    a0 = rng.normal(size=(3 * 9, 12)).astype(np.float32)
    alpha = 4.0
    a = torch.from_numpy(a0).double().reshape(3, 9, 12)
    want = torch.nn.functional.binary_cross_entropy(torch.sigmoid(alpha * a[:, :-1]), torch.sigmoid(alpha * a[:, 1:]))
    assert rl.activation_locality_loss(a0, 9, alpha) == pytest.approx(float(want), rel=1e-12)


def test_locality_loss_scalar_definition():
    """-[q ln p + (1 - q) ln(1 - p)] typed out with math.* on a two-token, two-expert stream;
    input is the earlier token, target the later one (swapping them changes the value)."""
    a0 = np.array([[0.5, -1.0], [2.0, 0.25]], dtype=np.float32)
    alpha = 1.5
    sig = lambda v: 1.0 / (1.0 + math.exp(-v))
    terms = []
    for i in range(2):
        p, q = sig(alpha * float(a0[0, i])), sig(alpha * float(a0[1, i]))
        terms.append(-(q * math.log(p) + (1 - q) * math.log(1 - p)))
    assert rl.activation_locality_loss(a0, 2, alpha) == pytest.approx(sum(terms) / 2, rel=1e-14)
    swapped = rl.activation_locality_loss(a0[::-1].copy(), 2, alpha)
    assert abs(swapped - sum(terms) / 2) > 1e-3


def test_locality_loss_closed_forms():
    rng = np.random.default_rng(1)
    a0 = rng.normal(size=(16, 8)).astype(np.float32)
    # alpha = 0: p = q = 1/2 everywhere
    assert rl.activation_locality_loss(a0, 16, 0.0) == pytest.approx(math.log(2.0), rel=1e-15)
    # identical neighbours: the cross entropy is the binary entropy of sigmoid(alpha * a)
    row = rng.normal(size=(1, 8)).astype(np.float32)
    same = np.repeat(row, 5, axis=0)
    p = 1.0 / (1.0 + np.exp(-2.0 * row.astype(np.float64)))
    h = -(p * np.log(p) + (1 - p) * np.log(1 - p))
    assert rl.activation_locality_loss(same, 5, 2.0) == pytest.approx(float(h.mean()), rel=1e-13)
    # sharp alpha: agreeing signs cost nothing, a flipped sign costs alpha * |a| (no clamping)
    agree = np.array([[1.0, -1.0], [2.0, -3.0]], dtype=np.float32)
    assert rl.activation_locality_loss(agree, 2, 1000.0) == pytest.approx(0.0, abs=1e-300)
    flip = np.array([[1.0], [-1.0]], dtype=np.float32)
    assert rl.activation_locality_loss(flip, 2, 1000.0) == pytest.approx(1000.0, rel=1e-15)
    # pairs never cross sequences; a length-1 sequence has no pair
    two = np.array([[1.0], [-1.0], [1.0], [1.0]], dtype=np.float32)
    assert rl.activation_locality_loss(two, 2, 1000.0) == pytest.approx(500.0, rel=1e-15)
    assert rl.activation_locality_loss(two, 4, 1000.0) == pytest.approx(2000.0 / 3, rel=1e-15)
    assert rl.activation_locality_loss(two, 1, 1000.0) == 0.0


def brute_cs(a0_int, seq_len, L):
    """Exact rational evaluation of Eq. 5 for integer pre-activations."""
    n_tok, E = a0_int.shape
    total, chunks = Fraction(0), 0
    for base in range(0, n_tok, seq_len):
        for j in range(seq_len // L):
            idle = [Fraction(1)] * E
            for t in range(base + j * L, base + (j + 1) * L):
                a1 = [max(int(v), 0) for v in a0_int[t]]
                s = sum(a1)
                for i in range(E):
                    idle[i] *= 1 - (Fraction(a1[i], s) if s else 0)
            total += sum(1 - v for v in idle) / E
            chunks += 1
    return float(total / chunks) if chunks else 0.0


@pytest.mark.parametrize("E,seq_len,n_seq,L", [(4, 6, 2, 3), (7, 10, 3, 4), (16, 8, 2, 8), (5, 5, 2, 1)])
def test_chunk_sparsification_exact_rational_brute_force(E, seq_len, n_seq, L):
    rng = np.random.default_rng(E + L)
    a0 = rng.integers(-6, 5, size=(seq_len * n_seq, E))
    a0[1] = -1          # a token with no active expert
    a0[2] = 0
    a0[2, 0] = 3        # a token with a single active expert: p = 1
    got = rl.chunk_sparsification_loss(a0.astype(np.float32), seq_len, L)
    assert got == pytest.approx(brute_cs(a0, seq_len, L), rel=1e-13)


def test_chunk_sparsification_closed_forms():
    E, L = 8, 4
    # one-hot tokens: an expert is active with probability 1 iff it is in the chunk's union
    onehot = np.full((L, E), -1.0, dtype=np.float32)
    for k, e in enumerate([2, 5, 2, 7]):
        onehot[k, e] = 3.0 + k
    assert rl.chunk_sparsification_loss(onehot, L, L) == pytest.approx(3 / E, rel=1e-15)
    # every expert equally active: P_act = 1 - (1 - 1/E)^L for each of them
    flat = np.full((L, E), 0.7, dtype=np.float32)
    assert rl.chunk_sparsification_loss(flat, L, L) == pytest.approx(1 - (1 - 1 / E) ** L, rel=1e-14)
    # L = 1: P_act = p, which sums to one over the experts of a token with any active expert
    rng = np.random.default_rng(3)
    a0 = rng.normal(size=(20, E)).astype(np.float32)
    a0[4] = -1.0
    nonempty = (a0 > 0).any(axis=1).mean()
    assert rl.chunk_sparsification_loss(a0, 20, 1) == pytest.approx(nonempty / E, rel=1e-13)
    # a chunk of all-inactive tokens costs nothing; positive rescaling changes nothing
    assert rl.chunk_sparsification_loss(np.full((4, E), -2.0, np.float32), 4, 4) == 0.0
    assert rl.chunk_sparsification_loss(4.0 * a0, 20, 5) == pytest.approx(rl.chunk_sparsification_loss(a0, 20, 5), rel=1e-12)
    # the tail shorter than L is left out; no chunk at all gives 0
    assert rl.chunk_sparsification_loss(a0, 20, 8) == pytest.approx(rl.chunk_sparsification_loss(a0[:16], 16, 8), rel=1e-15)
    assert rl.chunk_sparsification_loss(a0, 20, 21) == 0.0


def test_chunk_sparsification_bounds_the_union_ratio_from_below():
    """P_act <= 1 and is 0 for an expert outside the union, so L_cs never exceeds the share of
    experts active in the chunk (1 - CLS_L for that chunk), and grows with the chunk length."""
    rng = np.random.default_rng(5)
    E, L = 16, 8
    a0 = (rng.normal(size=(L * 10, E)) - 0.8).astype(np.float32)
    act = (a0 > 0).reshape(10, L, E).any(axis=1).mean()
    cs8 = rl.chunk_sparsification_loss(a0, L * 10, L)
    assert 0.0 < cs8 <= act
    assert rl.chunk_sparsification_loss(a0, L * 10, 4) <= cs8 + 1e-15
