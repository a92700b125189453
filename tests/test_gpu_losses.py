"""GPU parity of the router pre-activation output and of the forward values of the CLS-aware
objectives (Eq. 4, Eq. 5) against the oracle."""

import numpy as np
import pytest
import torch

from paper_2507_08771_amd import binding as B
from paper_2507_08771_amd import workloads as wl
import oracle
from oracle import router_losses as rl

import parity_util as pu

pytestmark = pytest.mark.gpu

RTOL = 1e-11   # fp64 sums of up to ~10^6 terms in a different order, device exp / log1p within a few ulp


def gpu_losses(a0_np, seq_len, E, L, alpha):
    a0 = torch.from_numpy(np.ascontiguousarray(a0_np, dtype=np.float32)).cuda()
    losses = torch.full((2,), -7.0, dtype=torch.float64, device="cuda")
    ws = torch.empty(B.blockffn_losses_workspace_bytes(), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)   # workspace contents are undefined on entry: NaN patterns must not leak
    B.blockffn_router_losses(a0, a0_np.shape[0], seq_len, E, L, alpha, losses, ws)
    torch.cuda.synchronize()
    return losses.cpu().numpy()


CASES = [
    # E, seq_len, n_seq, L, alpha
    (5, 7, 3, 3, 1.0),
    (64, 16, 40, 8, 8.0),
    (64, 1000, 3, 32, 64.0),     # more pairs than waves: grid-stride, sharp sigmoid
    (70, 33, 5, 4, 0.0),         # alpha = 0: ln 2
    (130, 64, 4, 64, 3.0),       # three words of experts, one chunk per sequence
    (256, 8, 200, 8, 1000.0),    # widest; saturated sigmoids
    (32, 1, 50, 1, 2.0),         # length-1 sequences: no pair, every token a chunk
    (16, 6, 4, 7, 2.0),          # chunk longer than the sequence: no chunk
]


@pytest.mark.parametrize("E,seq_len,n_seq,L,alpha", CASES)
def test_losses_match_oracle(E, seq_len, n_seq, L, alpha):
    rng = np.random.default_rng(E * 13 + seq_len)
    a0 = (rng.normal(size=(seq_len * n_seq, E)) - 0.84).astype(np.float32)
    a0[::7] = -1.0                      # tokens with no active expert
    if a0.shape[0] > 3:
        a0[3] = -1.0
        a0[3, E // 2] = 0.5             # a single active expert: p = 1, ln 0
    got = gpu_losses(a0, seq_len, E, L, alpha)
    want = (rl.activation_locality_loss(a0, seq_len, alpha), rl.chunk_sparsification_loss(a0, seq_len, L))
    assert got[0] == pytest.approx(want[0], rel=RTOL, abs=1e-300)
    assert got[1] == pytest.approx(want[1], rel=RTOL, abs=1e-300)


def test_losses_repeat_bit_for_bit():
    rng = np.random.default_rng(9)
    a0 = rng.normal(size=(4096, 64)).astype(np.float32)
    a = gpu_losses(a0, 512, 64, 8, 16.0)
    b = gpu_losses(a0, 512, 64, 8, 16.0)
    assert a.tobytes() == b.tobytes()


def test_empty_stream_gives_zero():
    got = gpu_losses(np.zeros((0, 64), np.float32), 16, 64, 8, 1.0)
    assert got[0] == 0.0 and got[1] == 0.0


@pytest.mark.parametrize("name,n_layers,n_chunks", [("tiny_f32_k4", 1, 16), ("spec_k8", 3, 200), ("paper_k32", 2, 6),
                                                  ("stack_decode_k8", 2, 2)])
def test_router_preact_and_losses_end_to_end(name, n_layers, n_chunks):
    """The pre-activations the router kernel reports are the values behind its masks, agree with
    the fp64 oracle to fp32 summation error, and leave scores / masks identical to blockffn_router.
    The losses of the chunks (sequence = chunk, so pairs stay among tokens sharing a centre) are
    then evaluated on the device values and compared with the oracle on the same values."""
    w = wl.WORKLOADS[name].replace(n_chunks=n_chunks)
    layers = wl.make_layers(w, n_layers, device="cuda")
    cl = wl.make_chunk_layer(w, n_layers, device="cuda")
    x = wl.make_tokens(w, layers, cl, device="cuda")
    L = B.Layer.from_dict(layers, gain=False)
    n_tok, E, W = w.n_tok, w.E, w.mask_words
    scores = torch.empty((n_tok, E), dtype=torch.float32, device="cuda")
    mask = torch.empty((n_tok, W), dtype=torch.int64, device="cuda")
    scores2, mask2 = torch.empty_like(scores), torch.empty_like(mask)
    pre = torch.full((n_tok, E), float("nan"), dtype=torch.float32, device="cuda")
    B.blockffn_router(L, x, w.n_chunks, w.k, scores, mask, cl)
    B.blockffn_router_preact(L, x, w.n_chunks, w.k, scores2, mask2, pre, cl)
    torch.cuda.synchronize()
    assert torch.equal(scores, scores2) and torch.equal(mask, mask2)
    pre_np = pre.cpu().numpy()
    m = mask.cpu().numpy().view(np.uint64)
    bits = np.zeros((n_tok, E), dtype=bool)
    for i in range(E):
        bits[:, i] = (m[:, i // 64] >> np.uint64(i % 64)) & np.uint64(1)
    np.testing.assert_array_equal(pre_np > 0, bits)
    layers_cpu = {n: (None if t is None else t.cpu()) for n, t in layers.items()}
    xs, cls = x.cpu().numpy(), cl.cpu().numpy()
    for c in range(w.n_chunks):
        OL = pu.oracle_layer(layers_cpu, int(cls[c]), use_gain=False)
        rows = slice(c * w.k, (c + 1) * w.k)
        _, _, a0 = oracle.router(OL, xs[rows], return_a0=True)
        mag = np.abs(xs[rows]).astype(np.float64) @ np.abs(layers_cpu["w_router"][int(cls[c])].double().numpy()).T
        assert np.all(np.abs(pre_np[rows] - a0) <= 1e-6 * (mag + 1.0))
    alpha = 16.0
    got = gpu_losses(pre_np, w.k, E, w.k, alpha)
    if w.k > 1:
        assert got[0] == pytest.approx(rl.activation_locality_loss(pre_np, w.k, alpha), rel=RTOL)
    assert got[1] == pytest.approx(rl.chunk_sparsification_loss(pre_np, w.k, w.k), rel=RTOL)
    # Eq. 5 is 0 for experts outside the chunk's union: it never exceeds the union's share
    union_share = bits.reshape(w.n_chunks, w.k, E).any(axis=1).mean()
    assert 0.0 < got[1] <= union_share
