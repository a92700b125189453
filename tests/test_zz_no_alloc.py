"""blockffn_sparse_ffn_static (the entry point that allocates nothing: its workspace is a static
device array) against blockffn_sparse_ffn on the same inputs, through the C ABI.

The two share their kernels, which write every output element exactly once in a fixed order, so
the results must agree bit for bit (stricter than the tolerance the outputs are held to against
the oracle).  Every case makes two calls in a row on the shared static array, the second with a
smaller input, so that whatever the first call left behind in the array is in the way of the
second."""

import numpy as np
import pytest
import torch

from paper_2507_08771_amd import binding as B
from paper_2507_08771_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu


def run_both(w, seed):
    """Router + union, then the FFN through both entry points; returns (y_workspace, y_static)."""
    w = w.replace(seed=seed)
    layers = wl.make_layers(w, 1)
    x = wl.make_tokens(w, layers).cuda()
    dev = pu.to_device(layers)
    L = B.Layer.from_dict(dev, gain=False)
    buf = B.Buffers(L, w.n_chunks, w.k)
    B.forward_chunks(L, x, buf)                       # fills scores / masks / lists and buf.y
    y_static = torch.full_like(buf.y, float("nan"))
    before = torch.cuda.memory_allocated()
    B.blockffn_sparse_ffn_static(L, x, buf.scores, buf.token_mask, buf.active_idx, buf.n_active, w.n_chunks, w.k,
                                 y_static)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return buf, x, layers, y_static


@pytest.mark.parametrize("first,second", [
    # few chunks (one workgroup per (slot, row tile), split down projection), then fewer and shorter
    (dict(d=2048, E=64, d_e=256, k=8, n_chunks=6, gated=True), dict(d=2048, E=64, d_e=256, k=5, n_chunks=2, gated=True)),
    # the persistent up kernel with its work list, then a launch too small for it
    (dict(d=2048, E=64, d_e=128, k=8, n_chunks=40, gated=True), dict(d=1024, E=32, d_e=128, k=1, n_chunks=9, gated=True)),
    # 32-token chunks (token-major mid, token bits, the block of zeros), Eq. 2 experts, two mask words
    (dict(d=2048, E=128, d_e=128, k=32, n_chunks=12, gated=False), dict(d=2048, E=128, d_e=128, k=20, n_chunks=3, gated=False)),
    # a large chunk on the matrix-core path (token lists, mid cleared by the library), then a short one
    (dict(d=1024, E=32, d_e=128, k=200, n_chunks=2, gated=True), dict(d=1024, E=32, d_e=128, k=40, n_chunks=1, gated=True)),
    # fp32 weights: the shape-generic kernels
    (dict(d=264, E=16, d_e=24, k=4, n_chunks=7, gated=True), dict(d=264, E=16, d_e=24, k=3, n_chunks=2, gated=False)),
])
def test_static_scratch_matches_the_workspace_entry_point(first, second):
    for i, cfg in enumerate((first, second)):
        wdtype = "f32" if cfg["d"] == 264 else "bf16"
        w = wl.Workload("no_alloc", wdtype=wdtype, sigma=0.3, **cfg)
        print("call", i, cfg, flush=True)
        buf, x, layers, y_static = run_both(w, seed=31 + i)
        assert torch.equal(y_static, buf.y), "call %d: static-scratch result differs from the workspace result" % i
        assert torch.isfinite(y_static).all()
        # and both are the right answer: chunk 0 against the oracle
        ref = pu.run_oracle(layers, x.cpu(), w.k, None, chunks=[0])
        e = pu.row_rel_err(y_static[:w.k].cpu().numpy(), ref["y"][:w.k]).max(initial=0.0)
        assert e <= (pu.GEMM_BAR if w.k > 32 else pu.TIGHT[wdtype]), e


def test_static_scratch_rejects_what_does_not_fit_and_leaves_y_alone():
    w = wl.Workload("no_alloc", d=2048, E=64, d_e=128, wdtype="bf16", gated=True, k=8, n_chunks=1024, sigma=0.3)
    layers = wl.make_layers(w, 1, device="cuda")
    L = B.Layer.from_dict(layers, gain=False)
    assert B.blockffn_workspace_bytes(L, w.n_chunks, w.k) > B.STATIC_SCRATCH_BYTES
    x = torch.zeros((w.n_tok, w.d), device="cuda")
    scores = torch.zeros((w.n_tok, w.E), device="cuda")
    mask = torch.zeros((w.n_tok, 1), dtype=torch.int64, device="cuda")
    idx = torch.full((w.n_chunks, w.E), -1, dtype=torch.int32, device="cuda")
    n_act = torch.zeros((w.n_chunks,), dtype=torch.int32, device="cuda")
    y = torch.full((w.n_tok, w.d), 7.0, device="cuda")
    with pytest.raises(B.BlockffnError) as err:
        B.blockffn_sparse_ffn_static(L, x, scores, mask, idx, n_act, w.n_chunks, w.k, y)
    assert err.value.code == B.ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())      # nothing was enqueued
