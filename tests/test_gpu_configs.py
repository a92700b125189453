"""GPU parity at the full sizes of the measured configurations, in the launch configurations
the benchmark uses (chunks rotating through distinct weight sets), checked on sampled chunks
against the oracle plus properties that hold at any size."""

import numpy as np
import pytest
import torch

from paper_2507_08771_amd import binding as B
from paper_2507_08771_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu


def popcount_rows(m):
    return np.array([bin(int(v)).count("1") for v in m.reshape(-1)]).reshape(m.shape).sum(axis=1)


def full_size_case(name, n_layers, chunks, dense_sampled=True):
    w = wl.WORKLOADS[name]
    layers = wl.make_layers(w, n_layers, device="cuda")
    cl = wl.make_chunk_layer(w, n_layers, device="cuda")
    x = wl.make_tokens(w, layers, cl, device="cuda")
    print("generated", name, flush=True)
    gpu = pu.run_gpu(layers, x, w.k, cl, dense=dense_sampled)
    layers_cpu = {n: (None if t is None else t.cpu()) for n, t in layers.items()}
    ref = pu.run_oracle(layers_cpu, x.cpu(), w.k, cl.cpu(), dense=dense_sampled, chunks=chunks)
    pu.assert_integers_equal(gpu, ref, chunks=chunks, k=w.k)
    rows = (np.asarray(chunks)[:, None] * w.k + np.arange(w.k)[None, :]).reshape(-1)
    print(pu.assert_floats_close(gpu, ref, "bf16", rows=rows, dense=dense_sampled))
    C, E, W = w.n_chunks, w.E, w.mask_words
    np.testing.assert_array_equal(popcount_rows(gpu["union_mask"]), gpu["n_active"])
    tm = gpu["token_mask"].reshape(C, w.k, W)
    np.testing.assert_array_equal(np.bitwise_or.reduce(tm, axis=1), gpu["union_mask"])
    assert gpu["stats"][1] == C * E - gpu["n_active"].sum()
    assert gpu["stats"][0] == w.n_tok * E - popcount_rows(gpu["token_mask"]).sum()
    e_tls, e_cls = wl.expected_sparsity(w.k, w.sigma, w.p_active, independent=w.independent)
    assert abs(gpu["stats"][0] / (w.n_tok * E) - e_tls) < 0.01
    assert abs(gpu["stats"][1] / (C * E) - e_cls) < 0.02
    assert np.isfinite(gpu["y"]).all()
    # tokens with no active expert get an exactly zero row, all others a non-zero one
    none_active = popcount_rows(gpu["token_mask"]) == 0
    assert np.all(gpu["y"][none_active] == 0)
    assert np.all(np.abs(gpu["y"][~none_active]).max(axis=1) > 0)


def test_decode_k1_full_size():
    """Single-token decode: 4096 independent tokens, d = 1024, 32 experts (TLS only: CLS_1 = TLS)."""
    full_size_case("decode_k1", 8, [0, 1, 7, 8, 1000, 2047, 2048, 4094, 4095] + list(range(300, 340)))


def test_tree_k32_full_size():
    """Tree verification: 512 sets x 4 sequences = 2048 chunks of 32 tokens, one union each."""
    full_size_case("tree_k32", 4, [0, 3, 1025, 2047], dense_sampled=False)


def test_paper_shape_two_mask_words():
    """The paper's 2.8B shape: Eq. 2 experts, N_e = 128 (two mask words), d_e = 128, k = 32."""
    full_size_case("paper_k32", 2, [0, 1, 255, 511], dense_sampled=False)


def test_paper_shape_table11_sparsity_levels():
    """The 2.8B shape at Table 11's levels: 12.45 % of the experts active per token (k = 1) and
    30.86 % active in the union of a 32-token tree (checked against the generator's closed form
    inside full_size_case)."""
    full_size_case("paper_ar_k1", 4, [0, 1, 63, 64, 2049, 4095] + list(range(700, 716)))
    full_size_case("paper_tree_k32", 2, [0, 1, 511, 1023], dense_sampled=False)
    w = wl.WORKLOADS["paper_tree_k32"]
    assert abs((1 - wl.expected_sparsity(w.k, w.sigma, w.p_active)[1]) - 0.3086) < 1e-4


def test_prefill_512_eight_chunks_through_eight_weight_sets():
    """The 512-token prefill chunk in the launch configuration the benchmark times: 8 chunks, each
    through its own weight set, on the matrix-core path (tiles that share an expert's weights
    run side by side on one XCD, items rotate their start in the contraction).  Two chunks are
    checked in full against the oracle; integers and union properties on all of them."""
    w = wl.WORKLOADS["stack_prefill_512"].replace(n_chunks=8)
    n_layers = 8
    layers = wl.make_layers(w, n_layers, device="cuda")
    cl = wl.make_chunk_layer(w, n_layers, device="cuda")
    x = wl.make_tokens(w, layers, cl, device="cuda")
    print("generated", flush=True)
    gpu = pu.run_gpu(layers, x, w.k, cl, dense=False)
    chunks = [0, 5]
    layers_cpu = {n: (None if t is None else t.cpu()) for n, t in layers.items()}
    ref = pu.run_oracle(layers_cpu, x.cpu(), w.k, cl.cpu(), dense=False, chunks=chunks)
    pu.assert_integers_equal(gpu, ref, chunks=chunks, k=w.k)
    rows = (np.asarray(chunks)[:, None] * w.k + np.arange(w.k)[None, :]).reshape(-1)
    print(pu.assert_floats_close(gpu, ref, "bf16", rows=rows, bar=pu.GEMM_BAR, l2_bar=pu.GEMM_L2_BAR))
    C, E, W = w.n_chunks, w.E, w.mask_words
    np.testing.assert_array_equal(popcount_rows(gpu["union_mask"]), gpu["n_active"])
    tm = gpu["token_mask"].reshape(C, w.k, W)
    np.testing.assert_array_equal(np.bitwise_or.reduce(tm, axis=1), gpu["union_mask"])
    assert gpu["n_active"].min() >= E - 2          # 64 groups of 8 tokens: the union is all but dense
    assert np.isfinite(gpu["y"]).all()
    none_active = popcount_rows(gpu["token_mask"]) == 0
    assert np.all(gpu["y"][none_active] == 0)
    assert np.all(np.abs(gpu["y"][~none_active]).max(axis=1) > 0)


def test_stack_decode_24_layers_chained():
    """24 layers, one k = 8 chunk walking through them: x_{l+1} = (x_l + y_l) rescaled per token to
    the rms of x_0 (stands in for the attention and norms between FFNs).  Every layer is checked
    against the oracle on the input the GPU path actually had.  Inputs after layer 0 are not
    drawn with the generator's guard band, so mask bits are compared wherever the fp64
    pre-activation is further from zero than the guard band; elsewhere either value is valid and
    the FFN is then compared on the tokens whose masks agree."""
    w = wl.WORKLOADS["stack_decode_k8"]
    NL = 24
    layers = wl.make_layers(w, NL, device="cuda")
    x0 = wl.make_tokens(w, {n: (None if t is None else t[:1]) for n, t in layers.items()}, device="cuda")
    L = B.Layer.from_dict(layers, gain=False)
    buf = B.Buffers(L, 1, w.k)
    layers_cpu = {n: (None if t is None else t.cpu()) for n, t in layers.items()}
    rms0 = x0.pow(2).mean(dim=1, keepdim=True).sqrt()
    x = x0.clone()
    unguarded = 0
    for l in range(NL):
        cl = torch.tensor([l], dtype=torch.int32, device="cuda")
        B.forward_chunks(L, x, buf, cl)
        torch.cuda.synchronize()
        OL = pu.oracle_layer(layers_cpu, l, use_gain=False)
        import oracle
        xs = x.cpu().numpy()
        scores, mask, a0 = oracle.router(OL, xs, return_a0=True)
        mag = np.abs(xs).astype(np.float64) @ np.abs(layers_cpu["w_router"][l].double().numpy()).T \
            + np.abs(layers_cpu["b_router"][l].double().numpy())
        safe = np.abs(a0) > wl.GUARD_REL * mag
        unguarded += int((~safe).sum())
        g_mask = buf.token_mask.cpu().numpy().view(np.uint64)
        g_bits = ((g_mask[:, 0:1] >> np.arange(w.E, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)
        r_bits = a0 > 0
        np.testing.assert_array_equal(g_bits[safe], r_bits[safe], err_msg="layer %d" % l)
        # oracle FFN driven by the GPU's own masks and lists (they are valid where they differ)
        g_idx, g_n = buf.active_idx.cpu().numpy(), buf.n_active.cpu().numpy()
        union = set(np.nonzero(g_bits.any(axis=0))[0].tolist())
        assert g_idx[0, :g_n[0]].tolist() == sorted(union) and np.all(g_idx[0, g_n[0]:] == -1)
        same = (g_bits == r_bits).all(axis=1)
        y_ref = oracle.sparse_ffn(OL, xs, scores, g_mask, g_idx, g_n, w.k)
        e_s = pu.row_rel_err(buf.scores.cpu().numpy()[same], scores[same]).max(initial=0.0)
        e_y = pu.row_rel_err(buf.y.cpu().numpy()[same], y_ref[same]).max(initial=0.0)
        assert e_s <= 1e-5 and e_y <= pu.TIGHT["bf16"], (l, e_s, e_y)
        z = x + buf.y
        x = (z * (rms0 / z.pow(2).mean(dim=1, keepdim=True).sqrt())).contiguous()
    print("pre-activations inside the guard band over 24 layers:", unguarded)
    assert unguarded < 8


def test_layer_stack_replayed_as_a_graph():
    """The launches of a few layers (router, union, FFN per layer, one k = 8 chunk) captured once as
    a graph of kernel nodes and replayed: every replay, with eager work and synchronisations of
    the program's own between them, must give the bits of the eager run."""
    w = wl.WORKLOADS["stack_decode_k8"]
    NL = 4
    layers = wl.make_layers(w, NL, device="cuda")
    L = B.Layer.from_dict(layers, gain=False)
    xs = [wl.make_tokens(w, {n: (None if t is None else t[l:l + 1]) for n, t in layers.items()}, device="cuda", seed=50 + l)
          for l in range(NL)]
    bufs = [B.Buffers(L, 1, w.k) for _ in range(NL)]
    cls = [torch.tensor([l], dtype=torch.int32, device="cuda") for l in range(NL)]

    def run_layers():
        for l in range(NL):
            B.forward_chunks(L, xs[l], bufs[l], cls[l])

    run_layers()
    torch.cuda.synchronize()
    want = [(b.y.clone(), b.scores.clone(), b.active_idx.clone(), b.stats.clone()) for b in bufs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_layers()
    for rep in range(3):
        for b in bufs:
            b.y.fill_(float("nan"))
            b.workspace.fill_(rep)            # eager work between the replays, on the buffers the graph uses
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l, b in enumerate(bufs):
            assert torch.equal(b.y, want[l][0]), (rep, l)
            assert torch.equal(b.scores, want[l][1]) and torch.equal(b.active_idx, want[l][2])
        # the counts are added to on every run (the capture itself launches nothing)
        assert torch.equal(bufs[0].stats, want[0][3] * (rep + 2))


@pytest.mark.parametrize("variant", range(8))
def test_read_stream_probe_runs_in_every_variant(variant):
    """blockffn_stream_read (the benchmark's ceiling measurement): every launch shape, plain and
    non-temporal loads, on a buffer whose size is no multiple of a tile; it only reads (the buffer
    and the sink keep their contents), and a stream of 1 GiB must run at a rate that is a memory
    rate at all (above 1 TB/s, below the 8 TB/s rating)."""
    n = (1 << 30) + 4096 + 16
    buf = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    sink = torch.full((1,), 123, dtype=torch.int32, device="cuda")
    B.blockffn_stream_read(buf, variant, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    B.blockffn_stream_read(buf, variant, sink)
    e1.record()
    torch.cuda.synchronize()
    rate = n / (e0.elapsed_time(e1) * 1e-3) / 1e12
    assert 1.0 < rate < 8.0, rate
    assert int(sink.item()) == 123
    assert int(buf[:4096].sum().item()) == 7 * 4096 and int(buf[-1].item()) == 7
