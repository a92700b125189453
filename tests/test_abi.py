"""The C-ABI library loads without a GPU, exports what the header declares, and rejects bad
arguments with the documented codes before anything is launched."""

import ctypes
import os
import re

import pytest

from paper_2507_08771_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "blockffn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(blockffn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = header_functions()
    assert set(B.EXPORTS) <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.blockffn_version() == 102


def test_binding_has_the_same_names():
    for n in header_functions():
        if n in ("blockffn_strerror", "blockffn_version"):
            continue
        assert hasattr(B, n), n


def test_strerror():
    assert B.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert B.strerror(code) not in ("ok", "unknown error code")
    assert B.strerror(-99) == "unknown error code"


def layer(**kw):
    base = dict(d=2048, n_experts=64, d_e=128, wdtype=B.BF16, expert_kind=B.EXPERT_GATED, n_layers=1,
                rms_eps=1e-6, reserved=0, w_router=0x1000, b_router=None, g_rms=None, w_up=0x2000,
                w_gate=0x3000, w_down=0x4000)
    base.update(kw)
    return B.BlockffnLayer(*[base[f[0]] for f in B.BlockffnLayer._fields_])


FAKE = ctypes.c_void_p(0x10000)   # never dereferenced: every call below fails validation or has no chunks


def router_rc(lay, n_chunks=1, k=8, x=FAKE, scores=FAKE, mask=FAKE):
    return B.lib().blockffn_router(ctypes.byref(lay), None, x, n_chunks, k, scores, mask, None)


def test_invalid_arguments_are_rejected_without_a_gpu():
    lib = B.lib()
    assert router_rc(layer(), n_chunks=0) == B.OK                    # nothing to do is fine
    assert lib.blockffn_router(None, None, FAKE, 1, 8, FAKE, FAKE, None) == B.ERR_INVALID
    assert router_rc(layer(), x=None) == B.ERR_INVALID
    assert router_rc(layer(), scores=None) == B.ERR_INVALID
    assert router_rc(layer(), k=0) == B.ERR_INVALID
    assert router_rc(layer(), n_chunks=-1) == B.ERR_INVALID
    assert router_rc(layer(), k=513) == B.ERR_UNSUPPORTED
    assert router_rc(layer(d=2044)) == B.ERR_INVALID
    assert router_rc(layer(d_e=12)) == B.ERR_INVALID
    assert router_rc(layer(n_experts=0)) == B.ERR_INVALID
    assert router_rc(layer(n_experts=257)) == B.ERR_UNSUPPORTED
    assert router_rc(layer(d_e=2048)) == B.ERR_UNSUPPORTED
    assert router_rc(layer(wdtype=7)) == B.ERR_UNSUPPORTED
    assert router_rc(layer(expert_kind=3)) == B.ERR_INVALID
    assert router_rc(layer(n_layers=0)) == B.ERR_INVALID
    assert router_rc(layer(rms_eps=-1.0)) == B.ERR_INVALID
    assert router_rc(layer(rms_eps=float("nan"))) == B.ERR_INVALID
    assert router_rc(layer(w_router=None)) == B.ERR_INVALID
    assert router_rc(layer(w_up=0x2008)) == B.ERR_INVALID            # not 16-byte aligned
    assert router_rc(layer(w_gate=None)) == B.ERR_INVALID            # gated needs w_gate
    assert router_rc(layer(expert_kind=B.EXPERT_SWISH)) == B.ERR_INVALID   # non-gated must not pass one
    assert router_rc(layer(expert_kind=B.EXPERT_SWISH, w_gate=None), n_chunks=0) == B.OK


def test_union_and_ffn_argument_checks():
    lib = B.lib()
    assert lib.blockffn_chunk_union(FAKE, 0, 8, 64, FAKE, FAKE, FAKE, None, None) == B.OK
    assert lib.blockffn_chunk_union(None, 1, 8, 64, FAKE, FAKE, FAKE, None, None) == B.ERR_INVALID
    assert lib.blockffn_chunk_union(FAKE, 1, 0, 64, FAKE, FAKE, FAKE, None, None) == B.ERR_INVALID
    assert lib.blockffn_chunk_union(FAKE, 1, 8, 0, FAKE, FAKE, FAKE, None, None) == B.ERR_INVALID
    assert lib.blockffn_chunk_union(FAKE, 1, 8, 300, FAKE, FAKE, FAKE, None, None) == B.ERR_UNSUPPORTED
    assert lib.blockffn_chunk_union(FAKE, 1, 600, 64, FAKE, FAKE, FAKE, None, None) == B.ERR_UNSUPPORTED
    lay = layer()
    need = lib.blockffn_workspace_bytes(ctypes.byref(lay), 4, 8)
    assert need >= 4 * 64 * 8 * 128 * 4 and need % 256 == 0
    assert lib.blockffn_workspace_bytes(ctypes.byref(layer(d=3)), 4, 8) == 0
    sparse = lambda ws, nbytes, n_act=FAKE: lib.blockffn_sparse_ffn(
        ctypes.byref(lay), None, FAKE, FAKE, FAKE, FAKE, n_act, 4, 8, FAKE, ws, nbytes, None)
    assert sparse(FAKE, need - 1) == B.ERR_WORKSPACE
    assert sparse(None, need) == B.ERR_INVALID
    assert sparse(ctypes.c_void_p(0x10010), need) == B.ERR_INVALID   # workspace not 256-byte aligned
    assert sparse(FAKE, need, n_act=None) == B.ERR_INVALID
    assert lib.blockffn_dense_ffn(ctypes.byref(lay), None, FAKE, FAKE, 4, 8, FAKE, FAKE, need - 1, None) == B.ERR_WORKSPACE
    assert lib.blockffn_dense_ffn(ctypes.byref(lay), None, FAKE, None, 4, 8, FAKE, FAKE, need, None) == B.ERR_INVALID
    assert lib.blockffn_dense_ffn(ctypes.byref(lay), None, FAKE, FAKE, 0, 8, FAKE, None, 0, None) == B.OK


def test_sizes_beyond_32_bit_indexing_are_unsupported():
    """(chunk, slot) pairs and tokens are indexed in 32 bits inside the kernels: larger calls are
    refused as unsupported before anything is launched (not reported as a launch failure)."""
    lib = B.lib()
    lay = layer()
    big = 1 << 40
    sparse = lambda n_chunks, k: lib.blockffn_sparse_ffn(ctypes.byref(lay), None, FAKE, FAKE, FAKE, FAKE, FAKE,
                                                         n_chunks, k, FAKE, FAKE, big, None)
    assert sparse(1 << 26, 8) == B.ERR_UNSUPPORTED       # 2^26 chunks x 64 experts = 2^32 pairs
    assert sparse(1 << 28, 8) == B.ERR_UNSUPPORTED       # 2^31 tokens
    assert router_rc(lay, n_chunks=1 << 28, k=8) == B.ERR_UNSUPPORTED
    assert lib.blockffn_dense_ffn(ctypes.byref(lay), None, FAKE, FAKE, 1 << 26, 8, FAKE, FAKE, big, None) == B.ERR_UNSUPPORTED
    assert lib.blockffn_workspace_bytes(ctypes.byref(lay), 1 << 28, 8) == 0


def test_static_scratch_entry_point_argument_checks():
    """The entry point without a workspace argument: same argument checks as blockffn_sparse_ffn,
    and a shape that needs more than the static array is refused with its own code.  None of
    these calls reaches the GPU."""
    lib = B.lib()
    lay = layer()
    f = lambda n_chunks=4, k=8, x=FAKE, scores=FAKE, mask=FAKE, idx=FAKE, n_act=FAKE, y=FAKE, l=lay: \
        lib.blockffn_sparse_ffn_static(ctypes.byref(l), None, x, scores, mask, idx, n_act, n_chunks, k, y, None)
    assert f(n_chunks=0) == B.OK
    assert f(x=None) == B.ERR_INVALID and f(scores=None) == B.ERR_INVALID and f(mask=None) == B.ERR_INVALID
    assert f(idx=None) == B.ERR_INVALID and f(n_act=None) == B.ERR_INVALID and f(y=None) == B.ERR_INVALID
    assert f(k=0) == B.ERR_INVALID and f(k=513) == B.ERR_UNSUPPORTED
    assert f(l=layer(d=2044)) == B.ERR_INVALID
    assert lib.blockffn_workspace_bytes(ctypes.byref(lay), 2048, 8) > B.STATIC_SCRATCH_BYTES
    assert f(n_chunks=2048) == B.ERR_SCRATCH
    # the capacities the header names
    big = layer(d_e=256)
    for n_chunks, k in ((200, 8), (56, 32), (1, 512)):
        assert lib.blockffn_workspace_bytes(ctypes.byref(big), n_chunks, k) <= B.STATIC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "blockffn.h")).read()
    assert re.search(r"#define\s+BLOCKFFN_STATIC_SCRATCH_BYTES\s+\(128u << 20\)", text)


def test_forward_chunks_argument_checks():
    lib = B.lib()
    lay = layer()
    f = lambda n_chunks=1, k=8, x=FAKE, scores=FAKE, mask=FAKE, union=FAKE, idx=FAKE, n_act=FAKE, y=FAKE, ws=FAKE, \
        nbytes=1 << 30, l=lay: lib.blockffn_forward_chunks(ctypes.byref(l), None, x, n_chunks, k, scores, mask, union,
                                                           idx, n_act, None, y, ws, nbytes, None)
    assert f(n_chunks=0) == B.OK
    assert lib.blockffn_forward_chunks(None, None, FAKE, 1, 8, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, 1 << 30,
                                       None) == B.ERR_INVALID
    for kw in (dict(x=None), dict(scores=None), dict(mask=None), dict(union=None), dict(idx=None), dict(n_act=None),
               dict(y=None), dict(ws=None), dict(k=0), dict(n_chunks=-1), dict(ws=ctypes.c_void_p(0x10010))):
        assert f(**kw) == B.ERR_INVALID, kw
    assert f(k=513) == B.ERR_UNSUPPORTED
    assert f(nbytes=256) == B.ERR_WORKSPACE
    # a shape that runs the three stages as they are is checked by them
    assert f(n_chunks=4096, x=None) == B.ERR_INVALID


def test_force_generic_modes():
    lib = B.lib()
    for mode in (1, 0, -1):
        assert lib.blockffn_force_generic(mode) == B.OK
    assert lib.blockffn_force_generic(2) == B.ERR_INVALID and lib.blockffn_force_generic(-2) == B.ERR_INVALID
    assert lib.blockffn_stream_read(None, 1024, 0, FAKE, None) == B.ERR_INVALID
    assert lib.blockffn_stream_read(FAKE, 1024, 8, FAKE, None) == B.ERR_INVALID
    assert lib.blockffn_stream_read(FAKE, 1024, 0, None, None) == B.ERR_INVALID


def test_statistics_argument_checks():
    lib = B.lib()
    sweep = lambda mask=FAKE, n_tok=64, seq=16, E=64, l_max=8, a=FAKE, b=FAKE, c=FAKE: lib.blockffn_cls_sweep(
        mask, n_tok, seq, E, l_max, a, b, c, None)
    assert sweep(mask=None) == B.ERR_INVALID
    assert sweep(n_tok=-1) == B.ERR_INVALID
    assert sweep(seq=0) == B.ERR_INVALID
    assert sweep(n_tok=65) == B.ERR_INVALID            # not a whole number of sequences
    assert sweep(E=0) == B.ERR_INVALID
    assert sweep(E=257) == B.ERR_UNSUPPORTED
    assert sweep(l_max=0) == B.ERR_INVALID
    assert sweep(l_max=65) == B.ERR_UNSUPPORTED
    assert sweep(a=None) == B.ERR_INVALID and sweep(b=None) == B.ERR_INVALID and sweep(c=None) == B.ERR_INVALID
    assert sweep(a=ctypes.c_void_p(0x10004)) == B.ERR_INVALID
    reuse = lambda mask=FAKE, n_tok=64, seq=16, E=64, a=FAKE, b=FAKE, c=FAKE: lib.blockffn_reuse_ratio(
        mask, n_tok, seq, E, a, b, c, None)
    assert reuse(mask=None) == B.ERR_INVALID
    assert reuse(n_tok=60) == B.ERR_INVALID
    assert reuse(E=300) == B.ERR_UNSUPPORTED
    assert reuse(a=None) == B.ERR_INVALID and reuse(b=None) == B.ERR_INVALID and reuse(c=None) == B.ERR_INVALID


def test_losses_argument_checks():
    lib = B.lib()
    need = lib.blockffn_losses_workspace_bytes()
    assert need > 0 and need % 8 == 0
    f = lambda a0=FAKE, n_tok=64, seq=16, E=64, L=8, alpha=1.0, out=FAKE, ws=FAKE, nbytes=need: \
        lib.blockffn_router_losses(a0, n_tok, seq, E, L, alpha, out, ws, nbytes, None)
    assert f(a0=None) == B.ERR_INVALID
    assert f(n_tok=65) == B.ERR_INVALID
    assert f(seq=0) == B.ERR_INVALID
    assert f(L=0) == B.ERR_INVALID
    assert f(E=0) == B.ERR_INVALID
    assert f(E=257) == B.ERR_UNSUPPORTED
    assert f(alpha=-1.0) == B.ERR_INVALID
    assert f(alpha=float("nan")) == B.ERR_INVALID
    assert f(alpha=float("inf")) == B.ERR_INVALID
    assert f(out=None) == B.ERR_INVALID and f(ws=None) == B.ERR_INVALID
    assert f(nbytes=need - 1) == B.ERR_WORKSPACE
    lay = layer()
    assert lib.blockffn_router_preact(ctypes.byref(lay), None, FAKE, 1, 8, FAKE, FAKE, ctypes.c_void_p(0x10002),
                                      None) == B.ERR_INVALID     # misaligned pre-activation buffer
    assert lib.blockffn_router_preact(ctypes.byref(lay), None, FAKE, 0, 8, FAKE, FAKE, None, None) == B.OK


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libblockffn.so"))
    with pytest.raises(RuntimeError):
        B.lib()
