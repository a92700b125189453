"""ctypes binding of ``libblockffn.so``: argument marshalling only.

Every function here has the name of the C entry point it calls (``include/blockffn.h``)
and passes device pointers of torch tensors straight through; no arithmetic of the layer
happens in Python.  ``lib()`` raises if the shared library has not been built: there is no
fallback path.
"""

from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libblockffn.so")

F32, BF16 = 0, 1
EXPERT_SWISH, EXPERT_GATED = 0, 1
OK, ERR_INVALID, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH, ERR_SCRATCH = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 128 << 20

EXPORTS = ("blockffn_router", "blockffn_chunk_union", "blockffn_sparse_ffn", "blockffn_dense_ffn",
           "blockffn_sparse_ffn_up", "blockffn_sparse_ffn_down", "blockffn_workspace_bytes", "blockffn_strerror",
           "blockffn_version", "blockffn_cls_sweep", "blockffn_reuse_ratio", "blockffn_router_preact",
           "blockffn_router_losses", "blockffn_losses_workspace_bytes", "blockffn_offload_sim",
           "blockffn_sparse_ffn_static", "blockffn_stream_read",
           "blockffn_force_generic", "blockffn_forward_chunks")


class BlockffnLayer(ctypes.Structure):
    """Mirror of ``struct blockffn_layer``."""

    _fields_ = [
        ("d", ctypes.c_int32), ("n_experts", ctypes.c_int32), ("d_e", ctypes.c_int32),
        ("wdtype", ctypes.c_int32), ("expert_kind", ctypes.c_int32), ("n_layers", ctypes.c_int32),
        ("rms_eps", ctypes.c_float), ("reserved", ctypes.c_int32),
        ("w_router", ctypes.c_void_p), ("b_router", ctypes.c_void_p), ("g_rms", ctypes.c_void_p),
        ("w_up", ctypes.c_void_p), ("w_gate", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
    ]


class BlockffnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, strerror(code), code))


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it is missing (build it first)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libblockffn.so is not built: run `python -m paper_2507_08771_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        lp = ctypes.POINTER(BlockffnLayer)
        L.blockffn_router.argtypes = [lp, vp, vp, i64, i32, vp, vp, vp]
        L.blockffn_chunk_union.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, vp]
        L.blockffn_sparse_ffn.argtypes = [lp, vp, vp, vp, vp, vp, vp, i64, i32, vp, vp, sz, vp]
        L.blockffn_dense_ffn.argtypes = [lp, vp, vp, vp, i64, i32, vp, vp, sz, vp]
        L.blockffn_sparse_ffn_static.argtypes = [lp, vp, vp, vp, vp, vp, vp, i64, i32, vp, vp]
        L.blockffn_sparse_ffn_up.argtypes = [lp, vp, vp, vp, vp, vp, vp, i64, i32, vp, sz, vp]
        L.blockffn_sparse_ffn_down.argtypes = [lp, vp, vp, vp, i64, i32, vp, vp, sz, vp]
        L.blockffn_router_preact.argtypes = [lp, vp, vp, i64, i32, vp, vp, vp, vp]
        L.blockffn_router_losses.argtypes = [vp, i64, i64, i32, i32, ctypes.c_float, vp, vp, sz, vp]
        L.blockffn_losses_workspace_bytes.argtypes = []
        L.blockffn_losses_workspace_bytes.restype = sz
        L.blockffn_offload_sim.argtypes = [vp, vp, i64, i32, i32, vp, vp]
        L.blockffn_offload_sim.restype = ctypes.c_int
        L.blockffn_cls_sweep.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
        L.blockffn_reuse_ratio.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp]
        L.blockffn_forward_chunks.argtypes = [lp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.blockffn_forward_chunks.restype = ctypes.c_int
        L.blockffn_force_generic.argtypes = [ctypes.c_int]
        L.blockffn_force_generic.restype = ctypes.c_int
        L.blockffn_stream_read.argtypes = [vp, sz, i32, vp, vp]
        L.blockffn_stream_read.restype = ctypes.c_int
        L.blockffn_workspace_bytes.argtypes = [lp, i64, i32]
        L.blockffn_workspace_bytes.restype = sz
        L.blockffn_strerror.argtypes = [ctypes.c_int]
        L.blockffn_strerror.restype = ctypes.c_char_p
        L.blockffn_version.restype = ctypes.c_int
        for n in ("blockffn_router", "blockffn_chunk_union", "blockffn_sparse_ffn", "blockffn_dense_ffn",
                  "blockffn_sparse_ffn_up", "blockffn_sparse_ffn_down", "blockffn_cls_sweep",
                  "blockffn_reuse_ratio", "blockffn_router_preact", "blockffn_router_losses",
                  "blockffn_sparse_ffn_static"):
            getattr(L, n).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().blockffn_strerror(int(code)).decode()


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(rc: int, where: str):
    if rc != OK:
        raise BlockffnError(rc, where)


class Layer:
    """Device weights of ``n_layers`` stacked layers plus the C struct describing them."""

    def __init__(self, w_router, w_up, w_down, w_gate=None, b_router=None, g_rms=None, eps: float = 1e-6):
        if w_router.dim() == 2:   # a single layer given without the leading dimension
            w_router, w_up, w_down = w_router[None], w_up[None], w_down[None]
            w_gate = None if w_gate is None else w_gate[None]
            b_router = None if b_router is None else b_router[None]
            g_rms = None if g_rms is None else g_rms[None]
        self.n_layers, self.E, self.d = w_router.shape
        self.d_e = w_up.shape[2]
        assert w_up.shape == (self.n_layers, self.E, self.d_e, self.d)
        assert w_down.shape == (self.n_layers, self.E, self.d, self.d_e)
        self.wdtype = BF16 if w_router.dtype == torch.bfloat16 else F32
        self.tensors = [t.contiguous() if t is not None else None
                        for t in (w_router, b_router, g_rms, w_up, w_gate, w_down)]
        self.gated = w_gate is not None
        self.W = (self.E + 63) // 64
        self.device = w_router.device
        t = self.tensors
        self.c = BlockffnLayer(self.d, self.E, self.d_e, self.wdtype,
                               EXPERT_GATED if self.gated else EXPERT_SWISH, self.n_layers, float(eps), 0,
                               *[None if q is None else q.data_ptr() for q in t])

    @classmethod
    def from_dict(cls, layers: Dict[str, torch.Tensor], eps: float = 1e-6, gain: bool = True) -> "Layer":
        return cls(layers["w_router"], layers["w_up"], layers["w_down"], layers.get("w_gate"),
                   layers.get("b_router"), layers.get("g_rms") if gain else None, eps)

    def ref(self):
        return ctypes.byref(self.c)


def blockffn_workspace_bytes(layer: Layer, n_chunks: int, k: int) -> int:
    return int(lib().blockffn_workspace_bytes(layer.ref(), n_chunks, k))


def blockffn_router(layer: Layer, x: torch.Tensor, n_chunks: int, k: int, scores: torch.Tensor,
                    token_mask: torch.Tensor, chunk_layer: Optional[torch.Tensor] = None, stream=None):
    _check(lib().blockffn_router(layer.ref(), _p(chunk_layer), _p(x), n_chunks, k, _p(scores), _p(token_mask),
                                 _stream(stream)), "blockffn_router")


def blockffn_chunk_union(token_mask: torch.Tensor, n_chunks: int, k: int, n_experts: int, union_mask: torch.Tensor,
                         active_idx: torch.Tensor, n_active: torch.Tensor, stats: Optional[torch.Tensor] = None,
                         stream=None):
    _check(lib().blockffn_chunk_union(_p(token_mask), n_chunks, k, n_experts, _p(union_mask), _p(active_idx),
                                      _p(n_active), _p(stats), _stream(stream)), "blockffn_chunk_union")


def blockffn_router_preact(layer: Layer, x, n_chunks: int, k: int, scores, token_mask, preact, chunk_layer=None,
                           stream=None):
    _check(lib().blockffn_router_preact(layer.ref(), _p(chunk_layer), _p(x), n_chunks, k, _p(scores), _p(token_mask),
                                        _p(preact), _stream(stream)), "blockffn_router_preact")


def blockffn_losses_workspace_bytes() -> int:
    return int(lib().blockffn_losses_workspace_bytes())


def blockffn_router_losses(preact: torch.Tensor, n_tok: int, seq_len: int, n_experts: int, chunk_len: int,
                           alpha: float, losses: torch.Tensor, workspace: torch.Tensor, stream=None):
    _check(lib().blockffn_router_losses(_p(preact), n_tok, seq_len, n_experts, chunk_len, alpha, _p(losses),
                                        _p(workspace), workspace.numel() * workspace.element_size(),
                                        _stream(stream)), "blockffn_router_losses")


def blockffn_offload_sim(active_idx: torch.Tensor, n_active: torch.Tensor, n_experts: int, capacity: int,
                         loads_per_chunk: Optional[torch.Tensor], totals: torch.Tensor):
    """HOST tensors (int32 lists, int64 outputs): the simulation runs on the CPU."""
    for t in (active_idx, n_active, loads_per_chunk, totals):
        if t is not None and (t.is_cuda or not t.is_contiguous()):
            raise ValueError("blockffn_offload_sim takes contiguous host tensors")
    _check(lib().blockffn_offload_sim(_p(active_idx), _p(n_active), n_active.numel(), n_experts, capacity,
                                      _p(loads_per_chunk), _p(totals)), "blockffn_offload_sim")


def blockffn_cls_sweep(token_mask: torch.Tensor, n_tok: int, seq_len: int, n_experts: int, l_max: int,
                       inactive: torch.Tensor, windows: torch.Tensor, cls: torch.Tensor, stream=None):
    _check(lib().blockffn_cls_sweep(_p(token_mask), n_tok, seq_len, n_experts, l_max, _p(inactive), _p(windows),
                                    _p(cls), _stream(stream)), "blockffn_cls_sweep")


def blockffn_reuse_ratio(token_mask: torch.Tensor, n_tok: int, seq_len: int, n_experts: int, num: torch.Tensor,
                         cnt: torch.Tensor, ratio: torch.Tensor, stream=None):
    _check(lib().blockffn_reuse_ratio(_p(token_mask), n_tok, seq_len, n_experts, _p(num), _p(cnt), _p(ratio),
                                      _stream(stream)), "blockffn_reuse_ratio")


def blockffn_sparse_ffn(layer: Layer, x, scores, token_mask, active_idx, n_active, n_chunks: int, k: int, y,
                        workspace: torch.Tensor, chunk_layer=None, stream=None):
    _check(lib().blockffn_sparse_ffn(layer.ref(), _p(chunk_layer), _p(x), _p(scores), _p(token_mask), _p(active_idx),
                                     _p(n_active), n_chunks, k, _p(y), _p(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)),
           "blockffn_sparse_ffn")


def blockffn_sparse_ffn_static(layer: Layer, x, scores, token_mask, active_idx, n_active, n_chunks: int, k: int, y,
                               chunk_layer=None, stream=None):
    """blockffn_sparse_ffn on the library's static scratch: no workspace argument, nothing allocated."""
    _check(lib().blockffn_sparse_ffn_static(layer.ref(), _p(chunk_layer), _p(x), _p(scores), _p(token_mask),
                                            _p(active_idx), _p(n_active), n_chunks, k, _p(y), _stream(stream)),
           "blockffn_sparse_ffn_static")


def blockffn_dense_ffn(layer: Layer, x, scores, n_chunks: int, k: int, y, workspace: torch.Tensor,
                       chunk_layer=None, stream=None):
    _check(lib().blockffn_dense_ffn(layer.ref(), _p(chunk_layer), _p(x), _p(scores), n_chunks, k, _p(y),
                                    _p(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "blockffn_dense_ffn")


def blockffn_force_generic(mode: int):
    """1: every later FFN call on the shape-generic kernels; 0: automatic choice; -1: as the environment says."""
    _check(lib().blockffn_force_generic(int(mode)), "blockffn_force_generic")


def blockffn_stream_read(buf: torch.Tensor, variant: int, sink: torch.Tensor, stream=None):
    """Plain read stream over the whole of ``buf`` (measurement helper)."""
    _check(lib().blockffn_stream_read(_p(buf), buf.numel() * buf.element_size(), variant, _p(sink), _stream(stream)),
           "blockffn_stream_read")


def blockffn_sparse_ffn_up(layer: Layer, x, scores, token_mask, active_idx, n_active, n_chunks: int, k: int,
                           workspace: torch.Tensor, chunk_layer=None, stream=None):
    _check(lib().blockffn_sparse_ffn_up(layer.ref(), _p(chunk_layer), _p(x), _p(scores), _p(token_mask),
                                        _p(active_idx), _p(n_active), n_chunks, k, _p(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)),
           "blockffn_sparse_ffn_up")


def blockffn_sparse_ffn_down(layer: Layer, active_idx, n_active, n_chunks: int, k: int, y, workspace: torch.Tensor,
                             chunk_layer=None, stream=None):
    _check(lib().blockffn_sparse_ffn_down(layer.ref(), _p(chunk_layer), _p(active_idx), _p(n_active), n_chunks, k,
                                          _p(y), _p(workspace), workspace.numel() * workspace.element_size(),
                                          _stream(stream)), "blockffn_sparse_ffn_down")


class Buffers:
    """Device buffers for one batch shape: outputs of the three stages and the workspace."""

    def __init__(self, layer: Layer, n_chunks: int, k: int):
        dev, T = layer.device, n_chunks * k
        self.n_chunks, self.k = n_chunks, k
        self.scores = torch.empty((T, layer.E), dtype=torch.float32, device=dev)
        self.token_mask = torch.empty((T, layer.W), dtype=torch.int64, device=dev)
        self.union_mask = torch.empty((n_chunks, layer.W), dtype=torch.int64, device=dev)
        self.active_idx = torch.empty((n_chunks, layer.E), dtype=torch.int32, device=dev)
        self.n_active = torch.empty((n_chunks,), dtype=torch.int32, device=dev)
        self.stats = torch.zeros((2,), dtype=torch.int64, device=dev)
        self.y = torch.empty((T, layer.d), dtype=torch.float32, device=dev)
        nbytes = max(blockffn_workspace_bytes(layer, n_chunks, k), 256)
        self.workspace = torch.empty((nbytes,), dtype=torch.uint8, device=dev)


def blockffn_forward_chunks(layer: Layer, x: torch.Tensor, n_chunks: int, k: int, scores, token_mask, union_mask,
                            active_idx, n_active, stats, y, workspace: torch.Tensor, chunk_layer=None, stream=None):
    """Router, chunk union and chunk-sparse FFN as ONE call of the library (three launches for a
    handful of short chunks, the three stages as they are otherwise)."""
    _check(lib().blockffn_forward_chunks(layer.ref(), _p(chunk_layer), _p(x), n_chunks, k, _p(scores), _p(token_mask),
                                         _p(union_mask), _p(active_idx), _p(n_active), _p(stats), _p(y), _p(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "blockffn_forward_chunks")


def forward_chunks(layer: Layer, x: torch.Tensor, buf: Buffers, chunk_layer=None, stream=None):
    """Router -> chunk union -> chunk-sparse FFN: three enqueues on one stream, nothing else."""
    C, k = buf.n_chunks, buf.k
    blockffn_router(layer, x, C, k, buf.scores, buf.token_mask, chunk_layer, stream)
    blockffn_chunk_union(buf.token_mask, C, k, layer.E, buf.union_mask, buf.active_idx, buf.n_active, buf.stats,
                         stream)
    blockffn_sparse_ffn(layer, x, buf.scores, buf.token_mask, buf.active_idx, buf.n_active, C, k, buf.y,
                        buf.workspace, chunk_layer, stream)
    return buf.y
