"""ctypes binding of libmixkv (see include/mixkv.h).  Argument marshalling only.

Every function here has the name of the C entry point it calls and does nothing
but build the C structs from torch tensors (device memory and the current HIP
stream come from torch) and check the returned status.  There is no fallback:
if the shared library has not been built, `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmixkv.so")

MIXKV_OK, MIXKV_ERR_INVALID_ARG, MIXKV_ERR_UNSUPPORTED, MIXKV_ERR_WORKSPACE_TOO_SMALL, MIXKV_ERR_HIP = range(5)
DTYPE = {"f32": 0, "bf16": 1}
POOL = {"none": 0, "avg": 1, "max": 2}
BUDGET_MODE = {"fixed": 0, "adaptive": 1, "per_head": 2}
INTRINSIC = {"none": 0, "vnorm": 1, "knorm": 2}
MIX = {"head_adaptive": 0, "sum": 1, "div_only": 2, "imp_only": 3, "given_r": 4}
TORCH_DTYPE = {0: torch.float32, 1: torch.bfloat16}
N_STAGES = 5


class MixkvParams(C.Structure):
    _fields_ = [
        ("dtype", C.c_int), ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("seq_len", C.c_int32), ("window", C.c_int32), ("budget", C.c_int32),
        ("pool", C.c_int), ("pool_kernel", C.c_int32), ("causal_window", C.c_int32),
        ("softmax_scale", C.c_float), ("eps", C.c_float), ("intrinsic", C.c_int), ("mix", C.c_int),
        ("budget_mode", C.c_int), ("budget_floor", C.c_int32), ("head_budgets", C.c_void_p),
    ]


class MixkvLayerIn(C.Structure):
    _fields_ = [("K", C.c_void_p), ("V", C.c_void_p), ("kv_stride_b", C.c_int64), ("kv_stride_h", C.c_int64),
                ("kv_stride_n", C.c_int64), ("Qwin", C.c_void_p), ("r_given", C.c_void_p),
                ("window_lse", C.c_void_p)]


class MixkvLayerOut(C.Structure):
    _fields_ = [("scores", C.c_void_p), ("redundancy", C.c_void_p), ("indices", C.c_void_p), ("counts", C.c_void_p),
                ("offsets", C.c_void_p), ("K_out", C.c_void_p), ("V_out", C.c_void_p)]


class MixkvRowsIn(C.Structure):
    _fields_ = [("X", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_n", C.c_int64)]


class MixkvSimilarityOut(C.Structure):
    _fields_ = [("redundancy", C.c_void_p), ("block_map", C.c_void_p)]


class MixkvDecodeLayer(C.Structure):
    _fields_ = [("K_cache", C.c_void_p), ("V_cache", C.c_void_p), ("counts", C.c_void_p), ("offsets", C.c_void_p),
                ("K_tail", C.c_void_p), ("V_tail", C.c_void_p), ("Q", C.c_void_p), ("out", C.c_void_p)]


class MixkvAppendLayer(C.Structure):
    _fields_ = [("K_new", C.c_void_p), ("V_new", C.c_void_p), ("K_tail", C.c_void_p), ("V_tail", C.c_void_p)]


class MixkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """Load libmixkv.so (built by `python -m paper_2510_20707_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2510_20707_amd.build`")
        L = C.CDLL(LIB_PATH)
        pp, pin, pout = C.POINTER(MixkvParams), C.POINTER(MixkvLayerIn), C.POINTER(MixkvLayerOut)
        L.mixkv_workspace_size.argtypes = [pp, C.c_int32, C.POINTER(C.c_size_t)]
        L.mixkv_workspace_size.restype = C.c_int
        L.mixkv_score.argtypes = [pp, pin, pout, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixkv_score.restype = C.c_int
        L.mixkv_select.argtypes = [pp, pout, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixkv_select.restype = C.c_int
        L.mixkv_compress.argtypes = [pp, pin, pout, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixkv_compress.restype = C.c_int
        L.mixkv_compress_static.argtypes = [pp, pin, pout, C.c_int32, C.c_void_p]
        L.mixkv_compress_static.restype = C.c_int
        L.mixkv_compress_profiled.argtypes = [pp, pin, pout, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                              C.POINTER(C.c_float)]
        L.mixkv_compress_profiled.restype = C.c_int
        L.mixkv_similarity_workspace_size.argtypes = [pp, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        L.mixkv_similarity_workspace_size.restype = C.c_int
        L.mixkv_similarity.argtypes = [pp, C.POINTER(MixkvRowsIn), C.POINTER(MixkvSimilarityOut), C.c_int32, C.c_int32,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixkv_similarity.restype = C.c_int
        L.mixkv_decode_attention.argtypes = [pp, C.POINTER(MixkvDecodeLayer), C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                             C.c_size_t, C.c_void_p]
        L.mixkv_decode_attention.restype = C.c_int
        L.mixkv_append.argtypes = [pp, C.POINTER(MixkvAppendLayer), C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.mixkv_append.restype = C.c_int
        L.mixkv_decode_workspace_size.argtypes = [pp, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        L.mixkv_decode_workspace_size.restype = C.c_int
        L.mixkv_stage_name.argtypes = [C.c_int32]
        L.mixkv_stage_name.restype = C.c_char_p
        L.mixkv_status_string.argtypes = [C.c_int]
        L.mixkv_status_string.restype = C.c_char_p
        L.mixkv_version.argtypes = []
        L.mixkv_version.restype = C.c_int32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().mixkv_status_string(status).decode()


def make_params(dtype: str, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, seq_len: int, window: int,
                budget: int, pool: str = "max", pool_kernel: int = 7, causal_window: bool = True,
                softmax_scale: float = 1.0, eps: float = 1e-6, intrinsic: str = "vnorm",
                budget_mode: str = "fixed", budget_floor: int = 0, mix: str = "head_adaptive",
                head_budgets=None) -> MixkvParams:
    """`head_budgets`: host int32 array [n_layers, n_kv_heads] for budget mode "per_head"."""
    p = MixkvParams(DTYPE[dtype], batch, n_q_heads, n_kv_heads, head_dim, seq_len, window, budget, POOL[pool],
                    pool_kernel, int(causal_window), softmax_scale, eps, INTRINSIC[intrinsic], MIX[mix],
                    BUDGET_MODE[budget_mode], budget_floor, None)
    if head_budgets is not None:
        hb = np.ascontiguousarray(head_budgets, dtype=np.int32)
        assert hb.ndim == 2 and hb.shape[1] == n_kv_heads
        p._head_budgets_keep = hb                   # the struct only holds the address
        p.head_budgets = hb.ctypes.data
    return p


@dataclass
class LayerOut:
    """Device tensors receiving one layer's outputs; members may be None where the C API allows NULL."""
    scores: Optional[torch.Tensor] = None        # [batch, Hkv, N] f32
    redundancy: Optional[torch.Tensor] = None    # [batch, Hkv] f32
    indices: Optional[torch.Tensor] = None       # [batch, Hkv, B] i32 (adaptive: packed per batch item)
    counts: Optional[torch.Tensor] = None        # [batch, Hkv] i32
    offsets: Optional[torch.Tensor] = None       # [batch, Hkv + 1] i32
    K_out: Optional[torch.Tensor] = None         # [batch, Hkv, B, D]
    V_out: Optional[torch.Tensor] = None


def alloc_layer_out(p: MixkvParams, device, scores=True, redundancy=True, select=True, gather=True) -> LayerOut:
    """Allocate one layer's outputs with torch (plumbing for tests and the benchmark)."""
    o = LayerOut()
    bt, h, n, b, d = p.batch, p.n_kv_heads, p.seq_len, p.budget, p.head_dim
    if scores:
        o.scores = torch.empty((bt, h, n), dtype=torch.float32, device=device)
    if redundancy:
        o.redundancy = torch.empty((bt, h), dtype=torch.float32, device=device)
    if select:
        o.indices = torch.empty((bt, h, b), dtype=torch.int32, device=device)
        o.counts = torch.empty((bt, h), dtype=torch.int32, device=device)
        o.offsets = torch.empty((bt, h + 1), dtype=torch.int32, device=device)
    if gather:
        o.K_out = torch.empty((bt, h, b, d), dtype=TORCH_DTYPE[p.dtype], device=device)
        o.V_out = torch.empty((bt, h, b, d), dtype=TORCH_DTYPE[p.dtype], device=device)
    return o


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _in_array(Ks, Vs, Qs, r_given=None, window_lse=None):
    """r_given: per layer a contiguous f32 [batch, Hkv] device tensor (mix "given_r"), or None;
    window_lse: per layer a contiguous f32 [batch, Hq, W] device tensor, or None."""
    n = len(Ks)
    arr = (MixkvLayerIn * n)()
    for i, (K, V, Q) in enumerate(zip(Ks, Vs, Qs)):
        assert K.dim() == 4 and K.stride(3) == 1 and V.shape == K.shape and V.stride() == K.stride()
        assert Q is None or Q.is_contiguous()
        rg = None if r_given is None else r_given[i]
        assert rg is None or (rg.is_contiguous() and rg.dtype == torch.float32 and rg.shape == K.shape[:2])
        lse = None if window_lse is None else window_lse[i]
        assert lse is None or (lse.is_contiguous() and lse.dtype == torch.float32 and lse.shape == Q.shape[:3])
        arr[i] = MixkvLayerIn(K.data_ptr(), V.data_ptr(), K.stride(0), K.stride(1), K.stride(2),
                              None if Q is None else Q.data_ptr(), None if rg is None else rg.data_ptr(),
                              None if lse is None else lse.data_ptr())
    return arr


def _out_array(outs: Sequence[LayerOut]):
    arr = (MixkvLayerOut * len(outs))()
    for i, o in enumerate(outs):
        arr[i] = MixkvLayerOut(_ptr(o.scores), _ptr(o.redundancy), _ptr(o.indices), _ptr(o.counts), _ptr(o.offsets),
                               _ptr(o.K_out), _ptr(o.V_out))
    return arr


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(status: int, where: str):
    if status != MIXKV_OK:
        raise MixkvError(status, where)


def mixkv_workspace_size(p: MixkvParams, n_layers: int) -> int:
    n = C.c_size_t(0)
    _check(lib().mixkv_workspace_size(C.byref(p), n_layers, C.byref(n)), "mixkv_workspace_size")
    return n.value


def alloc_workspace(p: MixkvParams, n_layers: int, device) -> torch.Tensor:
    return torch.empty(mixkv_workspace_size(p, n_layers), dtype=torch.uint8, device=device)


def _ws(workspace: Optional[torch.Tensor]):
    if workspace is None:
        return None, 0
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def mixkv_score(p: MixkvParams, Ks, Vs, Qs, outs: Sequence[LayerOut], workspace: torch.Tensor, stream=None,
                r_given=None, window_lse=None):
    wp, wb = _ws(workspace)
    _check(lib().mixkv_score(C.byref(p), _in_array(Ks, Vs, Qs, r_given, window_lse), _out_array(outs), len(outs), wp, wb, _stream(stream)),
           "mixkv_score")


def mixkv_select(p: MixkvParams, outs: Sequence[LayerOut], workspace: Optional[torch.Tensor] = None, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().mixkv_select(C.byref(p), _out_array(outs), len(outs), wp, wb, _stream(stream)), "mixkv_select")


def mixkv_compress(p: MixkvParams, Ks, Vs, Qs, outs: Sequence[LayerOut], workspace: torch.Tensor, stream=None,
                   r_given=None, window_lse=None):
    wp, wb = _ws(workspace)
    _check(lib().mixkv_compress(C.byref(p), _in_array(Ks, Vs, Qs, r_given, window_lse), _out_array(outs), len(outs), wp, wb,
                                _stream(stream)), "mixkv_compress")


STATIC_SCRATCH_BYTES = 32 << 20


def mixkv_compress_static(p: MixkvParams, Ks, Vs, Qs, outs: Sequence[LayerOut], stream=None, r_given=None, window_lse=None):
    """mixkv_compress on the library's own static workspace (no workspace argument, no allocation)."""
    _check(lib().mixkv_compress_static(C.byref(p), _in_array(Ks, Vs, Qs, r_given, window_lse), _out_array(outs), len(outs),
                                       _stream(stream)), "mixkv_compress_static")


def mixkv_similarity_workspace_size(p: MixkvParams, n_layers: int, block: int) -> int:
    n = C.c_size_t(0)
    _check(lib().mixkv_similarity_workspace_size(C.byref(p), n_layers, block, C.byref(n)),
           "mixkv_similarity_workspace_size")
    return n.value


class PreparedSimilarity:
    """The C argument arrays of one mixkv_similarity call, built once."""

    def __init__(self, p: MixkvParams, Xs, redundancy, block_maps, block: int, workspace: torch.Tensor):
        n = len(Xs)
        self.p, self.n, self.block = p, n, block
        self.ins, self.outs = (MixkvRowsIn * n)(), (MixkvSimilarityOut * n)()
        for i, X in enumerate(Xs):
            assert X.dim() == 4 and X.stride(3) == 1
            self.ins[i] = MixkvRowsIn(X.data_ptr(), X.stride(0), X.stride(1), X.stride(2))
            self.outs[i] = MixkvSimilarityOut(_ptr(None if redundancy is None else redundancy[i]),
                                              _ptr(None if block_maps is None else block_maps[i]))
        self.wp, self.wb = _ws(workspace)
        self._keep = (Xs, redundancy, block_maps, workspace)
        self._L = lib()

    def run(self, stream=None):
        _check(self._L.mixkv_similarity(C.byref(self.p), self.ins, self.outs, self.n, self.block, self.wp, self.wb,
                                        _stream(stream)), "mixkv_similarity")


def mixkv_similarity(p: MixkvParams, Xs, block: int, want_map: bool = True, workspace=None, stream=None):
    """Redundancy and (optionally) the block-mean similarity heat-map of every head of the layers Xs
    ([batch, Hkv, N, D] device tensors: keys or values).  Returns (redundancy list, block_map list)."""
    dev = Xs[0].device
    nb = (p.seq_len + block - 1) // block
    red = [torch.empty((p.batch, p.n_kv_heads), dtype=torch.float32, device=dev) for _ in Xs]
    maps = [torch.empty((p.batch, p.n_kv_heads, nb, nb), dtype=torch.float32, device=dev) for _ in Xs] if want_map else None
    if workspace is None:
        workspace = torch.empty(mixkv_similarity_workspace_size(p, len(Xs), block), dtype=torch.uint8, device=dev)
    PreparedSimilarity(p, Xs, red, maps, block, workspace).run(stream)
    return red, maps


class PreparedDecode:
    """The C argument array of one mixkv_decode_attention call, built once.

    caches: per layer a LayerOut as filled by mixkv_compress; tails: per layer (K_tail, V_tail)
    [batch, Hkv, tail_capacity, D] or None; Qs / outs: per layer [batch, Hq, D]."""

    def __init__(self, p: MixkvParams, caches: Sequence[LayerOut], tails, Qs, outs, tail_len: int, workspace="alloc"):
        n = len(caches)
        if isinstance(workspace, str):                # allocate what the shape needs (possibly nothing)
            need = mixkv_decode_workspace_size(p, n, tail_len)
            workspace = torch.empty(need, dtype=torch.uint8, device=Qs[0].device) if need else None
        self.wp, self.wb = _ws(workspace)
        self._ws_keep = workspace
        self.p, self.n, self.tail_len = p, n, tail_len
        self.tail_cap = 0 if tails is None else tails[0][0].shape[2]
        self.arr = (MixkvDecodeLayer * n)()
        for i, c in enumerate(caches):
            kt, vt = (None, None) if tails is None else tails[i]
            assert Qs[i].is_contiguous() and outs[i].is_contiguous() and (kt is None or kt.is_contiguous())
            self.arr[i] = MixkvDecodeLayer(_ptr(c.K_out), _ptr(c.V_out), _ptr(c.counts), _ptr(c.offsets), _ptr(kt), _ptr(vt),
                                           _ptr(Qs[i]), _ptr(outs[i]))
        self._keep = (caches, tails, Qs, outs)
        self._L = lib()

    def run(self, stream=None):
        _check(self._L.mixkv_decode_attention(C.byref(self.p), self.arr, self.n, self.tail_len, self.tail_cap,
                                              self.wp, self.wb, _stream(stream)), "mixkv_decode_attention")


def mixkv_decode_workspace_size(p: MixkvParams, n_layers: int, tail_len: int) -> int:
    n = C.c_size_t(0)
    _check(lib().mixkv_decode_workspace_size(C.byref(p), n_layers, tail_len, C.byref(n)), "mixkv_decode_workspace_size")
    return n.value


def mixkv_decode_attention(p: MixkvParams, caches, tails, Qs, tail_len: int, stream=None, workspace="alloc"):
    """Returns per layer the attention output [batch, Hq, D] of the new token (dtype of the inputs)."""
    outs = [torch.empty_like(q) for q in Qs]
    PreparedDecode(p, caches, tails, Qs, outs, tail_len, workspace).run(stream)
    return outs


def mixkv_append(p: MixkvParams, new_rows, tails, position: int, stream=None):
    """Copies per layer the new token's (K_new, V_new) [batch, Hkv, D] into row `position` of the
    layer's (K_tail, V_tail) [batch, Hkv, tail_capacity, D], in place."""
    n = len(tails)
    arr = (MixkvAppendLayer * n)()
    for i, ((kn, vn), (kt, vt)) in enumerate(zip(new_rows, tails)):
        assert kn.is_contiguous() and vn.is_contiguous() and kt.is_contiguous() and vt.is_contiguous()
        arr[i] = MixkvAppendLayer(_ptr(kn), _ptr(vn), _ptr(kt), _ptr(vt))
    _check(lib().mixkv_append(C.byref(p), arr, n, position, tails[0][0].shape[2], _stream(stream)), "mixkv_append")


class PreparedCall:
    """The C argument arrays of one call, built once (so a timed loop measures the library, not ctypes)."""

    def __init__(self, p: MixkvParams, Ks, Vs, Qs, outs: Sequence[LayerOut], workspace: torch.Tensor, r_given=None,
                 window_lse=None):
        self.p, self.n = p, len(outs)
        self.ins, self.outs = _in_array(Ks, Vs, Qs, r_given, window_lse), _out_array(outs)
        self.wp, self.wb = _ws(workspace)
        self._keep = (Ks, Vs, Qs, outs, workspace, r_given, window_lse)
        self._L = lib()

    def compress(self, stream=None):
        _check(self._L.mixkv_compress(C.byref(self.p), self.ins, self.outs, self.n, self.wp, self.wb, _stream(stream)),
               "mixkv_compress")

    def compress_profiled(self, stream=None) -> dict:
        ms = (C.c_float * N_STAGES)()
        _check(self._L.mixkv_compress_profiled(C.byref(self.p), self.ins, self.outs, self.n, self.wp, self.wb,
                                               _stream(stream), ms), "mixkv_compress_profiled")
        return {self._L.mixkv_stage_name(i).decode(): float(ms[i]) for i in range(N_STAGES)}

    def score(self, stream=None):
        _check(self._L.mixkv_score(C.byref(self.p), self.ins, self.outs, self.n, self.wp, self.wb, _stream(stream)),
               "mixkv_score")
