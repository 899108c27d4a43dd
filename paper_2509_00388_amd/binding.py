"""Thin ctypes binding of libgraphkv.so (include/graphkv.h).

Argument marshalling only: every step of the pass runs in the library's HIP
kernels.  PyTorch supplies device memory and the current stream, nothing else.
There is no fallback: if the library is missing or the GPU is absent the calls
raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgraphkv.so")

FP32, BF16 = 0, 1
POOL_AVG, POOL_MAX = 0, 1
SIGNAL_DECAY, SIGNAL_ENHANCED, SIGNAL_EVICTED = 0, 1, 2
IMPL_AUTO, IMPL_GENERIC = 0, 1
EDGES_KK, EDGES_KV, EDGES_VV = 0, 1, 2
SCORER_ATTENTION, SCORER_KNORM = 0, 1

EXPORTS = ("graphkv_workspace_bytes", "graphkv_score", "graphkv_score_knorm", "graphkv_propagate",
           "graphkv_select", "graphkv_compress", "graphkv_strerror", "graphkv_uses_mfma",
           "graphkv_profile_begin", "graphkv_profile_end", "graphkv_kernel_name",
           "graphkv_workspace_bytes_batched", "graphkv_compress_batched", "graphkv_propagate_edges",
           "graphkv_compress_static")
STATIC_SCRATCH_BYTES = 64 << 20
N_KERNELS = 23


class GraphKVError(RuntimeError):
    pass


class _CParams(ctypes.Structure):
    _fields_ = [
        ("n_kv_heads", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("n_tokens", ctypes.c_int32), ("window", ctypes.c_int32),
        ("pool_kernel", ctypes.c_int32), ("pool_mode", ctypes.c_int32),
        ("budget", ctypes.c_int32),
        ("n_sources", ctypes.c_int32), ("n_neighbors", ctypes.c_int32), ("rounds", ctypes.c_int32),
        ("decay", ctypes.c_float), ("reselect", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("signal", ctypes.c_int32), ("impl", ctypes.c_int32),
        ("edges", ctypes.c_int32), ("scorer", ctypes.c_int32),
    ]


@dataclass
class Params:
    """Mirror of graphkv_params (see include/graphkv.h for the constraints)."""
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    n_tokens: int
    window: int
    pool_kernel: int = 1
    pool_mode: int = POOL_AVG
    budget: int = 0
    n_sources: int = 0
    n_neighbors: int = 0
    rounds: int = 0
    decay: float = 1.0
    reselect: int = 1
    dtype: int = BF16
    softmax_scale: float = 0.0
    signal: int = SIGNAL_DECAY
    impl: int = IMPL_AUTO
    edges: int = EDGES_KK
    scorer: int = SCORER_ATTENTION

    @property
    def n_prefix(self) -> int:
        return self.n_tokens - self.window

    def c(self) -> _CParams:
        return _CParams(*(getattr(self, f[0]) for f in _CParams._fields_))

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == FP32 else torch.bfloat16


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libgraphkv.so built by paper_2509_00388_amd/build.py; raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise GraphKVError(f"{LIB_PATH} is missing: run `python -m paper_2509_00388_amd.build` "
                           "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    pp = ctypes.POINTER(_CParams)
    lib.graphkv_workspace_bytes.restype = sz
    lib.graphkv_workspace_bytes.argtypes = [pp]
    lib.graphkv_uses_mfma.restype = i32
    lib.graphkv_uses_mfma.argtypes = [pp]
    lib.graphkv_score.restype = i32
    lib.graphkv_score.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.graphkv_score_knorm.restype = i32
    lib.graphkv_score_knorm.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.graphkv_propagate.restype = i32
    lib.graphkv_propagate.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.graphkv_propagate_edges.restype = i32
    lib.graphkv_propagate_edges.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.graphkv_select.restype = i32
    lib.graphkv_select.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.graphkv_compress.restype = i32
    lib.graphkv_compress.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.graphkv_compress_static.restype = i32
    lib.graphkv_compress_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.graphkv_workspace_bytes_batched.restype = sz
    lib.graphkv_workspace_bytes_batched.argtypes = [pp, i32]
    lib.graphkv_compress_batched.restype = i32
    lib.graphkv_compress_batched.argtypes = [pp, i32, ctypes.POINTER(i32), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.graphkv_strerror.restype = ctypes.c_char_p
    lib.graphkv_strerror.argtypes = [i32]
    lib.graphkv_profile_begin.restype = i32
    lib.graphkv_profile_begin.argtypes = []
    lib.graphkv_profile_end.restype = i32
    lib.graphkv_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.graphkv_kernel_name.restype = ctypes.c_char_p
    lib.graphkv_kernel_name.argtypes = [i32]
    _lib = lib
    return lib


def graphkv_strerror(code: int) -> str:
    return load_library().graphkv_strerror(code).decode()


def _check(rc: int):
    if rc != 0:
        raise GraphKVError(f"graphkv error {rc}: {graphkv_strerror(rc)}")


def _arg(t: Optional[torch.Tensor], name: str, dtype, numel: int, optional: bool = False):
    """Device address of a tensor argument after checking what the library itself cannot see:
    that it lives on the GPU, is contiguous, has the element type the call expects and holds at
    least `numel` elements (a short or mistyped buffer would make the kernels read or write out
    of bounds)."""
    if t is None:
        if optional:
            return None
        raise GraphKVError(f"{name} is required")
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise GraphKVError(f"{name} must be a contiguous device tensor")
    if t.dtype != dtype:
        raise GraphKVError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if t.numel() < numel:
        raise GraphKVError(f"{name} holds {t.numel()} elements, the call needs {numel}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def graphkv_workspace_bytes(p: Params) -> int:
    cp = p.c()
    return int(load_library().graphkv_workspace_bytes(ctypes.byref(cp)))


def graphkv_uses_mfma(p: Params) -> bool:
    cp = p.c()
    return bool(load_library().graphkv_uses_mfma(ctypes.byref(cp)))


def alloc_workspace(p: Params, device="cuda") -> torch.Tensor:
    n = graphkv_workspace_bytes(p)
    if n == 0:
        raise GraphKVError("invalid params: workspace size is 0")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _ws(p: Params, ws, device, n_layers: int = 0):
    """(address, bytes) of the workspace: the caller's, or a fresh one of the right size."""
    need = graphkv_workspace_bytes_batched(p, n_layers) if n_layers else graphkv_workspace_bytes(p)
    if need == 0:
        raise GraphKVError("invalid params: workspace size is 0")
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return _arg(ws, "ws", torch.uint8, need), ws.numel(), ws


def _kv_numel(p: Params, layers: int = 1) -> int:
    return layers * p.n_kv_heads * p.n_tokens * p.head_dim


def _q_numel(p: Params, layers: int = 1) -> int:
    return layers * p.n_q_heads * p.window * p.head_dim


def _dbg_args(p: Params, dbg_src, dbg_nbr, dbg_e):
    T, n_src = max(p.rounds, 0), p.n_kv_heads * p.n_sources
    return (_arg(dbg_src, "dbg_src", torch.int32, T * n_src, optional=True),
            _arg(dbg_nbr, "dbg_nbr", torch.int32, T * n_src * p.n_neighbors, optional=True),
            _arg(dbg_e, "dbg_e", torch.float32, T * n_src * p.n_neighbors, optional=True))


def graphkv_score(p: Params, Kc, Qw, scores=None, ws=None):
    """scores [H_kv, P] fp32 (allocated if None).  Stage I."""
    if scores is None:
        scores = torch.empty((p.n_kv_heads, p.n_prefix), dtype=torch.float32, device=Kc.device)
    wp, wn, ws = _ws(p, ws, Kc.device)
    cp = p.c()
    _check(load_library().graphkv_score(
        ctypes.byref(cp), _arg(Kc, "Kc", p.torch_dtype, _kv_numel(p)), _arg(Qw, "Qw", p.torch_dtype, _q_numel(p)),
        _arg(scores, "scores", torch.float32, p.n_kv_heads * p.n_prefix), wp, wn, _stream()))
    return scores


def graphkv_score_knorm(p: Params, Kc, scores=None, ws=None):
    if scores is None:
        scores = torch.empty((p.n_kv_heads, p.n_prefix), dtype=torch.float32, device=Kc.device)
    cp = p.c()
    _check(load_library().graphkv_score_knorm(
        ctypes.byref(cp), _arg(Kc, "Kc", p.torch_dtype, _kv_numel(p)),
        _arg(scores, "scores", torch.float32, p.n_kv_heads * p.n_prefix),
        _arg(ws, "ws", torch.uint8, 0, optional=True), ws.numel() if ws is not None else 0, _stream()))
    return scores


def graphkv_propagate(p: Params, Kc, scores, dbg_src=None, dbg_nbr=None, dbg_e=None, ws=None):
    """Refines `scores` [H_kv, P] fp32 in place.  Stages II and III."""
    wp, wn, ws = _ws(p, ws, Kc.device)
    cp = p.c()
    _check(load_library().graphkv_propagate(
        ctypes.byref(cp), _arg(Kc, "Kc", p.torch_dtype, _kv_numel(p)),
        _arg(scores, "scores", torch.float32, p.n_kv_heads * p.n_prefix),
        *_dbg_args(p, dbg_src, dbg_nbr, dbg_e), wp, wn, _stream()))
    return scores


def graphkv_propagate_edges(p: Params, Ac, Bc, scores, dbg_src=None, dbg_nbr=None, dbg_e=None, ws=None):
    """The same rounds with edges cos(Ac[h, i], Bc[h, j]) (source's row from Ac)."""
    wp, wn, ws = _ws(p, ws, Ac.device)
    cp = p.c()
    _check(load_library().graphkv_propagate_edges(
        ctypes.byref(cp), _arg(Ac, "Ac", p.torch_dtype, _kv_numel(p)), _arg(Bc, "Bc", p.torch_dtype, _kv_numel(p)),
        _arg(scores, "scores", torch.float32, p.n_kv_heads * p.n_prefix),
        *_dbg_args(p, dbg_src, dbg_nbr, dbg_e), wp, wn, _stream()))
    return scores


def graphkv_select(p: Params, scores, idx=None, ws=None):
    """idx [H_kv, B] int32.  Stage IV, selection."""
    if idx is None:
        idx = torch.empty((p.n_kv_heads, p.budget), dtype=torch.int32, device=scores.device)
    cp = p.c()
    _check(load_library().graphkv_select(
        ctypes.byref(cp), _arg(scores, "scores", torch.float32, p.n_kv_heads * p.n_prefix),
        _arg(idx, "idx", torch.int32, p.n_kv_heads * max(p.budget, 0)),
        _arg(ws, "ws", torch.uint8, 0, optional=True), ws.numel() if ws is not None else 0, _stream()))
    return idx


def graphkv_compress(p: Params, Kc, Vc, Qw, Kout=None, Vout=None, idx=None, scores_out=None, ws=None):
    """The whole pass for one layer.  Returns (Kout, Vout, idx).  Qw may be None with
    scorer = SCORER_KNORM."""
    dev = Kc.device
    shape = (p.n_kv_heads, p.budget, p.head_dim)
    if Kout is None:
        Kout = torch.empty(shape, dtype=Kc.dtype, device=dev)
    if Vout is None:
        Vout = torch.empty(shape, dtype=Vc.dtype, device=dev)
    if idx is None:
        idx = torch.empty((p.n_kv_heads, p.budget), dtype=torch.int32, device=dev)
    wp, wn, ws = _ws(p, ws, dev)
    cp = p.c()
    n_out = p.n_kv_heads * max(p.budget, 0)
    knorm = p.scorer == SCORER_KNORM
    _check(load_library().graphkv_compress(
        ctypes.byref(cp), _arg(Kc, "Kc", p.torch_dtype, _kv_numel(p)), _arg(Vc, "Vc", p.torch_dtype, _kv_numel(p)),
        _arg(Qw, "Qw", p.torch_dtype, 0 if knorm else _q_numel(p), optional=knorm),
        _arg(Kout, "Kout", p.torch_dtype, n_out * p.head_dim), _arg(Vout, "Vout", p.torch_dtype, n_out * p.head_dim),
        _arg(idx, "idx", torch.int32, n_out),
        _arg(scores_out, "scores_out", torch.float32, p.n_kv_heads * p.n_prefix, optional=True),
        wp, wn, _stream()))
    return Kout, Vout, idx


def graphkv_compress_static(p: Params, Kc, Vc, Qw, Kout, Vout, idx, scores_out=None):
    """graphkv_compress on the library's built-in scratch buffer: no workspace, nothing is
    allocated here or in the library (the caller passes every output)."""
    cp = p.c()
    n_out = p.n_kv_heads * max(p.budget, 0)
    knorm = p.scorer == SCORER_KNORM
    _check(load_library().graphkv_compress_static(
        ctypes.byref(cp), _arg(Kc, "Kc", p.torch_dtype, _kv_numel(p)), _arg(Vc, "Vc", p.torch_dtype, _kv_numel(p)),
        _arg(Qw, "Qw", p.torch_dtype, 0 if knorm else _q_numel(p), optional=knorm),
        _arg(Kout, "Kout", p.torch_dtype, n_out * p.head_dim), _arg(Vout, "Vout", p.torch_dtype, n_out * p.head_dim),
        _arg(idx, "idx", torch.int32, n_out),
        _arg(scores_out, "scores_out", torch.float32, p.n_kv_heads * p.n_prefix, optional=True), _stream()))
    return Kout, Vout, idx


def graphkv_workspace_bytes_batched(p: Params, n_layers: int) -> int:
    cp = p.c()
    return int(load_library().graphkv_workspace_bytes_batched(ctypes.byref(cp), n_layers))


def graphkv_compress_batched(p: Params, n_layers: int, budgets, Kc, Vc, Qw, Kout=None, Vout=None,
                             idx=None, scores_out=None, ws=None):
    """The whole pass for n_layers contiguous layers: Kc, Vc [L, H_kv, N, d], Qw [L, H_q, w, d].
    budgets: per-layer budgets (sequence of ints) or None for p.budget everywhere.  Outputs are
    packed layer after layer: Kout, Vout [sum_l H_kv * B_l, d], idx [sum_l H_kv * B_l].
    Returns (Kout, Vout, idx)."""
    dev = Kc.device
    bl = [int(b) for b in budgets] if budgets is not None else [p.budget] * n_layers
    if len(bl) != n_layers or n_layers < 1:
        raise GraphKVError("one budget per layer is required")
    rows = p.n_kv_heads * sum(max(b, 0) for b in bl)
    if Kout is None:
        Kout = torch.empty((rows, p.head_dim), dtype=Kc.dtype, device=dev)
    if Vout is None:
        Vout = torch.empty((rows, p.head_dim), dtype=Vc.dtype, device=dev)
    if idx is None:
        idx = torch.empty((rows,), dtype=torch.int32, device=dev)
    wp, wn, ws = _ws(p, ws, dev, n_layers)
    cp = p.c()
    carr = (ctypes.c_int32 * n_layers)(*bl) if budgets is not None else None
    knorm = p.scorer == SCORER_KNORM
    _check(load_library().graphkv_compress_batched(
        ctypes.byref(cp), n_layers, carr,
        _arg(Kc, "Kc", p.torch_dtype, _kv_numel(p, n_layers)), _arg(Vc, "Vc", p.torch_dtype, _kv_numel(p, n_layers)),
        _arg(Qw, "Qw", p.torch_dtype, 0 if knorm else _q_numel(p, n_layers), optional=knorm),
        _arg(Kout, "Kout", p.torch_dtype, rows * p.head_dim), _arg(Vout, "Vout", p.torch_dtype, rows * p.head_dim),
        _arg(idx, "idx", torch.int32, rows),
        _arg(scores_out, "scores_out", torch.float32, n_layers * p.n_kv_heads * p.n_prefix, optional=True),
        wp, wn, _stream()))
    return Kout, Vout, idx


def graphkv_profile_begin():
    _check(load_library().graphkv_profile_begin())


def graphkv_profile_end():
    """{kernel name: (total ms, launches)} for the kernels launched since profile_begin."""
    ms = (ctypes.c_double * N_KERNELS)()
    cnt = (ctypes.c_int64 * N_KERNELS)()
    _check(load_library().graphkv_profile_end(ms, cnt))
    lib = load_library()
    return {lib.graphkv_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(N_KERNELS) if cnt[i]}


# ---- helpers to move the synthetic numpy tensors (fp32 / bf16 bits) to the device ----

def to_device(arr, dtype: int, device="cuda") -> torch.Tensor:
    import numpy as np
    if dtype == FP32:
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device)
    return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).to(device).view(torch.bfloat16)


def to_host_bits(t: torch.Tensor):
    """Device tensor -> numpy in the storage convention of synth.py."""
    import numpy as np
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()
