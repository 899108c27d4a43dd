"""ctypes front-end of the CPU oracle (oracle/graphkv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the GPU product imports this package
and this package imports nothing from the GPU product.

All functions take and return numpy arrays.  Stored tensors are float32 arrays
("fp32") or uint16 arrays holding bfloat16 bits ("bf16"); scores are float64.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_DT = {"fp32": 0, "bf16": 1}
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = ctypes.CDLL(path)
        _lib.gkv_oracle_topk.restype = None
        for name in ("gkv_oracle_score", "gkv_oracle_score_knorm", "gkv_oracle_propagate",
                     "gkv_oracle_select", "gkv_oracle_gather", "gkv_oracle_compress"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.gkv_oracle_cosine_row.restype = None
        _lib.gkv_oracle_cosine_row2.restype = None
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _i(x):
    return ctypes.c_int32(int(x))


def _d(x):
    return ctypes.c_double(float(x))


def _check_storage(a: np.ndarray, dtype: str):
    want = np.float32 if dtype == "fp32" else np.uint16
    if a.dtype != want or not a.flags["C_CONTIGUOUS"]:
        raise ValueError(f"expected contiguous {want} for {dtype}, got {a.dtype}")


def topk(x: np.ndarray, k: int, skip: int = -1) -> Tuple[np.ndarray, float]:
    """Indices (ascending) of the k largest entries, ties to the lowest index;
    also the relative gap at the cut."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    idx = np.empty(max(k, 1), dtype=np.int32)
    gap = ctypes.c_double(0.0)
    lib().gkv_oracle_topk(_p(x), _i(x.size), _i(k), _i(skip), _p(idx), ctypes.byref(gap))
    return idx[:k].copy(), gap.value


def score(Kc, Qw, dtype: str, pool_kernel: int, pool_mode: int = 0, scale: float = 0.0,
          want_votes: bool = False):
    _check_storage(Kc, dtype); _check_storage(Qw, dtype)
    Hkv, N, d = Kc.shape
    Hq, w, _ = Qw.shape
    P = N - w
    s = np.empty((Hkv, P), dtype=np.float64)
    votes = np.empty((Hq, P), dtype=np.float64) if want_votes else None
    rc = lib().gkv_oracle_score(_p(Kc), _p(Qw), _i(_DT[dtype]), _i(Hkv), _i(Hq), _i(d), _i(N),
                                _i(w), _i(pool_kernel), _i(pool_mode), _d(scale), _p(s), _p(votes))
    if rc:
        raise ValueError("gkv_oracle_score rejected the arguments")
    return (s, votes) if want_votes else s


def score_knorm(Kc, dtype: str, window: int) -> np.ndarray:
    _check_storage(Kc, dtype)
    Hkv, N, d = Kc.shape
    s = np.empty((Hkv, N - window), dtype=np.float64)
    rc = lib().gkv_oracle_score_knorm(_p(Kc), _i(_DT[dtype]), _i(Hkv), _i(d), _i(N), _i(window), _p(s))
    if rc:
        raise ValueError("gkv_oracle_score_knorm rejected the arguments")
    return s


def cosine_row(Kc, dtype: str, window: int, h: int, i: int, other=None) -> np.ndarray:
    """Edges of source i of head h to every prefix node (Eq. 1); with `other` the
    other node's row is taken from that tensor instead of Kc."""
    _check_storage(Kc, dtype)
    other = Kc if other is None else other
    _check_storage(other, dtype)
    Hkv, N, d = Kc.shape
    P = N - window
    e = np.empty(P, dtype=np.float64)
    lib().gkv_oracle_cosine_row2(_p(Kc), _p(other), _i(_DT[dtype]), _i(d), _i(N), _i(P), _i(h), _i(i),
                                 _p(e))
    return e


def propagate(Kc, dtype: str, window: int, s: np.ndarray, S: int, m: int, T: int,
              alpha: float = 1.0, reselect: int = 1, signal: int = 0,
              forced_src: Optional[np.ndarray] = None, debug: bool = False):
    """Key-to-key edges (Eq. 1).  Returns the refined scores (a new float64 array); with
    debug=True also a dict with src [T,H,S], nbr [T,H,S,m], e [T,H,S,m], gap_src [T,H],
    gap_nbr [T,H,S]."""
    return propagate_edges(Kc, Kc, dtype, window, s, S, m, T, alpha, reselect, signal,
                           forced_src, debug)


def propagate_edges(A, Bm, dtype: str, window: int, s: np.ndarray, S: int, m: int, T: int,
                    alpha: float = 1.0, reselect: int = 1, signal: int = 0,
                    forced_src: Optional[np.ndarray] = None, debug: bool = False):
    """Edges e_ij = cos(A[h,i,:], Bm[h,j,:]): the source's feature from A, the other
    node's from Bm (the Discussion's other pairings).  Same returns as propagate."""
    _check_storage(A, dtype); _check_storage(Bm, dtype)
    assert A.shape == Bm.shape
    Kc = A
    Hkv, N, d = Kc.shape
    P = N - window
    s = np.array(s, dtype=np.float64, order="C", copy=True)
    assert s.shape == (Hkv, P)
    Tn = max(T, 1)
    dbg = None
    if debug:
        dbg = dict(src=np.zeros((Tn, Hkv, S), np.int32), nbr=np.zeros((Tn, Hkv, S, m), np.int32),
                   e=np.zeros((Tn, Hkv, S, m), np.float64), gap_src=np.full((Tn, Hkv), np.inf),
                   gap_nbr=np.full((Tn, Hkv, S), np.inf))
    if forced_src is not None:
        forced_src = np.ascontiguousarray(forced_src, dtype=np.int32)
        assert forced_src.shape == (T, Hkv, S)
    rc = lib().gkv_oracle_propagate_edges(
        _p(A), _p(Bm), _i(_DT[dtype]), _i(Hkv), _i(d), _i(N), _i(window), _i(S), _i(m), _i(T),
        _d(alpha), _i(reselect), _i(signal), _p(s), _p(forced_src),
        _p(dbg["src"]) if dbg else _p(None), _p(dbg["nbr"]) if dbg else _p(None),
        _p(dbg["e"]) if dbg else _p(None), _p(dbg["gap_src"]) if dbg else _p(None),
        _p(dbg["gap_nbr"]) if dbg else _p(None))
    if rc:
        raise ValueError("gkv_oracle_propagate_edges rejected the arguments")
    if debug:
        for k in dbg:
            dbg[k] = dbg[k][:T]
        return s, dbg
    return s


def select(s: np.ndarray, n_tokens: int, window: int, budget: int):
    """idx [H,B] int32 (ascending prefix picks, then the window) and gap [H]."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    Hkv = s.shape[0]
    idx = np.empty((Hkv, budget), dtype=np.int32)
    gap = np.empty(Hkv, dtype=np.float64)
    rc = lib().gkv_oracle_select(_p(s), _i(Hkv), _i(n_tokens), _i(window), _i(budget), _p(idx), _p(gap))
    if rc:
        raise ValueError("gkv_oracle_select rejected the arguments")
    return idx, gap


def gather(Kc, Vc, dtype: str, idx: np.ndarray):
    _check_storage(Kc, dtype); _check_storage(Vc, dtype)
    Hkv, N, d = Kc.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    B = idx.shape[1]
    Kout = np.empty((Hkv, B, d), dtype=Kc.dtype)
    Vout = np.empty((Hkv, B, d), dtype=Vc.dtype)
    rc = lib().gkv_oracle_gather(_p(Kc), _p(Vc), _i(_DT[dtype]), _i(Hkv), _i(d), _i(N), _i(B),
                                 _p(idx), _p(Kout), _p(Vout))
    if rc:
        raise ValueError("gkv_oracle_gather: index out of range")
    return Kout, Vout


def compress(Kc, Vc, Qw, dtype: str, pool_kernel: int, budget: int, S: int, m: int, T: int,
             alpha: float = 1.0, reselect: int = 1, signal: int = 0, pool_mode: int = 0,
             scale: float = 0.0, edge_mode: int = 0, scorer: int = 0, window: Optional[int] = None):
    """The whole pass for one layer.  Returns a dict: Kout, Vout, idx, scores (s^(T),
    float64), s0 (float64); what was picked per round, src [T,H,S] and nbr [T,H,S,m]; the
    relative gap at every cut, gap_src [T,H], gap_nbr [T,H,S], gap_final [H]; and min_gap =
    their minima (source cut, neighbour cut, final cut).
    edge_mode: 0 key-key edges, 1 key-value, 2 value-value.
    scorer: 0 observation-window attention score, 1 KNorm (Qw may then be None and
    `window` gives w)."""
    _check_storage(Kc, dtype); _check_storage(Vc, dtype)
    Hkv, N, d = Kc.shape
    if Qw is not None:
        _check_storage(Qw, dtype)
        Hq, w, _ = Qw.shape
    elif scorer == 1 and window is not None:
        Hq, w = Hkv, int(window)          # KNorm reads no queries
    else:
        raise ValueError("Qw is required unless scorer=1 and window is given")
    P = N - w
    Tn = max(T, 1)
    Kout = np.empty((Hkv, budget, d), dtype=Kc.dtype)
    Vout = np.empty((Hkv, budget, d), dtype=Vc.dtype)
    idx = np.empty((Hkv, budget), dtype=np.int32)
    sc = np.empty((Hkv, P), dtype=np.float64)
    s0 = np.empty((Hkv, P), dtype=np.float64)
    src = np.zeros((Tn, Hkv, max(S, 1)), dtype=np.int32)
    nbr = np.zeros((Tn, Hkv, max(S, 1), max(m, 1)), dtype=np.int32)
    gs = np.full((Tn, Hkv), np.inf)
    gn = np.full((Tn, Hkv, max(S, 1)), np.inf)
    gf = np.full(Hkv, np.inf)
    rc = lib().gkv_oracle_compress(
        _p(Kc), _p(Vc), _p(Qw), _i(_DT[dtype]), _i(Hkv), _i(Hq), _i(d), _i(N),
        _i(w), _i(pool_kernel), _i(pool_mode), _d(scale), _i(budget), _i(S), _i(m), _i(T), _d(alpha),
        _i(reselect), _i(signal), _i(edge_mode), _i(scorer), _p(Kout), _p(Vout), _p(idx), _p(sc), _p(s0),
        _p(src), _p(nbr), _p(gs), _p(gn), _p(gf))
    if rc:
        raise ValueError("gkv_oracle_compress rejected the arguments")
    src, nbr, gs, gn = src[:T], nbr[:T], gs[:T], gn[:T]
    mg = np.array([gs.min() if T > 0 else np.inf, gn.min() if T > 0 else np.inf, gf.min()])
    return dict(Kout=Kout, Vout=Vout, idx=idx, scores=sc, s0=s0, src=src, nbr=nbr,
                gap_src=gs, gap_nbr=gn, gap_final=gf, min_gap=mg)
