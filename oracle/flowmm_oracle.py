"""ctypes front end of the fp64 CPU oracle (oracle/flowmm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg, never by the product path.  Argument marshalling only; every
number is computed by the C file, stage by stage, so that a test can feed one
stage's forced inputs (for instance the GPU's kept set) into the next.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flowmm_oracle.c")
_LIB = os.path.join(_HERE, "libflowmm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP across heads)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.fmo_flow.restype = C.c_int
        _lib.fmo_match.restype = C.c_int
        _lib.fmo_num_threads.restype = C.c_int
        _lib.fmo_cache_append.restype = C.c_int
        _lib.fmo_cache_remerge.restype = C.c_int
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return int(_load().fmo_num_threads())


def score(K, Q, mod, scale=None):
    """K [Hkv][L][d], Q [Hq][W][d], mod [L] -> I [Hkv][L] (float64), cross [Hq] (float64)."""
    K, Q, mod = _f32(K), _f32(Q), _i32(mod)
    Hkv, L, d = K.shape
    Hq, W, _ = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    I = np.empty((Hkv, L), dtype=np.float64)
    cross = np.empty(Hq, dtype=np.float64)
    _load().fmo_score(Hq, Hkv, L, W, d, C.c_double(scale), _p(K, C.c_float), _p(Q, C.c_float),
                      _p(mod, C.c_int32), _p(I, C.c_double), _p(cross, C.c_double))
    return I, cross


def flow(cross, theta, invert=False):
    """-> (rho, mode) with mode 1 = cross-modal merging, 0 = intra-modal; invert: the misaligned rule."""
    cross = _f64(cross)
    rho = C.c_double(0.0)
    mode = _load().fmo_flow(len(cross), _p(cross, C.c_double), C.c_double(theta), int(bool(invert)), C.byref(rho))
    return float(rho.value), int(mode)


def select(I, W, B):
    """I [L] -> kept_idx [B] ascending."""
    I = _f64(I)
    kept = np.empty(B, dtype=np.int32)
    _load().fmo_select(len(I), W, B, _p(I, C.c_double), _p(kept, C.c_int32))
    return kept


def match(K, I, kept_idx, mod, mode_cross, tau, with_margins=False):
    """K [L][d] -> assign [L], n_dropped (and u_best, u_second [L] if asked)."""
    K, I, kept_idx, mod = _f32(K), _f64(I), _i32(kept_idx), _i32(mod)
    L, d = K.shape
    assign = np.empty(L, dtype=np.int32)
    ub = np.empty(L, dtype=np.float64)
    us = np.empty(L, dtype=np.float64)
    nd = _load().fmo_match(L, d, len(kept_idx), _p(K, C.c_float), _p(I, C.c_double),
                           _p(kept_idx, C.c_int32), _p(mod, C.c_int32), int(mode_cross),
                           C.c_double(tau), _p(assign, C.c_int32), _p(ub, C.c_double),
                           _p(us, C.c_double))
    if with_margins:
        return assign, int(nd), ub, us
    return assign, int(nd)


def merge(K, V, kept_idx, assign):
    """K, V [L][d] -> Kout, Vout [B][d] float64 (unrounded), n_members [B]."""
    K, V, kept_idx, assign = _f32(K), _f32(V), _i32(kept_idx), _i32(assign)
    L, d = K.shape
    B = len(kept_idx)
    ko = np.empty((B, d), dtype=np.float64)
    vo = np.empty((B, d), dtype=np.float64)
    nm = np.empty(B, dtype=np.int32)
    _load().fmo_merge(L, d, B, _p(K, C.c_float), _p(V, C.c_float), _p(kept_idx, C.c_int32),
                      _p(assign, C.c_int32), _p(ko, C.c_double), _p(vo, C.c_double),
                      _p(nm, C.c_int32))
    return ko, vo, nm


def merge_weighted(K, V, kept_idx, assign):
    """Similarity-weighted merge: K, V [L][d] -> Kout, Vout [B][d] float64, n_members [B], wsum [B]."""
    K, V, kept_idx, assign = _f32(K), _f32(V), _i32(kept_idx), _i32(assign)
    L, d = K.shape
    B = len(kept_idx)
    ko = np.empty((B, d), dtype=np.float64)
    vo = np.empty((B, d), dtype=np.float64)
    nm = np.empty(B, dtype=np.int32)
    ws = np.empty(B, dtype=np.float64)
    _load().fmo_merge_weighted(L, d, B, _p(K, C.c_float), _p(V, C.c_float), _p(kept_idx, C.c_int32),
                               _p(assign, C.c_int32), _p(ko, C.c_double), _p(vo, C.c_double),
                               _p(nm, C.c_int32), _p(ws, C.c_double))
    return ko, vo, nm, ws


def decode_attention(q, Kc, Vc, scale=None):
    """q [G][d], Kc, Vc [B][d] -> out [G][d] float64: one decode step of attention over a compacted cache."""
    q, Kc, Vc = _f32(q), _f32(Kc), _f32(Vc)
    G, d = q.shape
    B = Kc.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((G, d), dtype=np.float64)
    _load().fmo_decode_attention(G, B, d, C.c_double(scale), _p(q, C.c_float), _p(Kc, C.c_float), _p(Vc, C.c_float),
                                 _p(out, C.c_double))
    return out


def round_output(x, dtype: str):
    """Nearest-even rounding of float64 to the cache dtype ("bf16" | "f32"); float32 array."""
    x = _f64(x)
    y = np.empty(x.shape, dtype=np.float32)
    _load().fmo_round(x.size, 1 if dtype == "bf16" else 0, _p(x, C.c_double), _p(y, C.c_float))
    return y


def layer_pass(K, V, Q, mod, B, dtype: str, theta: float, tau: float, scale=None):
    """All stages for one sequence and one layer.  K, V [Hkv][L][d]; Q [Hq][W][d]."""
    K, V, Q, mod = _f32(K), _f32(V), _f32(Q), _i32(mod)
    Hkv, L, d = K.shape
    Hq, W, _ = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    I = np.empty((Hkv, L), dtype=np.float64)
    rho = C.c_double(0.0)
    mode = C.c_int32(0)
    kept = np.empty((Hkv, B), dtype=np.int32)
    assign = np.empty((Hkv, L), dtype=np.int32)
    nd = np.empty(Hkv, dtype=np.int32)
    ko = np.empty((Hkv, B, d), dtype=np.float32)
    vo = np.empty((Hkv, B, d), dtype=np.float32)
    _load().fmo_layer(Hq, Hkv, L, W, d, B, 1 if dtype == "bf16" else 0, C.c_double(scale),
                      C.c_double(theta), C.c_double(tau), _p(K, C.c_float), _p(V, C.c_float),
                      _p(Q, C.c_float), _p(mod, C.c_int32), _p(I, C.c_double), C.byref(rho),
                      C.byref(mode), _p(kept, C.c_int32), _p(assign, C.c_int32), _p(nd, C.c_int32),
                      _p(ko, C.c_float), _p(vo, C.c_float))
    return dict(I=I, rho=float(rho.value), mode=int(mode.value), kept_idx=kept, assign=assign,
                n_dropped=nd, K_out=ko, V_out=vo)


def cache_append(Kc, Vc, length: int, k, v) -> int:
    """Cache-append equation on Kc, Vc [Hkv][capacity][d] (float32, contiguous, modified in place):
    row `length` of every kv head becomes k, v [Hkv][d].  Returns the new length, or -1 if the cache is full."""
    assert Kc.dtype == np.float32 and Vc.dtype == np.float32 and Kc.flags.c_contiguous and Vc.flags.c_contiguous
    k, v = _f32(k), _f32(v)
    Hkv, cap, d = Kc.shape
    return int(_load().fmo_cache_append(Hkv, cap, d, int(length), _p(Kc, C.c_float), _p(Vc, C.c_float),
                                        _p(k, C.c_float), _p(v, C.c_float)))


def cache_remerge(Kc, Vc, n: int, Q, B: int, dtype: str, tau: float, scale=None):
    """Re-merge of the first n rows of Kc, Vc [Hkv][capacity][d] (float32, contiguous, modified in place:
    rows [0, B) become the merged rows) with Q [Hq][W][d] the queries of the last W valid rows.
    Returns the plan of the re-merge (as layer_pass does, without the output rows) and the new length."""
    assert Kc.dtype == np.float32 and Vc.dtype == np.float32 and Kc.flags.c_contiguous and Vc.flags.c_contiguous
    Q = _f32(Q)
    Hkv, cap, d = Kc.shape
    Hq, W, _ = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    I = np.empty((Hkv, n), dtype=np.float64)
    rho = C.c_double(0.0)
    mode = C.c_int32(0)
    kept = np.empty((Hkv, B), dtype=np.int32)
    assign = np.empty((Hkv, n), dtype=np.int32)
    nd = np.empty(Hkv, dtype=np.int32)
    new_len = _load().fmo_cache_remerge(Hq, Hkv, cap, int(n), W, d, int(B), 1 if dtype == "bf16" else 0,
                                        C.c_double(scale), C.c_double(tau), _p(Kc, C.c_float), _p(Vc, C.c_float),
                                        _p(Q, C.c_float), _p(I, C.c_double), C.byref(rho), C.byref(mode),
                                        _p(kept, C.c_int32), _p(assign, C.c_int32), _p(nd, C.c_int32))
    return dict(I=I, rho=float(rho.value), mode=int(mode.value), kept_idx=kept, assign=assign, n_dropped=nd), int(new_len)
