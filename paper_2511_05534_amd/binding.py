"""Thin ctypes binding of libflowmm.so (include/flowmm.h): argument marshalling only.

Every step of the method runs in the library's HIP kernels; if the library is missing this
module raises instead of falling back to anything.  PyTorch appears only as the owner of
device memory and streams (`data_ptr()`, `cuda_stream`).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence, Tuple

import numpy as np

from . import build as _build

FLOWMM_OK, FLOWMM_EINVAL, FLOWMM_EUNSUPPORTED, FLOWMM_EWORKSPACE, FLOWMM_EHIP = range(5)
FLOWMM_F32, FLOWMM_BF16 = 0, 1
FLOWMM_FLAG_GENERIC_PATH, FLOWMM_FLAG_INVERT_FLOW, FLOWMM_FLAG_WEIGHTED_MERGE = 1, 2, 4
STATUS_NAMES = ["FLOWMM_OK", "FLOWMM_EINVAL", "FLOWMM_EUNSUPPORTED", "FLOWMM_EWORKSPACE", "FLOWMM_EHIP"]
PLAN_FIELDS = ("importance", "rho", "mode", "kept_idx", "assign", "n_dropped")
EXPORTS = ("flowmm_plan_sizes", "flowmm_plan", "flowmm_merge", "flowmm_plan_merge", "flowmm_plan_merge_static",
           "flowmm_static_workspace_bytes", "flowmm_flow_exact",
           "flowmm_cache_append", "flowmm_cache_remerge_sizes", "flowmm_cache_remerge",
           "flowmm_decode_attention", "flowmm_last_error",
           "flowmm_profile_kernel_count", "flowmm_profile_kernel_name", "flowmm_profile_select",
           "flowmm_profile_collect")


class flowmm_span(C.Structure):
    _fields_ = [("begin", C.c_int32), ("end", C.c_int32), ("modality", C.c_int32)]


class flowmm_params(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("dtype", C.c_int32), ("batch", C.c_int32),
        ("cu_seqlens", C.POINTER(C.c_int32)), ("budget_tokens", C.POINTER(C.c_int32)),
        ("spans", C.POINTER(flowmm_span)), ("cu_spans", C.POINTER(C.c_int32)),
        ("window", C.c_int32), ("scale", C.c_float), ("theta", C.c_float),
        ("tau", C.POINTER(C.c_float)),
        ("k_stride_layer", C.c_int64), ("k_stride_head", C.c_int64), ("k_stride_token", C.c_int64),
        ("q_stride_layer", C.c_int64), ("q_stride_head", C.c_int64), ("q_stride_token", C.c_int64),
        ("flags", C.c_int32),
    ]


class flowmm_plan_buffers(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in PLAN_FIELDS]


class FlowMMError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 5 else status}: {message}")
        self.status = status
        self.message = message


_lib = None


def load(build_if_missing: bool = True):
    """Load libflowmm.so; it is built first only if no library is there at all.

    PyTorch wheels carry a HIP runtime of their own.  Whichever of the two libraries is loaded first
    decides which runtime the process gets, and a process that ends up with two of them has one that
    sees no device.  Callers here always hand over PyTorch tensors, so PyTorch goes first when it is there."""
    global _lib
    if _lib is None:
        try:
            import torch  # noqa: F401  (only for its HIP runtime; see above)
        except ImportError:
            pass
        path = _build.library_path()
        if not os.path.exists(path):
            if not build_if_missing:
                raise FileNotFoundError(path)
            _build.build_library()
        lib = C.CDLL(path)
        lib.flowmm_last_error.restype = C.c_char_p
        lib.flowmm_plan_sizes.argtypes = [C.POINTER(flowmm_params), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        lib.flowmm_plan.argtypes = [C.POINTER(flowmm_params), C.c_void_p, C.c_void_p,
                                    C.POINTER(flowmm_plan_buffers), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.flowmm_merge.argtypes = [C.POINTER(flowmm_params), C.POINTER(flowmm_plan_buffers), C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.flowmm_plan_merge.argtypes = [C.POINTER(flowmm_params), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(flowmm_plan_buffers), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
        lib.flowmm_plan_merge_static.argtypes = [C.POINTER(flowmm_params), C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.POINTER(flowmm_plan_buffers), C.c_void_p, C.c_void_p, C.c_void_p]
        lib.flowmm_plan_merge_static.restype = C.c_int
        lib.flowmm_static_workspace_bytes.argtypes = []
        lib.flowmm_static_workspace_bytes.restype = C.c_size_t
        i32p = C.POINTER(C.c_int32)
        lib.flowmm_cache_append.argtypes = [C.POINTER(flowmm_params), i32p, i32p] + [C.c_void_p] * 5
        lib.flowmm_cache_append.restype = C.c_int
        lib.flowmm_cache_remerge_sizes.argtypes = [C.POINTER(flowmm_params), i32p, C.c_int32, C.c_int32,
                                                   C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        lib.flowmm_cache_remerge_sizes.restype = C.c_int
        lib.flowmm_cache_remerge.argtypes = [C.POINTER(flowmm_params), i32p, i32p, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.POINTER(flowmm_plan_buffers), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.flowmm_cache_remerge.restype = C.c_int
        lib.flowmm_flow_exact.argtypes = [C.POINTER(flowmm_params), C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                          C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.flowmm_flow_exact.restype = C.c_int
        lib.flowmm_decode_attention.argtypes = [C.POINTER(flowmm_params)] + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p]
        lib.flowmm_decode_attention.restype = C.c_int
        for f in (lib.flowmm_plan_sizes, lib.flowmm_plan, lib.flowmm_merge, lib.flowmm_plan_merge, lib.flowmm_profile_collect,
                  lib.flowmm_profile_kernel_count):
            f.restype = C.c_int
        lib.flowmm_profile_kernel_name.restype = C.c_char_p
        lib.flowmm_profile_kernel_name.argtypes = [C.c_int]
        lib.flowmm_profile_select.argtypes = [C.c_char_p]
        lib.flowmm_profile_select.restype = None
        lib.flowmm_profile_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_longlong)]
        _lib = lib
    return _lib


def _check(status: int):
    if status != FLOWMM_OK:
        raise FlowMMError(status, load().flowmm_last_error().decode())


class Params:
    """Owns the host arrays a flowmm_params points to."""

    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str,
                 seqlens: Sequence[int], budgets: Sequence[int],
                 spans: Sequence[Sequence[Tuple[int, int, int]]], window: int, theta: float,
                 tau: Sequence[float], scale: float = 0.0,
                 k_strides: Tuple[int, int, int] | None = None,
                 q_strides: Tuple[int, int, int] | None = None, flags: int = 0):
        self.batch = len(seqlens)
        self.seqlens = [int(x) for x in seqlens]
        self.budgets = [int(x) for x in budgets]
        self.total_tokens = int(sum(self.seqlens))
        self.sum_budget = int(sum(self.budgets))
        self.dtype = dtype
        self._cu = np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)
        self._bud = np.asarray(self.budgets, dtype=np.int32)
        flat = [s for seq in spans for s in seq]
        self._spans = (flowmm_span * max(1, len(flat)))(*[flowmm_span(int(a), int(b), int(m)) for a, b, m in flat])
        self._cu_spans = np.concatenate([[0], np.cumsum([len(s) for s in spans])]).astype(np.int32)
        self._tau = np.asarray(tau, dtype=np.float32)
        T, W, d = self.total_tokens, int(window), int(head_dim)
        if k_strides is None:
            k_strides = (n_kv_heads * T * d, T * d, d)
        if q_strides is None:
            q_strides = (n_q_heads * self.batch * W * d, self.batch * W * d, d)
        self.c = flowmm_params(
            n_layers, n_q_heads, n_kv_heads, head_dim, FLOWMM_BF16 if dtype == "bf16" else FLOWMM_F32,
            self.batch, self._cu.ctypes.data_as(C.POINTER(C.c_int32)),
            self._bud.ctypes.data_as(C.POINTER(C.c_int32)), self._spans,
            self._cu_spans.ctypes.data_as(C.POINTER(C.c_int32)), W, float(scale), float(theta),
            self._tau.ctypes.data_as(C.POINTER(C.c_float)), *k_strides, *q_strides, int(flags))
        self.n_layers, self.n_q_heads, self.n_kv_heads, self.head_dim, self.window = \
            n_layers, n_q_heads, n_kv_heads, head_dim, W

    @classmethod
    def from_workload(cls, wl, theta: float | None = None, tau: Sequence[float] | None = None, flags: int = 0):
        return cls(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.seqlens, wl.budgets,
                   wl.spans, wl.window, wl.theta if theta is None else theta, wl.tau if tau is None else tau,
                   flags=flags)


def flowmm_plan_sizes(params: Params):
    sizes = (C.c_size_t * 6)()
    ws = C.c_size_t(0)
    _check(load().flowmm_plan_sizes(C.byref(params.c), sizes, C.byref(ws)))
    return [int(x) for x in sizes], int(ws.value)


def _plan_struct(plan_ptrs: Sequence[int]) -> flowmm_plan_buffers:
    return flowmm_plan_buffers(*[C.c_void_p(int(p)) for p in plan_ptrs])


def flowmm_plan(params: Params, K: int, Q_window: int, plan_ptrs: Sequence[int], workspace: int,
                workspace_bytes: int, stream: int = 0):
    """All arguments after `params` are raw device addresses (ints)."""
    pb = _plan_struct(plan_ptrs)
    _check(load().flowmm_plan(C.byref(params.c), C.c_void_p(K), C.c_void_p(Q_window), C.byref(pb),
                              C.c_void_p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def flowmm_merge(params: Params, plan_ptrs: Sequence[int], K: int, V: int, K_out: int, V_out: int,
                 workspace: int, workspace_bytes: int, stream: int = 0):
    pb = _plan_struct(plan_ptrs)
    _check(load().flowmm_merge(C.byref(params.c), C.byref(pb), C.c_void_p(K), C.c_void_p(V),
                               C.c_void_p(K_out), C.c_void_p(V_out), C.c_void_p(workspace),
                               C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def flowmm_plan_merge(params: Params, K: int, V: int, Q_window: int, plan_ptrs: Sequence[int], K_out: int,
                      V_out: int, workspace: int, workspace_bytes: int, stream: int = 0):
    pb = _plan_struct(plan_ptrs)
    _check(load().flowmm_plan_merge(C.byref(params.c), C.c_void_p(K), C.c_void_p(V), C.c_void_p(Q_window),
                                    C.byref(pb), C.c_void_p(K_out), C.c_void_p(V_out), C.c_void_p(workspace),
                                    C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def flowmm_plan_merge_static(params: Params, K: int, V: int, Q_window: int, plan_ptrs: Sequence[int], K_out: int,
                             V_out: int, stream: int = 0):
    """flowmm_plan_merge on the library's own scratch array (no workspace argument)."""
    pb = _plan_struct(plan_ptrs)
    _check(load().flowmm_plan_merge_static(C.byref(params.c), C.c_void_p(K), C.c_void_p(V), C.c_void_p(Q_window),
                                           C.byref(pb), C.c_void_p(K_out), C.c_void_p(V_out), C.c_void_p(stream)))


def flowmm_static_workspace_bytes() -> int:
    return int(load().flowmm_static_workspace_bytes())


def _i32_array(values):
    a = np.asarray(values, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def flowmm_cache_append(params: Params, cu_capacity, lengths, K_c: int, V_c: int, k_new: int, v_new: int, stream: int = 0):
    """Cache-append equation: one new K/V row per sequence behind its `lengths[b]` valid rows.
    `params` describes the cache (its k strides are the cache's strides)."""
    cap, cap_p = _i32_array(cu_capacity)
    ln, ln_p = _i32_array(lengths)
    _check(load().flowmm_cache_append(C.byref(params.c), cap_p, ln_p, C.c_void_p(K_c), C.c_void_p(V_c),
                                      C.c_void_p(k_new), C.c_void_p(v_new), C.c_void_p(stream)))


def flowmm_cache_remerge_sizes(params: Params, cu_capacity, seq: int, length: int):
    cap, cap_p = _i32_array(cu_capacity)
    sizes = (C.c_size_t * 6)()
    ws = C.c_size_t(0)
    _check(load().flowmm_cache_remerge_sizes(C.byref(params.c), cap_p, int(seq), int(length), sizes, C.byref(ws)))
    return [int(x) for x in sizes], int(ws.value)


def flowmm_cache_remerge(params: Params, cu_capacity, lengths, seq: int, K_c: int, V_c: int, Q_window: int,
                         plan_ptrs: Sequence[int], workspace: int, workspace_bytes: int, stream: int = 0):
    """Compress the valid rows of sequence `seq` of the cache back to its budget (rows [0, B) of its range)."""
    cap, cap_p = _i32_array(cu_capacity)
    ln, ln_p = _i32_array(lengths)
    pb = _plan_struct(plan_ptrs)
    _check(load().flowmm_cache_remerge(C.byref(params.c), cap_p, ln_p, int(seq), C.c_void_p(K_c), C.c_void_p(V_c),
                                       C.c_void_p(Q_window), C.byref(pb), C.c_void_p(workspace),
                                       C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def flowmm_flow_exact(params: Params, K: int, Q_full: int, q_strides: Tuple[int, int, int], rho: int, mode: int,
                      workspace: int, workspace_bytes: int, stream: int = 0):
    _check(load().flowmm_flow_exact(C.byref(params.c), C.c_void_p(K), C.c_void_p(Q_full), *[C.c_int64(int(x)) for x in q_strides],
                                    C.c_void_p(rho), C.c_void_p(mode), C.c_void_p(workspace),
                                    C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def flowmm_decode_attention(params: Params, q: int, K_c: int, V_c: int, out: int, workspace: int,
                            workspace_bytes: int, stream: int = 0):
    _check(load().flowmm_decode_attention(C.byref(params.c), C.c_void_p(q), C.c_void_p(K_c), C.c_void_p(V_c),
                                          C.c_void_p(out), C.c_void_p(workspace), C.c_size_t(workspace_bytes),
                                          C.c_void_p(stream)))


def flowmm_profile_select(names: str = ""):
    load().flowmm_profile_select(names.encode())


def flowmm_profile_collect():
    """-> {kernel name: (total milliseconds, launches)} for the kernels bracketed since the last call."""
    lib = load()
    n = lib.flowmm_profile_kernel_count()
    ms = (C.c_double * n)()
    cnt = (C.c_longlong * n)()
    _check(lib.flowmm_profile_collect(ms, cnt))
    return {lib.flowmm_profile_kernel_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n) if cnt[i]}


# ---- device-memory plumbing (PyTorch owns the memory; nothing below computes) ------------------
def upload_workload(wl, device="cuda:0", layers=None):
    """K, V [Lyr][Hkv][T][d] and Q [Lyr][Hq][batch*W][d] of a synthetic workload as device tensors."""
    import torch
    layers = range(wl.n_layers) if layers is None else layers
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    Ks, Vs, Qs = [], [], []
    for l in layers:
        k, v, q = wl.layer_tensors(l)  # float32 values that are exact in the workload dtype
        Ks.append(torch.from_numpy(k).to(device).to(tdt))
        Vs.append(torch.from_numpy(v).to(device).to(tdt))
        Qs.append(torch.from_numpy(q).to(device).to(tdt))
    return torch.stack(Ks), torch.stack(Vs), torch.stack(Qs)


class DeviceBuffers:
    """Plan buffers, outputs and workspace for one Params, allocated with torch on `device`."""

    def __init__(self, params: Params, device="cuda:0"):
        import torch
        self.params = params
        sizes, ws = flowmm_plan_sizes(params)
        Lyr, Hkv, T, SB, Bt = params.n_layers, params.n_kv_heads, params.total_tokens, params.sum_budget, params.batch
        tdt = torch.bfloat16 if params.dtype == "bf16" else torch.float32
        self.importance = torch.empty((Lyr, Hkv, T), dtype=torch.float32, device=device)
        self.rho = torch.empty((Lyr, Bt), dtype=torch.float32, device=device)
        self.mode = torch.empty((Lyr, Bt), dtype=torch.int32, device=device)
        self.kept_idx = torch.empty((Lyr, Hkv, SB), dtype=torch.int32, device=device)
        self.assign = torch.empty((Lyr, Hkv, T), dtype=torch.int32, device=device)
        self.n_dropped = torch.empty((Lyr, Hkv, Bt), dtype=torch.int32, device=device)
        for name, nbytes in zip(PLAN_FIELDS, sizes):
            t = getattr(self, name)
            assert t.numel() * t.element_size() == nbytes, (name, nbytes)
        self.K_out = torch.empty((Lyr, Hkv, SB, params.head_dim), dtype=tdt, device=device)
        self.V_out = torch.empty_like(self.K_out)
        self.workspace_bytes = ws
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=device)

    @property
    def plan_ptrs(self) -> List[int]:
        return [getattr(self, n).data_ptr() for n in PLAN_FIELDS]

    def plan(self, K, Q, stream: int = 0):
        flowmm_plan(self.params, K.data_ptr(), Q.data_ptr(), self.plan_ptrs, self.workspace.data_ptr(),
                    self.workspace_bytes, stream)

    def plan_merge(self, K, V, Q, stream: int = 0):
        flowmm_plan_merge(self.params, K.data_ptr(), V.data_ptr(), Q.data_ptr(), self.plan_ptrs,
                          self.K_out.data_ptr(), self.V_out.data_ptr(), self.workspace.data_ptr(),
                          self.workspace_bytes, stream)

    def plan_merge_static(self, K, V, Q, stream: int = 0):
        flowmm_plan_merge_static(self.params, K.data_ptr(), V.data_ptr(), Q.data_ptr(), self.plan_ptrs,
                                 self.K_out.data_ptr(), self.V_out.data_ptr(), stream)

    def flow_exact(self, K, Q_full, stream: int = 0):
        """Q_full [Lyr][Hq][T][d] contiguous; fills self.rho and self.mode."""
        Hq, T, d = Q_full.shape[1:]
        flowmm_flow_exact(self.params, K.data_ptr(), Q_full.data_ptr(), (Hq * T * d, T * d, d), self.rho.data_ptr(),
                          self.mode.data_ptr(), self.workspace.data_ptr(), self.workspace_bytes, stream)

    def decode_attention(self, q, out, K_c=None, V_c=None, stream: int = 0):
        """q, out [Lyr][Hq][batch][d] contiguous; attends over self.K_out / self.V_out unless others are given."""
        K_c = self.K_out if K_c is None else K_c
        V_c = self.V_out if V_c is None else V_c
        flowmm_decode_attention(self.params, q.data_ptr(), K_c.data_ptr(), V_c.data_ptr(), out.data_ptr(),
                                self.workspace.data_ptr(), self.workspace_bytes, stream)

    def merge(self, K, V, stream: int = 0):
        flowmm_merge(self.params, self.plan_ptrs, K.data_ptr(), V.data_ptr(), self.K_out.data_ptr(),
                     self.V_out.data_ptr(), self.workspace.data_ptr(), self.workspace_bytes, stream)
