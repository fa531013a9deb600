"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes its buffers, and rejects malformed arguments before launching anything."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2511_05534_amd import binding as fb
from paper_2511_05534_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"^[a-z_ ]*?\**\b(flowmm_[a-z_]+)\s*\(", header, flags=re.M))
    assert declared == set(fb.EXPORTS)
    lib = fb.load()
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_the_header():
    assert C.sizeof(fb.flowmm_span) == 12
    assert C.sizeof(fb.flowmm_plan_buffers) == 48
    # int32 x6, 4 pointers, int32 + 2 floats (+pad), pointer, 6 int64
    assert C.sizeof(fb.flowmm_params) == 24 + 32 + 16 + 8 + 48 + 8


def params_for(**kw):
    base = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=128, dtype="bf16", seqlens=[300, 200],
                budgets=[30, 40], spans=[[(0, 100, 0), (100, 300, 1)], [(0, 200, 0)]], window=16,
                theta=0.25, tau=[0.1, 0.2])
    base.update(kw)
    return fb.Params(**base)


def test_plan_sizes():
    p = params_for()
    sizes, ws = fb.flowmm_plan_sizes(p)
    units, T, SB = 2 * 2, 500, 70
    assert sizes == [units * T * 4, 2 * 2 * 4, 2 * 2 * 4, units * SB * 4, units * T * 4, units * 2 * 4]
    assert ws > 0 and ws % 256 == 0
    for i in range(5):
        w = wl.config(i)
        sizes, ws = fb.flowmm_plan_sizes(fb.Params.from_workload(w))
        assert sizes[0] == w.n_layers * w.n_kv_heads * w.total_tokens * 4
        assert ws < 1 << 30


BAD = [
    (dict(n_q_heads=5), fb.FLOWMM_EINVAL, "multiple"),
    (dict(head_dim=96), fb.FLOWMM_EUNSUPPORTED, "head_dim"),
    (dict(window=0), fb.FLOWMM_EINVAL, "window"),
    (dict(window=201, budgets=[250, 200]), fb.FLOWMM_EINVAL, "exceeds"),
    (dict(budgets=[8, 40]), fb.FLOWMM_EINVAL, "budget"),
    (dict(budgets=[301, 40]), fb.FLOWMM_EINVAL, "budget"),
    (dict(spans=[[(0, 100, 0), (101, 300, 1)], [(0, 200, 0)]]), fb.FLOWMM_EINVAL, "contiguous"),
    (dict(spans=[[(0, 100, 0), (100, 299, 1)], [(0, 200, 0)]]), fb.FLOWMM_EINVAL, "cover"),
    (dict(spans=[[(0, 100, 0), (100, 300, 2)], [(0, 200, 0)]]), fb.FLOWMM_EINVAL, "modality"),
    (dict(tau=[float("nan"), 0.1]), fb.FLOWMM_EINVAL, "tau"),
    (dict(theta=float("nan")), fb.FLOWMM_EINVAL, "theta"),
    (dict(scale=-1.0), fb.FLOWMM_EINVAL, "scale"),
    (dict(k_strides=(2 * 500 * 128, 500 * 128, 100)), fb.FLOWMM_EINVAL, "stride"),
    (dict(k_strides=(2 * 500 * 128, 500 * 128, 132)), fb.FLOWMM_EINVAL, "16 bytes"),
    (dict(n_q_heads=64, n_kv_heads=1, window=128, budgets=[130, 140]), fb.FLOWMM_EUNSUPPORTED, "LDS"),
    (dict(seqlens=[300, 0], budgets=[30, 0]), fb.FLOWMM_EINVAL, "increasing"),
    (dict(flags=8), fb.FLOWMM_EINVAL, "flags"),
    # the two query heads of a kv head 5 GiB apart: beyond the kernels' 32-bit offsets
    (dict(q_strides=(1 << 34, 5 << 29, 128)), fb.FLOWMM_EUNSUPPORTED, "4 GiB"),
]


@pytest.mark.parametrize("kw,status,word", BAD)
def test_bad_arguments_are_rejected_on_the_host(kw, status, word):
    p = params_for(**kw)
    with pytest.raises(fb.FlowMMError) as ei:
        fb.flowmm_plan_sizes(p)
    assert ei.value.status == status
    assert word in ei.value.message, ei.value.message


def test_pointer_checks_happen_before_any_launch():
    """No GPU here: these calls must fail in validation and never reach a HIP call."""
    p = params_for()
    sizes, ws = fb.flowmm_plan_sizes(p)
    good = 0x10000
    plan = [good] * 6
    cases = [
        (lambda: fb.flowmm_plan(p, 0, good, plan, good, ws), "NULL"),
        (lambda: fb.flowmm_plan(p, good + 8, good, plan, good, ws), "aligned"),
        (lambda: fb.flowmm_plan(p, good, good, [good, good, 0, good, good, good], good, ws), "plan->mode"),
        (lambda: fb.flowmm_merge(p, plan, good, good, 0, good, good, ws), "NULL"),
        (lambda: fb.flowmm_merge(p, plan, good, 1 << 40, good + 256, 1 << 41, good, ws), "overlap"),
        (lambda: fb.flowmm_merge(p, plan, good, 1 << 40, 1 << 41, 1 << 41, 1 << 42, ws), "overlap"),
    ]
    far = [1 << 40, 1 << 41, 1 << 42, 1 << 43]
    qs = (4 * 500 * 128, 500 * 128, 128)
    cases += [
        (lambda: fb.flowmm_plan_merge(p, good, far[0], 0, plan, far[1], far[2], good, ws), "NULL"),
        (lambda: fb.flowmm_plan_merge(p, good, far[0], far[3], plan, far[1], 0, good, ws), "NULL"),
        (lambda: fb.flowmm_plan_merge(p, good, far[0], far[3], plan, far[1], far[1] + 256, good, ws), "overlap"),
        (lambda: fb.flowmm_plan_merge(p, good, far[0], far[3], [good, good, good, 0, good, good], far[1], far[2], good, ws),
         "plan->kept_idx"),
        (lambda: fb.flowmm_plan_merge_static(p, good, far[0], 0, plan, far[1], far[2]), "NULL"),
        (lambda: fb.flowmm_plan_merge_static(p, good, far[0], far[3], plan, far[1], far[1] + 256), "overlap"),
        (lambda: fb.flowmm_plan_merge_static(p, good + 8, far[0], far[3], plan, far[1], far[2]), "aligned"),
        (lambda: fb.flowmm_flow_exact(p, good, 0, qs, good, good, good, ws), "NULL"),
        (lambda: fb.flowmm_flow_exact(p, good, far[0], qs, good + 2, good, good, ws), "4-byte"),
        (lambda: fb.flowmm_flow_exact(p, good, far[0], (qs[0], qs[1], 100), good, good, good, ws), "stride"),
        (lambda: fb.flowmm_flow_exact(p, good, far[0], (qs[0], qs[1], 132), good, good, good, ws), "16 bytes"),
        (lambda: fb.flowmm_decode_attention(p, good, far[0], far[1], 0, good, ws), "NULL"),
        (lambda: fb.flowmm_decode_attention(p, good + 4, far[0], far[1], far[2], good, ws), "aligned"),
    ]
    for call, word in cases:
        with pytest.raises(fb.FlowMMError) as ei:
            call()
        assert ei.value.status == fb.FLOWMM_EINVAL and word in ei.value.message, ei.value.message
    for call in (lambda: fb.flowmm_plan(p, good, good, plan, good, ws - 1),
                 lambda: fb.flowmm_plan_merge(p, good, far[0], far[3], plan, far[1], far[2], good, ws - 1),
                 lambda: fb.flowmm_flow_exact(p, good, far[0], qs, good, good, good, ws - 1),
                 lambda: fb.flowmm_decode_attention(p, good, far[0], far[1], far[2], good, ws - 1)):
        with pytest.raises(fb.FlowMMError) as ei:
            call()
        assert ei.value.status == fb.FLOWMM_EWORKSPACE


def test_last_error_is_never_null():
    assert isinstance(fb.load().flowmm_last_error(), bytes)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more ends with a message and a non-zero status
    before anything touches a device."""
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    """flowmm_plan_merge_static works on a 64 MiB array inside the library: shapes that need more are
    refused on the host, with both sizes in the message, before any HIP call."""
    cap = fb.flowmm_static_workspace_bytes()
    assert cap == 64 << 20
    far = [1 << 40, 1 << 41, 1 << 42, 1 << 43, 1 << 44]
    plan = [0x10000] * 6
    for i, fits in ((1, True), (2, True), (3, False), (4, False)):
        p = fb.Params.from_workload(wl.config(i))
        _, ws = fb.flowmm_plan_sizes(p)
        assert (ws <= cap) == fits
        if not fits:
            with pytest.raises(fb.FlowMMError) as ei:
                fb.flowmm_plan_merge_static(p, far[0], far[1], far[2], plan, far[3], far[4])
            assert ei.value.status == fb.FLOWMM_EWORKSPACE
            assert str(ws) in ei.value.message and str(cap) in ei.value.message


def test_cache_maintenance_argument_checks():
    """flowmm_cache_append / flowmm_cache_remerge validate on the host before any HIP call."""
    p = params_for(seqlens=[40, 50], budgets=[30, 40], spans=[[(0, 40, 0)], [(0, 50, 0)]], window=8)
    good, far = 0x10000, [1 << 40, 1 << 41, 1 << 42]
    cap = [0, 40, 90]
    bad = [
        (lambda: fb.flowmm_cache_append(p, cap, [30, 50], good, far[0], far[1], far[2]), "full"),
        (lambda: fb.flowmm_cache_append(p, cap, [30, 51], good, far[0], far[1], far[2]), "outside"),
        (lambda: fb.flowmm_cache_append(p, [0, 40, 40], [30, 40], good, far[0], far[1], far[2]), "increasing"),
        (lambda: fb.flowmm_cache_append(p, [1, 40, 90], [30, 40], good, far[0], far[1], far[2]), "cu_capacity[0]"),
        (lambda: fb.flowmm_cache_append(p, cap, [30, 40], 0, far[0], far[1], far[2]), "NULL"),
        (lambda: fb.flowmm_cache_append(p, cap, [30, 40], good + 4, far[0], far[1], far[2]), "aligned"),
        (lambda: fb.flowmm_cache_remerge_sizes(p, cap, 2, 40), "outside the batch"),
        (lambda: fb.flowmm_cache_remerge_sizes(p, cap, 1, 51), "capacity"),
        (lambda: fb.flowmm_cache_remerge_sizes(p, cap, 1, 39), "budget"),   # fewer rows than the budget
        (lambda: fb.flowmm_cache_remerge(p, cap, [40, 50], 0, good, far[0], 0, [good] * 6, far[1], 1 << 30), "NULL"),
        (lambda: fb.flowmm_cache_remerge(p, cap, [40, 50], 0, good, far[0], far[2], [good] * 6, 0, 1 << 30), "NULL"),
    ]
    for call, word in bad:
        with pytest.raises(fb.FlowMMError) as ei:
            call()
        assert ei.value.status == fb.FLOWMM_EINVAL and word in ei.value.message, ei.value.message
    sizes, ws = fb.flowmm_cache_remerge_sizes(p, cap, 1, 50)
    assert sizes == [2 * 2 * 50 * 4, 2 * 4, 2 * 4, 2 * 2 * 40 * 4, 2 * 2 * 50 * 4, 2 * 2 * 4]
    out_bytes = 2 * 2 * 40 * 128 * 2
    assert ws % 256 == 0 and ws >= 2 * out_bytes
    with pytest.raises(fb.FlowMMError) as ei:
        fb.flowmm_cache_remerge(p, cap, [40, 50], 1, good, far[0], far[2], [good] * 6, far[1], ws - 1)
    assert ei.value.status == fb.FLOWMM_EWORKSPACE
