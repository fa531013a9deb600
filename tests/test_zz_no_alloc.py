"""flowmm_plan_merge_static (the entry point for callers that cannot allocate: its scratch is a device
array inside the library) against flowmm_plan_merge with a caller-allocated workspace, through the C ABI.
Both run the same kernels, so every output must be bit-identical; two calls in a row share the array,
the second on a smaller input, so nothing may depend on what the first one left there."""
import numpy as np
import pytest

from paper_2511_05534_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _both(w, flags=0):
    import torch
    from paper_2511_05534_amd import binding as fb
    K, V, Q = fb.upload_workload(w, "cuda:0")
    params = fb.Params.from_workload(w, flags=flags)
    stream = torch.cuda.current_stream().cuda_stream
    ref = fb.DeviceBuffers(params)
    ref.plan_merge(K, V, Q, stream)
    got = fb.DeviceBuffers(params)
    for n in fb.PLAN_FIELDS + ("K_out", "V_out"):
        getattr(got, n).fill_(0)
    got.workspace = None  # not used by the call under test
    got.plan_merge_static(K, V, Q, stream)
    torch.cuda.synchronize()
    return ref, got


def _assert_identical(ref, got, what):
    import torch
    from paper_2511_05534_amd import binding as fb
    for n in fb.PLAN_FIELDS + ("K_out", "V_out"):
        a, b = getattr(ref, n), getattr(got, n)
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (what, n)


def test_static_scratch_equals_caller_workspace_on_two_calls_in_a_row(oracle):
    from paper_2511_05534_amd import binding as fb
    from parity_utils import check_layer
    # first call: several key tiles, a ragged tail, two sequences, the multi-workgroup kernels (they are the
    # ones that stage row statistics, pivot lists, member lists and partial sums in the scratch)
    big = wl.make_workload("no_alloc_big", "bf16", 31, 2, 4, 2, 128, 32, [[100, 2300, 50, 1700, 77], [64, 700, 69]], [7, 20])
    # second call: a smaller input of another shape, same array
    small = wl.make_workload("no_alloc_small", "bf16", 32, 2, 6, 2, 128, 32, [[37, 411, 83]], [10])
    for w, flags in ((big, 0), (small, 1), (small, 0)):  # the last one takes the unit-resident kernels
        print(f"{w.name} flags={flags}: L={w.seqlens} B={w.budgets}", flush=True)
        assert fb.flowmm_plan_sizes(fb.Params.from_workload(w, flags=flags))[1] <= fb.flowmm_static_workspace_bytes()
        ref, got = _both(w, flags)
        _assert_identical(ref, got, w.name)
    # ... and against the oracle, to the parity bar of every other test (the last call's result)
    out = {n: getattr(got, n).cpu().numpy() for n in fb.PLAN_FIELDS}
    out["K_out"] = got.K_out.float().cpu().numpy()
    out["V_out"] = got.V_out.float().cpu().numpy()
    for l in range(small.n_layers):
        check_layer(oracle, small, out, l)


def test_static_scratch_refuses_shapes_beyond_the_array():
    import torch
    from paper_2511_05534_amd import binding as fb
    w = wl.config(3, n_layers=32)
    params = fb.Params.from_workload(w)
    assert fb.flowmm_plan_sizes(params)[1] > fb.flowmm_static_workspace_bytes()
    t = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(fb.FlowMMError) as ei:
        fb.flowmm_plan_merge_static(params, t.data_ptr(), t.data_ptr() + (1 << 40), t.data_ptr(), [t.data_ptr()] * 6,
                                    t.data_ptr() + (1 << 41), t.data_ptr() + (1 << 42))
    assert ei.value.status == fb.FLOWMM_EWORKSPACE and "scratch" in ei.value.message


def test_static_entry_point_in_a_hip_graph():
    """What the entry point is for: a caller under stream capture.  Every replay of the captured call (with
    eager work and a synchronisation in between) must reproduce the eager result of flowmm_plan_merge."""
    import torch
    from paper_2511_05534_amd import binding as fb
    for name, flags in (("no_alloc_graph_unit", 0), ("no_alloc_graph_generic", 1)):
        w = wl.make_workload(name, "bf16", 33, 3, 4, 2, 128, 32, [[37, 411, 83]], [10])
        K, V, Q = fb.upload_workload(w, "cuda:0")
        params = fb.Params.from_workload(w, flags=flags)
        ref = fb.DeviceBuffers(params)
        ref.plan_merge(K, V, Q, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got = fb.DeviceBuffers(params)
        got.workspace = None
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            got.plan_merge_static(K, V, Q, side.cuda_stream)  # first use outside the capture: symbol look-up, function attributes
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            got.plan_merge_static(K, V, Q, torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            for n in fb.PLAN_FIELDS + ("K_out", "V_out"):
                getattr(got, n).fill_(0)
            torch.randn(1 << 20, device="cuda:0").sum().item()  # unrelated eager work and a synchronisation
            graph.replay()
            torch.cuda.synchronize()
            _assert_identical(ref, got, (name, rep))
