#!/usr/bin/env python3
"""Benchmark of the FlowMM prefill-time KV-cache merge on one MI355X.

A step is one pass of the whole hot path (flowmm_plan_merge = flowmm_plan + flowmm_merge: score, flow, select,
match, merge) over every layer and head of one synthetic prefill cache that already sits in
HBM.  Prints ONE JSON line: tokens merged per second, the roofline of the dominant kernel
(timed live with HIP events on the launch stream) and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(wl):
    """Bytes each step of the method must move, per full pass, from the shapes alone.

    whole pass (a fused implementation): K twice (before and after the top-B split), V once,
    compacted rows written once, Q window, importance written+read and assign written:
    3 L d s + 2 B d s + G W d s + 12 L per (sequence, layer, kv head).
    Per kernel: what that kernel's own inputs and outputs amount to at the library boundary."""
    s = 2 if wl.dtype == "bf16" else 4
    d, G, W = wl.head_dim, wl.group, wl.window
    units = wl.n_layers * wl.n_kv_heads
    tot = {k: 0 for k in ("whole_pass", "score_stats", "score_colsum", "match", "merge_tasks",
                          "select", "merge_csr", "unit_plan", "unit_merge", "unit_flow_merge")}
    for L, B in zip(wl.seqlens, wl.budgets):
        row = d * s
        tot["whole_pass"] += units * (3 * L * row + 2 * B * row + G * W * row + 12 * L)
        tot["score_stats"] += units * (L * row + G * W * row)              # K once, Q window
        tot["score_colsum"] += units * (L * row + G * W * row + 4 * L)     # K once, Q, importance out
        # importance in, assign + kept out; pivot rows in, packed rows + tables out
        tot["select"] += units * (4 * L + 4 * L + 4 * B + 2 * B * row + 8 * B)
        tot["match"] += units * (L * row + 4 * L + 4 * L + 4 * B)          # K once, assign in/out, kept
        tot["merge_csr"] += units * (4 * L + 4 * (L - B))                  # assign in, member list out
        tot["merge_tasks"] += units * (2 * L * row + 2 * B * row + 4 * (L - B))  # K and V rows in, compacted out
        # unit-resident kernels (short prompts)
        # score + select + match in one kernel: the method needs K before and after the top-B split
        # (the split depends on every key), which is what the whole-pass figure counts; the kernel
        # keeps the unit's keys in registers, so its measured traffic is about one K less than this
        tot["unit_plan"] += units * (2 * L * row + G * W * row + 12 * L + 4 * B)
        tot["unit_merge"] += units * (2 * L * row + 2 * B * row + 4 * L + 4 * B)  # K, V rows, assign, kept in; compacted out
        tot["unit_flow_merge"] = tot["unit_merge"]  # the merge launch that also settles the layer strategies
    return tot


def measured_traffic(config: int, kernel: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary of this workload, if there is one."""
    for tag in ("unit_path", "generic_path"):
        path = os.path.join(ROOT, "profiles", f"{tag}_config{config}_hbm_traffic.txt")
        try:
            for line in open(path):
                f = [x.strip() for x in line.split("|")]
                if not line.startswith("#") and len(f) >= 4 and f[0] == kernel:
                    return float(f[3])
        except OSError:
            pass
    return None


def cpu_baseline(wl, budget_s: float):
    """Time the CPU oracle (as it stands) on whole layers of the same workload."""
    import oracle
    oracle.build()
    done, t_total = 0, 0.0
    while done < wl.n_layers and (done == 0 or t_total + t_total / done <= budget_s):
        K, V, Q = wl.layer_tensors(done)
        t0 = time.perf_counter()
        for b in range(wl.batch):
            sl = wl.seq_slice(b)
            W = wl.window
            oracle.layer_pass(K[:, sl], V[:, sl], Q[:, b * W:(b + 1) * W], wl.modality(b), wl.budgets[b],
                              wl.dtype, wl.theta, wl.tau[b])
        t_total += time.perf_counter() - t0
        done += 1
    t_full = t_total * wl.n_layers / done
    return {"value": wl.total_tokens / t_full, "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"layers 0..{done - 1} of {wl.n_layers} (all heads, all sequences), {t_total:.2f} s, "
                      f"scaled linearly to the full depth"}


def bench_flow_exact(args, wl, dev):
    """The exact flow ratio is a dense causal contraction: report it against the MFMA peak of its dtype."""
    import torch
    from paper_2511_05534_amd import binding as fb
    K, V, Q = fb.upload_workload(wl, dev)
    del V, Q
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    Qf = torch.randn((wl.n_layers, wl.n_q_heads, wl.total_tokens, wl.head_dim), generator=gen, device=dev).to(tdt)
    params = fb.Params.from_workload(wl)
    bufs = fb.DeviceBuffers(params, dev)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(args.warmup):
        bufs.flow_exact(K, Qf, stream)
    torch.cuda.synchronize()
    fb.flowmm_profile_select("flow_exact")
    t0 = time.perf_counter()
    for _ in range(args.steps):
        bufs.flow_exact(K, Qf, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms, n = fb.flowmm_profile_collect()["flow_exact"]
    fb.flowmm_profile_select("")
    flops = sum(2.0 * wl.head_dim * L * (L + 1) / 2 for L in wl.seqlens) * wl.n_q_heads * wl.n_layers
    peak = 2500.0 if wl.dtype == "bf16" else 157.3
    k_us = 1e3 * ms / n
    ms_per_step = 1e3 * (t1 - t0) / args.steps
    print(json.dumps({
        "metric": "exact cross-modal interaction ratio (all prompt queries), prompt tokens per second",
        "value": wl.total_tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {wl.name}", "layers": wl.n_layers, "q_heads": wl.n_q_heads,
                   "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "seqlens": wl.seqlens, "entry_point": "flowmm_flow_exact"},
        "roofline": {"bound": "mfma", "kernel": "flow_exact", "achieved": flops / (k_us * 1e-6) / 1e12, "peak": peak,
                     "unit": "TFLOP/s", "frac": flops / (k_us * 1e-6) / 1e12 / peak, "traffic": None, "kernel_us": k_us,
                     "algorithmic_flops_per_launch": flops},
    }))


def bench_decode(args, wl, dev):
    """Decode-step attention over the compacted cache at the budgets of the paper's latency table
    (shape of the trend only: attention over the cache, not a model's whole decode step)."""
    import torch
    from paper_2511_05534_amd import binding as fb
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    s = 2 if wl.dtype == "bf16" else 4
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for pct in (100, 50, 35, 20, 5):
        budgets = [min(L, max(wl.window, (L * pct + 50) // 100)) for L in wl.seqlens]
        params = fb.Params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.seqlens, budgets,
                           wl.spans, wl.window, wl.theta, wl.tau)
        bufs = fb.DeviceBuffers(params, dev)
        bufs.K_out.copy_(torch.randn(bufs.K_out.shape, generator=gen, device=dev).to(tdt))
        bufs.V_out.copy_(torch.randn(bufs.V_out.shape, generator=gen, device=dev).to(tdt))
        q = torch.randn((wl.n_layers, wl.n_q_heads, wl.batch, wl.head_dim), generator=gen, device=dev).to(tdt)
        out = torch.empty_like(q)
        for _ in range(args.warmup):
            bufs.decode_attention(q, out, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            bufs.decode_attention(q, out, stream=stream)
        torch.cuda.synchronize()
        us = 1e6 * (time.perf_counter() - t0) / args.steps
        nbytes = 2 * wl.n_layers * wl.n_kv_heads * sum(budgets) * wl.head_dim * s + 2 * q.numel() * s
        rows.append({"budget_pct": pct, "slots": budgets, "us_per_step": us, "cache_bytes": nbytes,
                     "GBs": nbytes / (us * 1e-6) / 1e9, "frac_of_hbm_peak": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS})
        del bufs
    full = rows[0]
    print(json.dumps({
        "metric": "decode-step attention over the compacted cache, latency per step by budget",
        "value": full["us_per_step"] / rows[-1]["us_per_step"], "unit": "x faster at 5 % budget than at 100 %",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rows[-1]["us_per_step"] / 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {wl.name}", "layers": wl.n_layers, "q_heads": wl.n_q_heads,
                   "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "seqlens": wl.seqlens,
                   "entry_point": "flowmm_decode_attention"},
        "roofline": {"bound": "hbm", "kernel": "decode_partial", "achieved": full["GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": full["frac_of_hbm_peak"], "traffic": None},
        "by_budget": rows,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload 0..4 (1 = the metric's configuration)")
    ap.add_argument("--layers", type=int, default=0,
                    help="depth override for kernel tuning runs (0 = the configuration's own depth, which the metric needs)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays of it (the library neither allocates nor "
                         "synchronises, so a serving loop can do this); per-kernel events are then taken from the warm-up")
    ap.add_argument("--two-calls", action="store_true",
                    help="run flowmm_plan then flowmm_merge instead of the one-call flowmm_plan_merge")
    ap.add_argument("--flow-exact", action="store_true",
                    help="time flowmm_flow_exact (the interaction ratio over all prompt queries) instead of the merge path")
    ap.add_argument("--decode", action="store_true",
                    help="time flowmm_decode_attention over compacted caches of this configuration at 100/50/35/20/5 %% budget")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the CPU-oracle leg; 0 skips it")
    ap.add_argument("--kernel", type=str, default="", help="kernel to report the roofline for (default: the slowest)")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="measured HBM bytes per launch of the roofline kernel (from the rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2511_05534_amd import binding as fb
    from paper_2511_05534_amd import workloads

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(3)
    fb.load(build_if_missing=False)
    wl = workloads.config(args.config, n_layers=args.layers or None)
    dev = "cuda:0"
    if args.flow_exact:
        return bench_flow_exact(args, wl, dev)
    if args.decode:
        return bench_decode(args, wl, dev)
    K, V, Q = fb.upload_workload(wl, dev)
    params = fb.Params.from_workload(wl)
    bufs = fb.DeviceBuffers(params, dev)
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        nonlocal stream
        if args.two_calls:
            bufs.plan(K, Q, stream)
            bufs.merge(K, V, stream)
        else:
            bufs.plan_merge(K, V, Q, stream)

    if args.pmc_calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # warm-up; its last steps are bracketed kernel by kernel to find the dominant one
    for _ in range(max(args.warmup - 5, 0)):
        step()
    torch.cuda.synchronize()
    fb.flowmm_profile_select("all")
    for _ in range(min(5, max(args.warmup, 1))):
        step()
    torch.cuda.synchronize()
    per_kernel = fb.flowmm_profile_collect()
    kernels_us = {k: 1e3 * ms / n for k, (ms, n) in per_kernel.items()}
    dominant = args.kernel or max(kernels_us, key=kernels_us.get)

    if args.graph:
        # the dominant kernel's duration comes from eager steps (events cannot be recorded inside the graph)
        fb.flowmm_profile_select(dominant)
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        dom_ms, dom_n = fb.flowmm_profile_collect()[dominant]
        fb.flowmm_profile_select("")
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            stream = torch.cuda.current_stream().cuda_stream
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        # timed region: exactly K steps; only the dominant kernel carries events
        fb.flowmm_profile_select(dominant)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dom_ms, dom_n = fb.flowmm_profile_collect()[dominant]
        fb.flowmm_profile_select("")

    ms_per_step = 1e3 * (t1 - t0) / args.steps
    tokens_per_s = wl.total_tokens / (ms_per_step * 1e-3)
    alg = algorithmic_bytes(wl)
    dom_us = 1e3 * dom_ms / dom_n
    achieved = alg.get(dominant, 0) / (dom_us * 1e-6) / 1e9
    out = {
        "metric": "KV tokens merged/sec per GPU + achieved HBM GB/s (% of peak), full prefill cache",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {wl.name}", "layers": wl.n_layers, "q_heads": wl.n_q_heads,
                   "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "seqlens": wl.seqlens, "budgets": wl.budgets,
                   "window": wl.window, "theta": wl.theta, "tokens_per_step": wl.total_tokens,
                   "entry_point": "flowmm_plan + flowmm_merge" if args.two_calls else "flowmm_plan_merge",
                   "hip_graph_replay": bool(args.graph),
                   "token_layer_kvheads_per_s": tokens_per_s * wl.n_layers * wl.n_kv_heads},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": args.traffic_bytes if args.traffic_bytes is not None else measured_traffic(args.config, dominant),
                     "kernel_us": dom_us, "algorithmic_bytes_per_launch": alg.get(dominant, 0)},
        "full_pass": {"algorithmic_bytes": alg["whole_pass"],
                      "achieved_GBs": alg["whole_pass"] / (ms_per_step * 1e-3) / 1e9,
                      "frac_of_hbm_peak": alg["whole_pass"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "host_enqueue_us_per_step": 1e6 * t_host / args.steps},
        "kernels_us": kernels_us,
    }
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
