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


MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}

# Kernels that together make up one step of the method and share its algorithmic bytes: the two
# streaming passes of the score (the row statistics of the softmax, then the column sums) need K once
# between them by the method's own dependencies, so the group is credited one K read and is timed as a whole.
# 1024 SIMDs x 2.4 GHz x 64 lanes / 18 issue cycles per softmax logit
ALU_PEAK_LOGITS = 1024 * 2.4e9 * 64 / 18
GROUPS = {"score_stats": "score", "score_combine": "score", "score_colsum": "score"}


def algorithmic_work(wl):
    """Bytes and flops the method itself must move / compute per full pass, from the shapes alone.

    Whole pass, per (sequence, layer, kv head): K twice (before and after the top-B split, which
    depends on every key), V once, the compacted rows written once, the window queries, and the
    importance written + read and the assignment written:
        3 L d s + 2 B d s + G W d s + 12 L  bytes.
    The per-kernel credits below add up to exactly that (asserted): a kernel is credited what the
    method needs at its step, not what this implementation happens to re-read (the generic path
    reads K four times; the match kernel's own K read is such a re-read and is credited nothing: it
    is the dense contraction and is measured against the matrix-core peak instead).
    Flops: score 2 G W L d (causal mask ignored), match 2 (L - B) B d."""
    s = 2 if wl.dtype == "bf16" else 4
    d, G, W = wl.head_dim, wl.group, wl.window
    units = wl.n_layers * wl.n_kv_heads
    byt = {k: 0 for k in ("whole_pass", "score", "select", "match", "merge_csr", "merge_tasks", "merge_fold",
                          "unit_plan", "unit_match", "unit_merge", "unit_flow_merge")}
    flops = {"score": 0.0, "match": 0.0}
    for L, B in zip(wl.seqlens, wl.budgets):
        row = d * s
        byt["whole_pass"] += units * (3 * L * row + 2 * B * row + G * W * row + 12 * L)
        # generic path
        byt["score"] += units * (L * row + G * W * row + 4 * L)        # K once, window queries, importance out
        byt["select"] += units * (4 * L + 4 * L)                       # importance in, assignment out
        byt["merge_tasks"] += units * (2 * L * row + 2 * B * row)      # K and V rows in, compacted rows out
        # unit-resident path (short prompts): the plan kernel keeps the keys on chip from the score to the match
        byt["unit_plan"] += units * (L * row + G * W * row + 12 * L)
        byt["unit_merge"] += units * (2 * L * row + 2 * B * row)
        flops["score"] += units * 2.0 * G * W * L * d
        flops["match"] += units * 2.0 * (L - B) * B * d
    byt["unit_flow_merge"] = byt["unit_merge"]
    assert byt["score"] + byt["select"] + byt["merge_tasks"] == byt["whole_pass"]
    assert byt["unit_plan"] + byt["unit_merge"] == byt["whole_pass"]
    return byt, flops


def measured_traffic(config: int, kernels):
    """HBM bytes per launch (summed over `kernels`) from the committed rocprofv3 counter summary of this
    workload, and the file they were read from; (None, None) if there is none."""
    for tag in ("unit_path", "generic_path"):
        rel = os.path.join("profiles", f"{tag}_config{config}_hbm_traffic.txt")
        found = {}
        try:
            for line in open(os.path.join(ROOT, rel)):
                f = [x.strip() for x in line.split("|")]
                if not line.startswith("#") and len(f) >= 4 and f[0] in kernels:
                    found[f[0]] = float(f[3])
        except OSError:
            continue
        if len(found) == len(kernels):
            return sum(found.values()), rel
    return None, None


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
    # the oracle's parallel loops run over the kv heads of a layer: that many threads work, if the host has them
    return {"value": wl.total_tokens / t_full, "unit": "tokens/s", "cores": min(oracle.num_threads(), wl.n_kv_heads),
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


def bench_cache(args, wl, dev):
    """Decode-time maintenance of the compacted cache: every sequence holds its budget of merged rows plus
    a quarter of that as head room; a cycle appends one token per step until the head room is full and then
    compresses every sequence back to its budget (append equation of the Preliminary section; the re-merge
    is this build's reading of how the method is kept up while decoding)."""
    import numpy as np
    import torch
    from paper_2511_05534_amd import binding as fb
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    s = 2 if wl.dtype == "bf16" else 4
    Lyr, Hq, Hkv, d, W, batch = wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.batch
    Bs = list(wl.budgets)
    R = max(1, min(Bs) // 4)
    cu_cap = np.concatenate([[0], np.cumsum([B + R for B in Bs])]).astype(np.int32)
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    Kc = torch.randn((Lyr, Hkv, int(cu_cap[-1]), d), generator=gen, device=dev).to(tdt)
    Vc = torch.randn((Lyr, Hkv, int(cu_cap[-1]), d), generator=gen, device=dev).to(tdt)
    k_new = torch.randn((Lyr, Hkv, batch, d), generator=gen, device=dev).to(tdt)
    v_new = torch.randn((Lyr, Hkv, batch, d), generator=gen, device=dev).to(tdt)
    Qw = torch.randn((Lyr, Hq, W, d), generator=gen, device=dev).to(tdt)
    cache = fb.Params(Lyr, Hq, Hkv, d, wl.dtype, [B + R for B in Bs], Bs, [[(0, B + R, 0)] for B in Bs], W, 0.0,
                      [4.0 / B for B in Bs], q_strides=(Hq * W * d, W * d, d))
    plans, ws_bytes = [], 0
    for b in range(batch):
        n, B = Bs[b] + R, Bs[b]
        sizes, ws = fb.flowmm_cache_remerge_sizes(cache, cu_cap, b, n)
        ws_bytes = max(ws_bytes, ws)
        plans.append([torch.empty(sz, dtype=torch.uint8, device=dev) for sz in sizes])
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    lengths = list(Bs)

    def appends():
        for _ in range(R):
            fb.flowmm_cache_append(cache, cu_cap, lengths, Kc.data_ptr(), Vc.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), stream)
            for b in range(batch):
                lengths[b] += 1

    def remerges():
        for b in range(batch):
            fb.flowmm_cache_remerge(cache, cu_cap, lengths, b, Kc.data_ptr(), Vc.data_ptr(), Qw.data_ptr(),
                                    [t.data_ptr() for t in plans[b]], workspace.data_ptr(), ws_bytes, stream)
            lengths[b] = Bs[b]

    cycles = max(1, args.steps // 10)
    for _ in range(max(1, args.warmup // 10)):
        appends(); remerges()
    torch.cuda.synchronize()
    # one more cycle with every kernel bracketed by events: what the GPU spends, apart from the host's enqueueing
    fb.flowmm_profile_select("all")
    appends(); remerges()
    torch.cuda.synchronize()
    prof = fb.flowmm_profile_collect()
    fb.flowmm_profile_select("")
    k_append = 1e3 * prof["cache_append"][0] / max(prof["cache_append"][1], 1)
    k_remerge = {k: 1e3 * ms for k, (ms, n) in prof.items() if n and k != "cache_append"}
    t_app = t_rem = 0.0
    for _ in range(cycles):
        t0 = time.perf_counter()
        appends()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        remerges()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        t_app += t1 - t0
        t_rem += t2 - t1
    us_append = 1e6 * t_app / (cycles * R)
    us_remerge = 1e6 * t_rem / cycles
    units = Lyr * Hkv
    row = d * s
    G = Hq // Hkv
    rem_bytes = sum(units * (3 * (B + R) * row + 2 * B * row + G * W * row + 12 * (B + R)) for B in Bs)
    app_bytes = units * batch * 2 * 2 * row  # the new K and V rows read and written
    per_token = us_append + us_remerge / R
    print(json.dumps({
        "metric": "decode-time maintenance of the compacted cache, microseconds per generated token (appends + re-merge amortised)",
        "value": per_token, "unit": "us/token", "n_gpus": 1, "steps": cycles, "warmup": max(1, args.warmup // 10),
        "ms_per_step": (us_append * R + us_remerge) / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {wl.name}", "layers": Lyr, "q_heads": Hq, "kv_heads": Hkv, "head_dim": d,
                   "budgets": Bs, "head_room": R, "window": W, "entry_point": "flowmm_cache_append + flowmm_cache_remerge",
                   "step": "one cycle: head_room appends, then every sequence back to its budget"},
        "roofline": {"bound": "hbm", "kernel": "re-merge of all sequences (the kernels of flowmm_plan_merge on the cache rows)",
                     "achieved": rem_bytes / (us_remerge * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": rem_bytes / (us_remerge * 1e-6) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": rem_bytes},
        "append": {"us_per_step": us_append, "kernel_us": k_append, "bytes": app_bytes,
                   "note": "a step is one call through the Python binding: its time is the host's, the kernel's is kernel_us"},
        "remerge": {"us_per_cycle": us_remerge, "bytes": rem_bytes, "kernels_us_per_cycle": k_remerge},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3,
                    help="workload 0..4 of BASELINE.json's configs (default 3: the largest that is one sequence on one GPU)")
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
    ap.add_argument("--cache", action="store_true",
                    help="time flowmm_cache_append / flowmm_cache_remerge cycles on compacted caches of this configuration")
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
    if args.cache:
        return bench_cache(args, wl, dev)
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
    # the roofline is reported for the slowest step: a kernel, or the score's group of three
    group_us = {}
    for k, us in kernels_us.items():
        group_us[GROUPS.get(k, k)] = group_us.get(GROUPS.get(k, k), 0.0) + us
    dominant = args.kernel or max(group_us, key=group_us.get)
    members = [k for k in kernels_us if GROUPS.get(k, k) == dominant]
    if not members:
        print(f"no kernel or group named {dominant} ran; choose from {sorted(group_us)}", file=sys.stderr)
        sys.exit(2)
    select_names = ",".join(members)

    if args.graph:
        # the dominant kernel's duration comes from eager steps (events cannot be recorded inside the graph)
        fb.flowmm_profile_select(select_names)
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        dom = fb.flowmm_profile_collect()
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
        # timed region: exactly K steps; only the dominant kernel (or group) carries events
        fb.flowmm_profile_select(select_names)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dom = fb.flowmm_profile_collect()
        fb.flowmm_profile_select("")

    ms_per_step = 1e3 * (t1 - t0) / args.steps
    tokens_per_s = wl.total_tokens / (ms_per_step * 1e-3)
    byt, flops = algorithmic_work(wl)
    dom_us = sum(1e3 * dom[k][0] / dom[k][1] for k in members)  # average duration per launch (per pass for a group)
    traffic, traffic_src = measured_traffic(args.config, members) if not args.layers else (None, None)
    if args.traffic_bytes is not None:
        traffic, traffic_src = args.traffic_bytes, "--traffic-bytes"
    if dominant == "match":
        # the one dense contraction: 2 (L - B) B d flops per (sequence, layer, kv head) against the matrix-core peak
        peak = MFMA_PEAK_TFLOPS[wl.dtype]
        achieved = flops["match"] / (dom_us * 1e-6) / 1e12
        roofline = {"bound": "mfma", "kernel": "match", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                    "frac": achieved / peak, "algorithmic_flops_per_launch": flops["match"]}
    else:
        achieved = byt.get(dominant, 0) / (dom_us * 1e-6) / 1e9
        roofline = {"bound": "hbm", "kernel": "+".join(members), "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "algorithmic_bytes_per_launch": byt.get(dominant, 0)}
    roofline.update({"traffic": traffic, "kernel_us": dom_us,
                     "traffic_source": (f"{traffic_src}: committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of this "
                                        "command, scaled by a plain copy; not measured in this run") if traffic_src else None})
    # every step of the pass against its own bound, from the warm-up's bracketed kernels
    steps_roofline = {}
    for name, us in group_us.items():
        if name == "match":
            steps_roofline[name] = {"bound": "mfma", "us": us, "TFLOPs": flops["match"] / (us * 1e-6) / 1e12,
                                    "frac": flops["match"] / (us * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS[wl.dtype]}
        elif byt.get(name):
            steps_roofline[name] = {"bound": "hbm", "us": us, "GBs": byt[name] / (us * 1e-6) / 1e9,
                                    "frac": byt[name] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
            if name == "score":
                # the same step against the vector units: both heavy passes turn every logit into a
                # probability (fma, v_exp_f32 at a quarter of the rate, add, half a max3: 18 issue cycles per
                # 64 logits and SIMD), flops["score"] / (2 d) logits per pass
                logits = 2 * flops["score"] / (2.0 * wl.head_dim)
                steps_roofline[name]["alu"] = {"logits": logits, "peak_logits_per_s": ALU_PEAK_LOGITS,
                                               "frac": logits / (us * 1e-6) / ALU_PEAK_LOGITS}
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
        "roofline": roofline,
        "full_pass": {"algorithmic_bytes": byt["whole_pass"],
                      "achieved_GBs": byt["whole_pass"] / (ms_per_step * 1e-3) / 1e9,
                      "frac_of_hbm_peak": byt["whole_pass"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "host_enqueue_us_per_step": 1e6 * t_host / args.steps},
        "kernels_us": kernels_us,
        "kernels_us_note": "from warm-up steps in which every kernel is bracketed with events (their sum can exceed the "
                           "timed step, which brackets only the roofline kernel)",
        "steps_roofline": steps_roofline,
    }
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
