"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

from paper_2511_05534_amd import workloads as wl

from parity_utils import ATOL_OUT, Report, bf16_ulp, check_layer, run_gpu, upload

pytestmark = pytest.mark.gpu


def small(name, dtype="bf16", Hq=4, Hkv=2, d=128, W=32, spans=((40, 300, 60),), pct=(15,), seed=11,
          n_layers=2, budgets=None, first_mod=wl.TEXT, theta=0.25, tau_factor=4.0):
    return wl.make_workload(name, dtype, seed, n_layers, Hq, Hkv, d, W, [list(s) for s in spans], list(pct),
                            theta=theta, tau_factor=tau_factor, budgets=budgets, first_mod=first_mod)


SMALL_CASES = {
    "mha_bf16_d128": dict(Hq=2, Hkv=2),
    "gqa_bf16_ragged_tail": dict(Hq=6, Hkv=2, spans=((37, 411, 83),), W=32),
    "f32_d64_w16": dict(dtype="f32", Hq=4, Hkv=4, d=64, W=16, spans=((32, 256, 32),), pct=(20,)),
    "f32_d128": dict(dtype="f32", Hq=2, Hkv=1, d=128, W=8, spans=((20, 200, 19),)),
    "bf16_d64_gqa": dict(Hq=8, Hkv=2, d=64, W=24, spans=((50, 500, 77),)),
    "window_5": dict(Hq=3, Hkv=3, W=5, spans=((16, 180, 33),)),
    "window_40_pads_to_64": dict(Hq=4, Hkv=2, W=40, spans=((30, 520, 90),)),
    "image_tokens_in_window": dict(Hq=4, Hkv=2, W=32, spans=((30, 400, 10, 12),), pct=(12,)),
    "image_first": dict(Hq=2, Hkv=2, W=16, spans=((200, 100),), first_mod=wl.IMAGE),
    "text_only": dict(Hq=2, Hkv=1, W=16, spans=((300,),)),
    "multi_tile_1300": dict(Hq=4, Hkv=1, W=32, spans=((100, 500, 50, 600, 50),), pct=(7,)),
    "batch_of_3": dict(Hq=4, Hkv=2, W=16, spans=((30, 260, 40), (64, 700, 69), (20, 100, 17)), pct=(10, 20, 5)),
    "budget_equals_window": dict(Hq=2, Hkv=2, W=16, spans=((30, 200, 30),), budgets=(16,)),
    "budget_equals_length": dict(Hq=2, Hkv=2, W=16, spans=((30, 200, 30),), budgets=(260,)),
    "pivots_over_one_tile": dict(Hq=2, Hkv=1, W=32, spans=((60, 900, 64),), pct=(30,)),
    "intra_forced": dict(Hq=4, Hkv=2, spans=((40, 300, 60),), theta=2.0),
    "cross_forced": dict(Hq=4, Hkv=2, spans=((40, 300, 60),), theta=-1.0),
    "gate_off": dict(Hq=4, Hkv=2, spans=((40, 300, 60),), tau_factor=float("inf")),
    "gate_drops_everything": dict(Hq=4, Hkv=2, spans=((40, 300, 60),), tau_factor=-1.0),
    "unit_four_tiles_per_wave": dict(Hq=2, Hkv=2, W=32, spans=((60, 880, 60),), pct=(20,)),
    "unit_d64": dict(Hq=2, Hkv=2, d=64, W=24, spans=((50, 500, 77),)),
    "unit_two_row_blocks_gqa": dict(Hq=4, Hkv=2, W=32, spans=((20, 600, 40),), pct=(12,)),
    "shortest": dict(Hq=1, Hkv=1, W=1, spans=((1,),), budgets=(1,), n_layers=1),
    "tiny_3_tokens": dict(Hq=2, Hkv=1, W=2, spans=((1, 2),), budgets=(2,), n_layers=1),
    # the limits of the unit-resident kernels: 1024 tokens, 256 pivots, 8 sequences, 32 spans; and one step beyond
    "unit_limit_1024_tokens_256_pivots": dict(Hq=2, Hkv=1, W=32, spans=((100, 800, 124),), budgets=(256,), n_layers=1),
    "one_token_beyond_the_unit_limit": dict(Hq=2, Hkv=1, W=32, spans=((100, 800, 125),), budgets=(256,), n_layers=1),
    "unit_twelve_tiles": dict(Hq=2, Hkv=2, W=32, spans=((30, 300, 54),), pct=(15,), n_layers=1),
    "unit_batch_of_8": dict(Hq=2, Hkv=1, W=16, n_layers=1, pct=(10, 20, 5, 10, 20, 5, 10, 20),
                            spans=((30, 100, 20), (20, 200, 30), (40, 60, 17), (25, 300, 33), (16,), (50, 400, 50),
                                   (10, 90, 16), (33, 150, 47))),
    "unit_32_spans": dict(Hq=2, Hkv=1, W=16, n_layers=1, pct=(12,), spans=(tuple([20, 10] * 15 + [25, 17]),)),
    "more_spans_than_the_unit_path_takes": dict(Hq=2, Hkv=1, W=16, n_layers=1, pct=(12,),
                                                spans=(tuple([20, 10] * 16 + [25, 17]),)),
    # the top-B split keeps 4, 8 or 16 keys per thread in registers, or none beyond 16384 tokens (then for
    # every sequence of the batch)
    "select_8_keys_per_thread": dict(Hq=2, Hkv=1, d=64, W=16, n_layers=1, pct=(6,), spans=((300, 5000, 700),)),
    "select_16_keys_per_thread": dict(Hq=1, Hkv=1, d=64, W=16, n_layers=1, pct=(4,), spans=((400, 9000, 1100),)),
    "select_keys_from_memory": dict(Hq=1, Hkv=1, d=64, W=16, n_layers=1, pct=(3,), spans=((500, 15000, 1000),)),
    # a budget whose pivot positions do not fit in LDS next to the member-counting table of the merge (one
    # wave then walks the tokens and looks the pivots up in memory)
    "budget_of_19000": dict(Hq=1, Hkv=1, d=64, W=16, n_layers=1, budgets=(19000,), spans=((500, 19000, 800),)),
    "select_long_and_short_in_a_batch": dict(Hq=1, Hkv=1, d=64, W=16, n_layers=1, pct=(3, 10),
                                             spans=((500, 15000, 1000), (40, 300, 60))),
}


@pytest.mark.parametrize("path", ["auto", "generic", "fused"])
@pytest.mark.parametrize("name", list(SMALL_CASES))
def test_small_cases_match_oracle(oracle, name, path):
    """`auto` lets the library pick (short bf16 prompts take the unit-resident kernels); `generic`
    forces the multi-workgroup kernels on the same inputs; `fused` is the one-call entry point
    (short bf16 prompts take the streaming kernel that merges right after matching)."""
    w = small(name, **SMALL_CASES[name])
    print(f"case {name} [{path}]: L={w.seqlens} B={w.budgets} dtype={w.dtype}", flush=True)
    gpu = run_gpu(w, flags=1 if path == "generic" else 0, fused=path == "fused")
    rep = Report()
    for l in range(w.n_layers):
        check_layer(oracle, w, gpu, l, report=rep)
    print(rep, flush=True)


def test_both_paths_agree_on_decisions(oracle):
    """Same kept sets and assignments from the unit-resident and the generic kernels (decisions are
    taken on fp32 numbers that may differ in the last bits, so compare where they are equal); where
    they differ, each side's choice must lie inside the oracle's margin band (check_layer)."""
    w = small("paths", Hq=2, Hkv=2, spans=((35, 576, 64),), pct=(10,), n_layers=3)
    a = run_gpu(w, flags=0)
    b = run_gpu(w, flags=1)
    for l in range(w.n_layers):
        check_layer(oracle, w, a, l)
        check_layer(oracle, w, b, l)
    same_I = (a["importance"] == b["importance"]).mean()
    print(f"identical importances: {same_I:.4f}", flush=True)
    assert np.allclose(a["importance"], b["importance"], rtol=1e-5, atol=0)
    agree = (a["assign"] == b["assign"]).mean()
    assert agree > 0.995, agree
    assert (a["mode"] == b["mode"]).all()


VARIANT_SHAPES = {
    "unit": dict(Hq=4, Hkv=2, spans=((40, 300, 60),)),
    "unit_big_slots": dict(Hq=2, Hkv=2, W=32, spans=((60, 880, 60),), pct=(8,)),
    "unit_d64": dict(Hq=2, Hkv=2, d=64, W=24, spans=((50, 500, 77),)),
    "f32": dict(dtype="f32", Hq=4, Hkv=4, d=64, W=16, spans=((32, 256, 32),), pct=(20,)),
    "f32_d128": dict(dtype="f32", Hq=2, Hkv=1, d=128, W=8, spans=((20, 200, 19),)),
    "multi_tile": dict(Hq=4, Hkv=1, W=32, spans=((100, 500, 50, 600, 50),), pct=(7,)),
    "batch_of_3": dict(Hq=4, Hkv=2, W=16, spans=((30, 260, 40), (64, 700, 69), (20, 100, 17)), pct=(10, 20, 5)),
}


@pytest.mark.parametrize("path", ["auto", "generic", "fused"])
@pytest.mark.parametrize("variant", ["inverted_flow", "weighted_merge", "both"])
@pytest.mark.parametrize("name", list(VARIANT_SHAPES))
def test_ablation_variants_match_oracle(oracle, name, variant, path):
    """The switches of the paper's component ablation: the strategy misaligned with the flow
    (FLOWMM_FLAG_INVERT_FLOW) and the similarity-weighted merge (FLOWMM_FLAG_WEIGHTED_MERGE)."""
    flags = {"inverted_flow": 2, "weighted_merge": 4, "both": 6}[variant]
    for theta in ((0.25, 2.0) if flags & 2 else (0.25,)):  # the inverse of both outcomes of the rule
        w = small(name, theta=theta, **VARIANT_SHAPES[name])
        print(f"case {name} [{variant}, {path}] theta={theta}: L={w.seqlens} B={w.budgets} dtype={w.dtype}", flush=True)
        gpu = run_gpu(w, flags=flags | (1 if path == "generic" else 0), fused=path == "fused")
        if flags & 2:
            assert (gpu["mode"] == (0 if gpu["rho"].min() > theta else 1)).all()
        rep = Report()
        for l in range(w.n_layers):
            check_layer(oracle, w, gpu, l, report=rep, flags=flags)
        print(rep, flush=True)


def test_weighted_merge_of_identical_keys_is_the_uniform_mean(oracle):
    """Every weight is 1 when all keys point the same way: both merge operators must agree with each
    other and with the oracle (every cosine is 1: all assignments are exact ties, any eligible pivot is valid)."""
    import torch
    w = small("same_direction", Hq=2, Hkv=2, spans=((40, 300, 60),), n_layers=1)
    K, V, Q = upload(w)
    direction = torch.randn(w.head_dim, device=K.device).to(K.dtype)
    scale = (1 + torch.arange(K.shape[2], device=K.device) % 4).to(K.dtype)[None, None, :, None]  # exact multiples
    K = (direction[None, None, None, :] * scale).expand_as(K).contiguous()
    host = (K[0].float().cpu().numpy(), V[0].float().cpu().numpy(), Q[0].float().cpu().numpy())
    for flags in (0, 1):
        a = run_gpu(w, tensors=(K, V, Q), flags=flags)
        b = run_gpu(w, tensors=(K, V, Q), flags=flags | 4)
        check_layer(oracle, w, a, 0, tensors_np=host)
        check_layer(oracle, w, b, 0, tensors_np=host, flags=4)
        assert (a["assign"] == b["assign"]).all()
        assert np.allclose(a["V_out"], b["V_out"], rtol=0, atol=2e-2)
        assert np.allclose(a["K_out"], b["K_out"], rtol=0, atol=2e-2 * 4)


FLOW_EXACT_CASES = {
    "mha_one_tile": dict(Hq=2, Hkv=2, spans=((40, 150, 30),)),
    "gqa_three_tiles_ragged": dict(Hq=4, Hkv=2, spans=((37, 411, 83, 120),)),
    "d64": dict(Hq=2, Hkv=2, d=64, W=24, spans=((50, 500, 77),)),
    "f32_d64": dict(dtype="f32", Hq=4, Hkv=4, d=64, W=16, spans=((32, 256, 32),)),
    "f32_d128": dict(dtype="f32", Hq=2, Hkv=1, d=128, W=8, spans=((20, 200, 19, 300),)),
    "image_first": dict(Hq=2, Hkv=2, W=16, spans=((200, 100),), first_mod=wl.IMAGE),
    "text_only": dict(Hq=2, Hkv=1, W=16, spans=((300,),)),
    "many_key_steps": dict(Hq=2, Hkv=1, W=32, spans=((100, 500, 50, 600, 50),)),
    "batch_of_3": dict(Hq=4, Hkv=2, W=16, spans=((30, 260, 40), (64, 700, 69), (20, 100, 17)), pct=(10, 20, 5)),
    "shortest": dict(Hq=1, Hkv=1, W=1, spans=((1,),), budgets=(1,), n_layers=1),
}


@pytest.mark.parametrize("name", list(FLOW_EXACT_CASES))
def test_flow_exact_matches_the_literal_ratio(oracle, name):
    """flowmm_flow_exact against the oracle's score with every token as a proxy (W = L), which a CPU
    pin shows to be the paper's rho equation evaluated on the dense L x L attention matrix."""
    import torch
    from paper_2511_05534_amd import binding as fb
    w = small(name, **FLOW_EXACT_CASES[name])
    print(f"case {name}: L={w.seqlens} dtype={w.dtype}", flush=True)
    K, V, Q = upload(w)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    qf_np = [w.layer_queries_full(l) for l in range(w.n_layers)]
    Qf = torch.stack([torch.from_numpy(q) for q in qf_np]).to("cuda:0").to(tdt)
    for theta, flags in ((w.theta, 0), (0.05, 2)):
        params = fb.Params.from_workload(w, theta=theta, flags=flags)
        bufs = fb.DeviceBuffers(params)
        bufs.rho.fill_(-1.0)
        bufs.mode.fill_(-1)
        bufs.flow_exact(K, Qf, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        rho_g, mode_g = bufs.rho.cpu().numpy(), bufs.mode.cpu().numpy()
        cu = w.cu_seqlens
        for l in range(w.n_layers):
            Kl = w.layer_tensors(l)[0]
            for b in range(w.batch):
                sl = slice(int(cu[b]), int(cu[b + 1]))
                _, cross = oracle.score(Kl[:, sl], qf_np[l][:, sl], w.modality(b))  # W = L: every token is a query
                rho_o, mode_o = oracle.flow(cross, theta, invert=bool(flags & 2))
                assert abs(rho_g[l, b] - rho_o) <= 2e-4 * max(rho_o, 1e-6) + 1e-7, (l, b, rho_g[l, b], rho_o)
                if abs(rho_o - theta) > 1e-3 * abs(theta):
                    assert mode_g[l, b] == mode_o


DECODE_CASES = {
    "mha_small": dict(Hq=2, Hkv=2, spans=((40, 150, 30),)),
    "gqa_2": dict(Hq=4, Hkv=2, spans=((37, 411, 83),)),
    "gqa_7_like_qwen2": dict(Hq=7, Hkv=1, W=8, spans=((50, 400, 62),), pct=(20,)),
    "gqa_12_two_batches_of_heads": dict(Hq=12, Hkv=1, W=4, spans=((30, 200, 26),), pct=(20,)),
    "d64": dict(Hq=2, Hkv=2, d=64, W=24, spans=((50, 500, 77),)),
    "f32_d64": dict(dtype="f32", Hq=4, Hkv=4, d=64, W=16, spans=((32, 256, 32),), pct=(20,)),
    "f32_d128": dict(dtype="f32", Hq=2, Hkv=1, d=128, W=8, spans=((20, 200, 19),)),
    "many_slots_split_ranges": dict(Hq=4, Hkv=1, W=32, spans=((100, 2500, 50, 1600, 50),), pct=(30,), n_layers=1),
    "batch_of_3": dict(Hq=4, Hkv=2, W=16, spans=((30, 260, 40), (64, 700, 69), (20, 100, 17)), pct=(10, 20, 5)),
    "one_slot": dict(Hq=1, Hkv=1, W=1, spans=((1,),), budgets=(1,), n_layers=1),
}


@pytest.mark.parametrize("name", list(DECODE_CASES))
def test_decode_attention_over_the_compacted_cache(oracle, name):
    """flowmm_decode_attention on the cache flowmm_plan_merge has just written, against the oracle's
    softmax attention over the same merged rows (max-abs error as for the merged rows themselves)."""
    import torch
    w = small(name, **DECODE_CASES[name])
    print(f"case {name}: L={w.seqlens} B={w.budgets} dtype={w.dtype} G={w.group}", flush=True)
    from paper_2511_05534_amd import binding as fb
    K, V, Q = upload(w)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    params = fb.Params.from_workload(w)
    bufs = fb.DeviceBuffers(params)
    bufs.plan_merge(K, V, Q)
    gen = torch.Generator(device="cuda:0").manual_seed(5)
    q = torch.randn((w.n_layers, w.n_q_heads, w.batch, w.head_dim), generator=gen, device="cuda:0").to(tdt)
    out = torch.full_like(q, float("nan"))
    bufs.decode_attention(q, out, stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    Kc, Vc = bufs.K_out.float().cpu().numpy(), bufs.V_out.float().cpu().numpy()
    qn, got = q.float().cpu().numpy(), out.float().cpu().numpy()
    assert np.isfinite(got).all()
    cuk, G = w.cu_kept, w.group
    worst = 0.0
    for l in range(w.n_layers):
        for g in range(w.n_kv_heads):
            for b in range(w.batch):
                rows = slice(int(cuk[b]), int(cuk[b + 1]))
                want = oracle.decode_attention(qn[l, g * G:(g + 1) * G, b], Kc[l, g, rows], Vc[l, g, rows])
                err = np.abs(got[l, g * G:(g + 1) * G, b] - want)
                tol = np.full(want.shape, ATOL_OUT[w.dtype])
                if w.dtype == "bf16":
                    tol = np.maximum(tol, bf16_ulp(want))
                assert (err <= tol).all(), (l, g, b, err.max())
                worst = max(worst, float(err.max()))
    print(f"max abs error {worst:.2e}", flush=True)


def _random_case(rng, i):
    """A seeded random small shape: lengths, spans, window, budgets, head grouping, dtype, path and flags."""
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.integers(1, 3))
    G = int(rng.choice([1, 1, 2, 3])) if dtype == "bf16" else int(rng.choice([1, 2]))
    batch = int(rng.choice([1, 1, 1, 2, 3]))
    W = int(rng.integers(1, 41))
    spans, budgets = [], []
    for _ in range(batch):
        n_spans = int(rng.integers(1, 6))
        lens = [int(rng.integers(1, 260)) for _ in range(n_spans)]
        L = sum(lens)
        if L < W:
            lens[-1] += W - L
            L = W
        spans.append(tuple(lens))
        budgets.append(int(rng.integers(W, L + 1)))
    flags = int(rng.choice([0, 0, 2, 4, 6]))
    path = str(rng.choice(["auto", "generic", "fused"]))
    theta = float(rng.choice([0.25, 0.25, -1.0, 2.0]))
    tau_factor = float(rng.choice([4.0, 4.0, 1.0, float("inf")]))
    w = wl.make_workload(f"random{i}", dtype, 1000 + i, int(rng.integers(1, 3)), Hkv * G, Hkv, d, W,
                         [list(sp) for sp in spans], [10] * batch, theta=theta, tau_factor=tau_factor, budgets=budgets,
                         first_mod=int(rng.integers(0, 2)))
    return w, flags, path


@pytest.mark.parametrize("block", range(4))
def test_random_shapes_match_oracle(oracle, block):
    """Forty seeded random shapes (ten per block) through a random path and random variant flags."""
    rng = np.random.default_rng(2511_05534 + block)
    for i in range(10):
        w, flags, path = _random_case(rng, 10 * block + i)
        print(f"random case {10 * block + i} [{path}, flags={flags}]: L={w.seqlens} B={w.budgets} W={w.window} "
              f"Hq={w.n_q_heads} Hkv={w.n_kv_heads} d={w.head_dim} {w.dtype} theta={w.theta}", flush=True)
        gpu = run_gpu(w, flags=flags | (1 if path == "generic" else 0), fused=path == "fused")
        for l in range(w.n_layers):
            check_layer(oracle, w, gpu, l, flags=flags)


def test_hip_graph_replay_equals_eager():
    """The library neither allocates nor synchronises, so its calls can be captured into a HIP graph:
    every replay (with eager work and synchronisation in between) must reproduce the eager result."""
    import torch
    from paper_2511_05534_amd import binding as fb
    for name, flags in (("graph_unit", 0), ("graph_generic", 1)):
        w = small(name, Hq=4, Hkv=2, spans=((37, 411, 83),), n_layers=3)
        K, V, Q = upload(w)
        params = fb.Params.from_workload(w, flags=flags)
        eager = fb.DeviceBuffers(params)
        eager.plan_merge(K, V, Q, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want = {n: getattr(eager, n).clone() for n in fb.PLAN_FIELDS + ("K_out", "V_out")}
        bufs = fb.DeviceBuffers(params)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            bufs.plan_merge(K, V, Q, side.cuda_stream)  # warm-up outside the capture (function attributes, lazy loading)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            bufs.plan_merge(K, V, Q, torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            for n in fb.PLAN_FIELDS + ("K_out", "V_out"):
                getattr(bufs, n).fill_(0)
            scratch = torch.randn(1 << 20, device="cuda:0").sum().item()  # unrelated eager work and a synchronisation
            graph.replay()
            torch.cuda.synchronize()
            for n in fb.PLAN_FIELDS + ("K_out", "V_out"):
                assert torch.equal(getattr(bufs, n), want[n]), (name, rep, n)


def test_one_call_equals_two_calls(oracle):
    """flowmm_plan_merge against flowmm_plan + flowmm_merge: the same decisions up to the last bits of
    the importances (the two spread the key tiles over their waves differently), and bit-identical
    merged rows wherever the decisions are the same (both merge alike); where the decisions differ,
    each side's choice must lie inside the oracle's margin band (check_layer)."""
    for theta in (0.25, 2.0):
        w = small("onecall", Hq=4, Hkv=2, spans=((35, 576, 64),), pct=(10,), n_layers=3, theta=theta)
        a = run_gpu(w)
        b = run_gpu(w, fused=True)
        for l in range(w.n_layers):
            check_layer(oracle, w, a, l)
            check_layer(oracle, w, b, l)
        assert np.allclose(a["importance"], b["importance"], rtol=1e-5, atol=0)
        assert (a["mode"] == b["mode"]).all() and np.allclose(a["rho"], b["rho"], rtol=1e-5, atol=0)
        agree = (a["assign"] == b["assign"]).mean()
        assert agree > 0.995, agree
        same = (a["assign"] == b["assign"]).all(axis=-1) & (a["kept_idx"] == b["kept_idx"]).all(axis=-1)
        assert (a["K_out"][same] == b["K_out"][same]).all() and (a["V_out"][same] == b["V_out"][same]).all()
        c = run_gpu(w, fused=True)
        for k in b:
            assert (b[k] == c[k]).all() or np.array_equal(b[k], c[k], equal_nan=True), k


def test_config1_generic_path_sampled(oracle):
    w = wl.config(1, n_layers=2)
    gpu = run_gpu(w, flags=1)
    rep = check_layer(oracle, w, gpu, 1, kv_heads=[3, 30])
    print(rep, flush=True)


def test_config0_tiny_f32(oracle):
    w = wl.config(0)
    gpu = run_gpu(w)
    rep = check_layer(oracle, w, gpu, 0)
    print(rep, flush=True)
    for theta in (-1.0, 2.0):
        g2 = run_gpu(w, theta=theta)
        assert (g2["mode"] == (1 if theta < 0 else 0)).all()
        check_layer(oracle, w, g2, 0, theta=theta)


def test_invariants_and_determinism():
    w = small("inv", Hq=4, Hkv=2, spans=((37, 411, 83),), n_layers=3)
    a = run_gpu(w)
    b = run_gpu(w)
    for k in a:
        assert (a[k].view(np.uint32) == b[k].view(np.uint32)).all() if a[k].dtype == np.float32 else (a[k] == b[k]).all(), k
    L, B = w.seqlens[0], w.budgets[0]
    for l in range(w.n_layers):
        for g in range(w.n_kv_heads):
            assert abs(a["importance"][l][g].astype(np.float64).sum() - 1.0) < 1e-4
            kept = a["kept_idx"][l][g]
            asg = a["assign"][l][g]
            assert len(set(kept.tolist())) == B
            assert ((asg >= -1) & (asg < B)).all()
            assert (asg[kept] == np.arange(B)).all()


def test_full_budget_leaves_the_cache_unchanged():
    w = small("full", Hq=2, Hkv=2, W=16, spans=((30, 200, 30),), budgets=(260,))
    K, V, Q = upload(w)
    gpu = run_gpu(w, tensors=(K, V, Q))
    assert (gpu["K_out"] == K.float().cpu().numpy()).all()
    assert (gpu["V_out"] == V.float().cpu().numpy()).all()
    assert (gpu["n_dropped"] == 0).all()


def test_packed_token_major_layout(oracle):
    """The same cache stored [T][Hkv][d] (varlen layout) through the stride arguments."""
    import torch
    from paper_2511_05534_amd import binding as fb
    w = small("strided", Hq=4, Hkv=2, spans=((37, 300, 40),), n_layers=2)
    K, V, Q = upload(w)
    ref = run_gpu(w, tensors=(K, V, Q))
    Lyr, Hkv, T, d = K.shape
    Kt = K.permute(0, 2, 1, 3).contiguous()  # [Lyr][T][Hkv][d]
    Vt = V.permute(0, 2, 1, 3).contiguous()
    params = fb.Params(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, w.seqlens, w.budgets,
                       w.spans, w.window, w.theta, w.tau, k_strides=(T * Hkv * d, d, Hkv * d))
    bufs = fb.DeviceBuffers(params)
    bufs.plan(Kt, Q)
    bufs.merge(Kt, Vt)
    torch.cuda.synchronize()
    assert (bufs.assign.cpu().numpy() == ref["assign"]).all()
    assert (bufs.K_out.float().cpu().numpy() == ref["K_out"]).all()
    assert (bufs.V_out.float().cpu().numpy() == ref["V_out"]).all()


def test_ragged_batch_equals_each_sequence_alone():
    w = small("batch", Hq=4, Hkv=2, W=16, spans=((30, 260, 40), (64, 700, 69), (20, 100, 17)), pct=(10, 20, 5))
    K, V, Q = upload(w)
    full = run_gpu(w, tensors=(K, V, Q))
    cu, cuk, W = w.cu_seqlens, w.cu_kept, w.window
    for b in range(w.batch):
        one = wl.Workload(name="one", dtype=w.dtype, seed=w.seed, n_layers=w.n_layers, n_q_heads=w.n_q_heads,
                          n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, window=W, seqlens=[w.seqlens[b]],
                          budgets=[w.budgets[b]], spans=[w.spans[b]], span_mu=[w.span_mu[b]], sinks=[w.sinks[b]],
                          theta=w.theta, tau=[w.tau[b]])
        t = (K[:, :, cu[b]:cu[b + 1]].contiguous(), V[:, :, cu[b]:cu[b + 1]].contiguous(),
             Q[:, :, b * W:(b + 1) * W].contiguous())
        alone = run_gpu(one, tensors=t)
        assert (alone["assign"] == full["assign"][:, :, cu[b]:cu[b + 1]]).all()
        assert (alone["kept_idx"] == full["kept_idx"][:, :, cuk[b]:cuk[b + 1]]).all()
        assert (alone["K_out"] == full["K_out"][:, :, cuk[b]:cuk[b + 1]]).all()
        assert (alone["V_out"] == full["V_out"][:, :, cuk[b]:cuk[b + 1]]).all()
        # the workgroup shape follows the longest sequence of the call, and with it the order in which the
        # row statistics of the softmax are folded: the last bits of rho may differ
        assert np.allclose(alone["rho"][:, 0], full["rho"][:, b], rtol=1e-5, atol=0)


def _whole_result_invariants(w, gpu):
    """Properties that hold at any size, over every layer, head and sequence of a result."""
    cu, cuk = w.cu_seqlens, w.cu_kept
    for b in range(w.batch):
        L, B = w.seqlens[b], w.budgets[b]
        imp = gpu["importance"][:, :, cu[b]:cu[b + 1]].astype(np.float64)
        assert np.abs(imp.sum(axis=-1) - 1.0).max() < 1e-3
        kept = gpu["kept_idx"][:, :, cuk[b]:cuk[b + 1]]
        assert (np.diff(kept, axis=-1) > 0).all() and kept.min() >= 0 and kept.max() < L
        assert (kept[:, :, B - w.window:] == np.arange(L - w.window, L)).all(), "a proxy token was evicted"
        asg = gpu["assign"][:, :, cu[b]:cu[b + 1]]
        assert ((asg >= -1) & (asg < B)).all()
        own = np.take_along_axis(asg, kept, axis=-1)
        assert (own == np.arange(B)).all()
        assert ((asg == -1).sum(axis=-1) == gpu["n_dropped"][:, :, b]).all()
        assert np.isfinite(gpu["K_out"][:, :, cuk[b]:cuk[b + 1]]).all() and np.isfinite(gpu["V_out"][:, :, cuk[b]:cuk[b + 1]]).all()


# (layer, kv heads) samples: the first, a middle and the last layer, two kv heads each
FULL_DEPTH = {
    1: dict(sample=[(0, [0, 17]), (15, [9, 31]), (31, [5, 22])], seqs=None),
    2: dict(sample=[(0, [0, 3]), (13, [1, 2]), (27, [0, 2])], seqs=None),
    3: dict(sample=[(0, [2, 7]), (16, [0, 5]), (31, [3, 6])], seqs=None),
    4: dict(sample=[(0, [1, 2]), (14, [0, 3]), (27, [1, 3])], seqs="ends"),
}


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_benchmark_configs_full_depth_sampled_units(oracle, cfg):
    """The benchmark configurations at their full depth, through flowmm_plan_merge as bench.py runs them:
    sampled (layer, kv head) units against the oracle one by one, properties of the whole result.
    Run twice on the same cache: with the default theta (0.25 selects the cross-modal strategy on these
    inputs) and with theta = 2, which forces the intra-modal one, so the class-split match and the two
    pivot lists per unit are compared at full size too.  Config 4 checks both ends of the batch and its
    shortest and longest sequence."""
    w = wl.config(cfg)
    spec = FULL_DEPTH[cfg]
    tensors = upload(w)
    seqs = None
    if spec["seqs"] == "ends":
        seqs = sorted({0, w.batch - 1, int(np.argmin(w.seqlens)), int(np.argmax(w.seqlens))})
    for theta in (None, 2.0):
        print(f"config {cfg}: {w.name} layers={w.n_layers} T={w.total_tokens} theta={theta}", flush=True)
        gpu = run_gpu(w, theta=theta, tensors=tensors, fused=True)
        assert (gpu["mode"] == (0 if theta is not None else 1)).all()
        rep = Report()
        for layer, heads in spec["sample"]:
            check_layer(oracle, w, gpu, layer, theta=theta, kv_heads=heads, seqs=seqs, report=rep)
            print(f"  layer {layer} heads {heads} seqs {seqs}: {rep}", flush=True)
        _whole_result_invariants(w, gpu)


def test_config1_two_calls_full_depth(oracle):
    """The short-prompt configuration through flowmm_plan + flowmm_merge (three unit-resident launches)."""
    w = wl.config(1)
    gpu = run_gpu(w, fused=False)
    rep = Report()
    for layer, heads in [(0, [0, 17]), (31, [5])]:
        check_layer(oracle, w, gpu, layer, kv_heads=heads, report=rep)
    print(rep, flush=True)
    _whole_result_invariants(w, gpu)


def _planted_edge_rows(w, layer):
    """Layer tensors of `w` with the degenerate rows the method has to cope with planted into K:
    zero-norm keys among the evicted tokens and among the pivots (the proxy tokens are always pivots),
    evicted keys that are exact positive multiples of a pivot's key (cosine 1), pivots with identical
    keys (every token that prefers them sees an exact tie), evicted duplicates of each other, and an
    image-span key that is a multiple of a text pivot (eligible only in a cross-modal layer)."""
    K, V, Q = (x.copy() for x in w.layer_tensors(layer))
    L = w.seqlens[0]
    piv_a, piv_b, piv_dup, piv_zero = L - 5, L - 9, L - 12, L - 3
    K[:, piv_zero] = 0.0                      # zero-norm pivot
    K[:, piv_dup] = K[:, piv_b]               # two pivots with the same key
    K[:, 60] = 0.0                            # zero-norm keys in the body (image span)
    K[:, 61] = 0.0
    K[:, 10] = 0.0                            # ... and in the leading text span
    for i in (70, 150, 333):                  # image-span tokens: multiples of a text pivot
        K[:, i] = 0.5 * K[:, piv_a]
    for i in (5, 20):                         # text tokens: multiples of a text pivot
        K[:, i] = 0.25 * K[:, piv_a]
    for i in (15, 90, 200):                   # exact ties between the two identical pivots
        K[:, i] = 0.5 * K[:, piv_b]
    K[:, 101] = K[:, 100]                     # duplicated body keys (equal importances, equal matches)
    K[:, 103] = K[:, 100]
    return K, V, Q, dict(piv_a=piv_a, piv_b=piv_b, piv_dup=piv_dup, piv_zero=piv_zero)


@pytest.mark.parametrize("theta", [-1.0, 2.0], ids=["cross", "intra"])
@pytest.mark.parametrize("path", ["auto", "generic", "fused"])
def test_planted_zero_rows_multiples_and_ties(oracle, path, theta):
    import torch
    w = small("edge_rows", Hq=4, Hkv=2, W=32, spans=((40, 560, 100),), pct=(15,), n_layers=2, theta=theta)
    L, B = w.seqlens[0], w.budgets[0]
    host = [_planted_edge_rows(w, l) for l in range(w.n_layers)]
    tdt = torch.bfloat16
    K, V, Q = (torch.stack([torch.from_numpy(h[i]) for h in host]).to("cuda:0").to(tdt) for i in range(3))
    gpu = run_gpu(w, tensors=(K, V, Q), flags=1 if path == "generic" else 0, fused=path == "fused")
    rep = Report()
    for l in range(w.n_layers):
        Kl, Vl, Ql, where = host[l]
        check_layer(oracle, w, gpu, l, report=rep, tensors_np=(Kl, Vl, Ql))
        for g in range(w.n_kv_heads):
            kept, asg = gpu["kept_idx"][l][g], gpu["assign"][l][g]
            slot = {int(t): s for s, t in enumerate(kept)}
            is_kept = np.zeros(L, dtype=bool)
            is_kept[kept] = True
            # the planted roles did come out as planned (otherwise the case would test nothing)
            assert not is_kept[[60, 61, 10]].any(), "a zero-norm body key became a pivot"
            assert not is_kept[[5, 20, 15, 90, 200]].any()
            # a multiple of an eligible pivot goes to that pivot (text tokens in both strategies,
            # image-span tokens only when the layer merges across modalities)
            for i in (5, 20):
                assert asg[i] == slot[where["piv_a"]]
            for i in (70, 150, 333):
                if not is_kept[i] and theta < 0:
                    assert asg[i] == slot[where["piv_a"]]
                if not is_kept[i] and theta > 1:
                    assert asg[i] == -1 or w.modality(0)[kept[asg[i]]] == 1
            # an exact tie between identical pivots: either is right (the oracle takes the lower slot)
            for i in (15,):
                assert asg[i] in (slot[where["piv_b"]], slot[where["piv_dup"]])
            # duplicated evicted keys match alike
            if not is_kept[[100, 101, 103]].any():
                assert asg[100] == asg[101] == asg[103]
            # a zero-norm evicted key has cosine 0 with every pivot: any eligible slot is a tie; it must not be dropped
            assert asg[10] >= 0
    print(rep, flush=True)


CACHE_CASES = {
    # prefill shape, head room R per sequence, sequence to re-merge, flags of the re-merge
    "short_unit_path": dict(shape=dict(Hq=4, Hkv=2, W=16, spans=((40, 300, 60),), pct=(15,)), R=24, seq=0, flags=0),
    "short_generic_kernels": dict(shape=dict(Hq=4, Hkv=2, W=16, spans=((40, 300, 60),), pct=(15,)), R=24, seq=0, flags=1),
    "many_rows_gqa": dict(shape=dict(Hq=6, Hkv=2, W=32, spans=((100, 2300, 50, 1700, 77),), pct=(30,), n_layers=1), R=200, seq=0, flags=0),
    "f32_d64": dict(shape=dict(dtype="f32", Hq=4, Hkv=4, d=64, W=8, spans=((32, 256, 32),), pct=(20,)), R=19, seq=0, flags=0),
    "batch_of_3_middle_sequence": dict(shape=dict(Hq=4, Hkv=2, W=16, spans=((30, 260, 40), (64, 700, 69), (20, 100, 17)),
                                                  pct=(10, 20, 15)), R=33, seq=1, flags=0),
    "weighted_merge": dict(shape=dict(Hq=2, Hkv=2, W=8, spans=((30, 400, 50),), pct=(10,)), R=40, seq=0, flags=4),
}


@pytest.mark.parametrize("name", list(CACHE_CASES))
def test_cache_append_and_remerge(oracle, name):
    """Decode-time maintenance through the C ABI: flowmm_cache_append (cache-append equation of the
    Preliminary section) fills the head room behind the merged prompt rows token by token, bit-exact
    against the oracle's append; flowmm_cache_remerge compresses one sequence back to its budget and is
    compared stage by stage with the oracle run on the same cache rows as a single-modality prompt."""
    import torch
    from paper_2511_05534_amd import binding as fb
    case = CACHE_CASES[name]
    w = small(name, **case["shape"])
    R, seq, flags = case["R"], case["seq"], case["flags"]
    dev, tdt = "cuda:0", (torch.bfloat16 if w.dtype == "bf16" else torch.float32)
    Lyr, Hq, Hkv, d, W, batch = w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.window, w.batch
    K, V, Q = upload(w)
    pre = fb.DeviceBuffers(fb.Params.from_workload(w))
    pre.plan_merge(K, V, Q)
    # the cache: per sequence its merged prompt rows and R rows of head room
    Bs = list(w.budgets)
    cu_cap = np.concatenate([[0], np.cumsum([B + R for B in Bs])]).astype(np.int32)
    cuk = w.cu_kept
    Kc = torch.full((Lyr, Hkv, int(cu_cap[-1]), d), 3.0, dtype=tdt, device=dev)
    Vc = torch.full_like(Kc, -3.0)
    for b in range(batch):
        Kc[:, :, cu_cap[b]:cu_cap[b] + Bs[b]] = pre.K_out[:, :, cuk[b]:cuk[b + 1]]
        Vc[:, :, cu_cap[b]:cu_cap[b] + Bs[b]] = pre.V_out[:, :, cuk[b]:cuk[b + 1]]
    tau = [4.0 / B for B in Bs]
    cache = fb.Params(Lyr, Hq, Hkv, d, w.dtype, [B + R for B in Bs], Bs, [[(0, B + R, 0)] for B in Bs], W, 0.0, tau,
                      q_strides=(Hq * W * d, W * d, d), flags=flags)
    # host mirror of the cache, maintained by the oracle
    mirror_k, mirror_v = Kc.float().cpu().numpy(), Vc.float().cpu().numpy()
    lengths = list(Bs)
    gen = torch.Generator(device=dev).manual_seed(123)
    for step in range(R):
        k_new = torch.randn((Lyr, Hkv, batch, d), generator=gen, device=dev).to(tdt)
        v_new = torch.randn((Lyr, Hkv, batch, d), generator=gen, device=dev).to(tdt)
        fb.flowmm_cache_append(cache, cu_cap, lengths, Kc.data_ptr(), Vc.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                               torch.cuda.current_stream().cuda_stream)
        kh, vh = k_new.float().cpu().numpy(), v_new.float().cpu().numpy()
        for b in range(batch):
            for l in range(Lyr):
                mk = np.ascontiguousarray(mirror_k[l][:, cu_cap[b]:cu_cap[b + 1]])
                mv = np.ascontiguousarray(mirror_v[l][:, cu_cap[b]:cu_cap[b + 1]])
                assert oracle.cache_append(mk, mv, lengths[b], kh[l][:, b], vh[l][:, b]) == lengths[b] + 1
                mirror_k[l][:, cu_cap[b]:cu_cap[b + 1]] = mk
                mirror_v[l][:, cu_cap[b]:cu_cap[b + 1]] = mv
            lengths[b] += 1
    torch.cuda.synchronize()
    assert (Kc.float().cpu().numpy() == mirror_k).all() and (Vc.float().cpu().numpy() == mirror_v).all()
    # every sequence is full now: one more append is refused on the host
    with pytest.raises(fb.FlowMMError) as ei:
        fb.flowmm_cache_append(cache, cu_cap, lengths, Kc.data_ptr(), Vc.data_ptr(), k_new.data_ptr(), v_new.data_ptr())
    assert ei.value.status == fb.FLOWMM_EINVAL and "full" in ei.value.message

    # re-merge one sequence
    n, B = lengths[seq], Bs[seq]
    Qw = torch.randn((Lyr, Hq, W, d), generator=gen, device=dev).to(tdt)
    sizes, ws_bytes = fb.flowmm_cache_remerge_sizes(cache, cu_cap, seq, n)
    assert sizes[0] == Lyr * Hkv * n * 4 and sizes[3] == Lyr * Hkv * B * 4
    plan = {"importance": torch.empty((Lyr, Hkv, n), dtype=torch.float32, device=dev),
            "rho": torch.empty((Lyr, 1), dtype=torch.float32, device=dev),
            "mode": torch.empty((Lyr, 1), dtype=torch.int32, device=dev),
            "kept_idx": torch.empty((Lyr, Hkv, B), dtype=torch.int32, device=dev),
            "assign": torch.empty((Lyr, Hkv, n), dtype=torch.int32, device=dev),
            "n_dropped": torch.empty((Lyr, Hkv, 1), dtype=torch.int32, device=dev)}
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    fb.flowmm_cache_remerge(cache, cu_cap, lengths, seq, Kc.data_ptr(), Vc.data_ptr(), Qw.data_ptr(),
                            [plan[f].data_ptr() for f in fb.PLAN_FIELDS], workspace.data_ptr(), ws_bytes,
                            torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    after_k, after_v = Kc.float().cpu().numpy(), Vc.float().cpu().numpy()
    lo, hi = int(cu_cap[seq]), int(cu_cap[seq + 1])
    # nothing outside rows [0, B) of the sequence's range has changed
    keep = np.ones(after_k.shape[2], dtype=bool)
    keep[lo:lo + B] = False
    assert (after_k[:, :, keep] == mirror_k[:, :, keep]).all() and (after_v[:, :, keep] == mirror_v[:, :, keep]).all()
    # the plan and the merged rows against the oracle on the same cache rows (one modality, the last W rows are the proxies)
    as_prompt = wl.make_workload("cache_rows", w.dtype, 0, Lyr, Hq, Hkv, d, W, [[n]], [100], theta=-1.0, budgets=[B])
    as_prompt.tau = [tau[seq]]
    gpu = {f: plan[f].cpu().numpy() for f in fb.PLAN_FIELDS}
    gpu["K_out"], gpu["V_out"] = after_k[:, :, lo:lo + B], after_v[:, :, lo:lo + B]
    qh = Qw.float().cpu().numpy()
    rep = Report()
    for l in range(Lyr):
        rows_k = np.ascontiguousarray(mirror_k[l][:, lo:lo + n])
        rows_v = np.ascontiguousarray(mirror_v[l][:, lo:lo + n])
        check_layer(oracle, as_prompt, gpu, l, report=rep, tensors_np=(rows_k, rows_v, qh[l]), flags=flags & 4)
        assert gpu["rho"][l][0] == 0.0
        if not flags & 4:
            # the oracle's own re-merge from the GPU's decisions is covered by check_layer; its bookkeeping here
            mk, mv = rows_k.copy(), rows_v.copy()
            _, new_len = oracle.cache_remerge(mk, mv, n, qh[l], B, w.dtype, tau[seq])
            assert new_len == B
    print(rep, flush=True)
    # the books: the sequence is back at its budget and takes tokens again
    lengths[seq] = B
    others_full = [b for b in range(batch) if b != seq]
    if not others_full:
        fb.flowmm_cache_append(cache, cu_cap, lengths, Kc.data_ptr(), Vc.data_ptr(), k_new.data_ptr(), v_new.data_ptr())
        torch.cuda.synchronize()
        assert torch.equal(Kc[:, :, lo + B], k_new[:, :, seq]) and torch.equal(Vc[:, :, lo + B], v_new[:, :, seq])
