"""Seeded synthetic KV-cache workloads.

This module only *draws inputs*: sequence layouts, modality spans, budgets and
the K / V / Q-window tensors.  It contains none of the method's arithmetic, so
both the CPU oracle's tests and the HIP path's tests may import it.

The caches stand in for the multi-image long-context prompts the paper
evaluates on (its experimental-settings section: many images per sample, a few
hundred words of text, cache budgets from 5 % to 60 %): image tokens make up
most of the context, the question text sits at the end, and a handful of
high-norm "sink" keys attract most of the attention mass.

Recipe (per sequence):
  * spans alternate text / image; text tokens are N(0,1), image tokens are
    mu_span + 0.8*N(0,1) (applied to K and V);
  * round(0.01*L) sink positions are drawn without replacement from
    [0, L-W), shared by all layers and heads; the K rows (not V) there are
    multiplied by 8;
  * Q-window rows are N(0,1) (the window is text in every configuration);
  * every tensor is rounded (nearest-even) to the workload's dtype before
    anybody sees it; arrays are handed out as float32 holding exactly those
    values.
Each (layer, tensor) has its own generator stream, so single layers can be
drawn without drawing the whole cache.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

TEXT, IMAGE = 0, 1


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def budget_tokens(L: int, pct: int, W: int) -> int:
    """Integer round-half-up of pct % of L, clamped to [W, L]."""
    return int(min(L, max(W, (L * pct + 50) // 100)))


@dataclass
class Workload:
    name: str
    dtype: str  # "bf16" | "f32"
    seed: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    seqlens: List[int]
    budgets: List[int]  # kept tokens per sequence
    spans: List[List[Tuple[int, int, int]]]  # per sequence: (begin, end, modality)
    span_mu: List[List[float]]  # per sequence, per span: mean offset (0 for text)
    sinks: List[np.ndarray]  # per sequence: sink positions
    theta: float = 0.25
    tau: List[float] = field(default_factory=list)
    image_scale: float = 0.8
    sink_gain: float = 8.0

    # ---- layout helpers -------------------------------------------------
    @property
    def batch(self) -> int:
        return len(self.seqlens)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)

    @property
    def cu_kept(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.budgets)]).astype(np.int32)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def modality(self, b: int) -> np.ndarray:
        """int32 modality label of every token of sequence b."""
        m = np.zeros(self.seqlens[b], dtype=np.int32)
        for (s, e, mod) in self.spans[b]:
            m[s:e] = mod
        return m

    def seq_slice(self, b: int) -> slice:
        cu = self.cu_seqlens
        return slice(int(cu[b]), int(cu[b + 1]))

    # ---- tensors --------------------------------------------------------
    def _round(self, x: np.ndarray) -> np.ndarray:
        if self.dtype == "bf16":
            return round_to_bf16(x)
        return np.ascontiguousarray(x, dtype=np.float32)

    def _token_affine(self):
        T = self.total_tokens
        mu = np.zeros(T, dtype=np.float32)
        sc = np.ones(T, dtype=np.float32)
        gain = np.ones(T, dtype=np.float32)
        cu = self.cu_seqlens
        for b in range(self.batch):
            for (s, e, mod), m in zip(self.spans[b], self.span_mu[b]):
                if mod == IMAGE:
                    mu[cu[b] + s:cu[b] + e] = m
                    sc[cu[b] + s:cu[b] + e] = self.image_scale
            gain[cu[b] + np.asarray(self.sinks[b], dtype=np.int64)] = self.sink_gain
        return mu, sc, gain

    def layer_tensors(self, layer: int):
        """K [Hkv][T][d], V [Hkv][T][d], Q [Hq][batch*W][d]; float32 arrays of dtype-rounded values."""
        T, d = self.total_tokens, self.head_dim
        mu, sc, gain = self._token_affine()
        out = []
        for tensor_id in (0, 1):
            rng = np.random.default_rng([self.seed, layer, tensor_id])
            x = rng.standard_normal((self.n_kv_heads, T, d), dtype=np.float32)
            x *= sc[None, :, None]
            x += mu[None, :, None]
            if tensor_id == 0:
                x *= gain[None, :, None]
            out.append(self._round(x))
        rng = np.random.default_rng([self.seed, layer, 2])
        q = rng.standard_normal((self.n_q_heads, self.batch * self.window, d), dtype=np.float32)
        out.append(self._round(q))
        return tuple(out)

    def layer_queries_full(self, layer: int):
        """Queries of EVERY prompt token, Q_full [Hq][T][d] (for the exact flow ratio): text rows N(0,1),
        image rows shifted and scaled like the image keys; float32 array of dtype-rounded values."""
        T, d = self.total_tokens, self.head_dim
        mu, sc, _ = self._token_affine()
        rng = np.random.default_rng([self.seed, layer, 3])
        q = rng.standard_normal((self.n_q_heads, T, d), dtype=np.float32)
        q *= sc[None, :, None]
        q += mu[None, :, None]
        return self._round(q)

    def all_tensors(self):
        """K, V [Lyr][Hkv][T][d] and Q [Lyr][Hq][batch*W][d] stacked over layers."""
        Ks, Vs, Qs = [], [], []
        for l in range(self.n_layers):
            k, v, q = self.layer_tensors(l)
            Ks.append(k); Vs.append(v); Qs.append(q)
        return np.stack(Ks), np.stack(Vs), np.stack(Qs)


def _alternating_spans(lengths: Sequence[int], first_mod: int = TEXT):
    spans, pos, mod = [], 0, first_mod
    for n in lengths:
        if n > 0:
            spans.append((pos, pos + n, mod))
        pos += n
        mod = 1 - mod
    return spans


def make_workload(name, dtype, seed, n_layers, n_q_heads, n_kv_heads, head_dim, window,
                  span_lengths: Sequence[Sequence[int]], budget_pct: Sequence[int],
                  random_mu: bool = False, theta: float = 0.25, tau_factor: float = 4.0,
                  first_mod: int = TEXT, budgets: Sequence[int] | None = None) -> Workload:
    """Build a workload from per-sequence alternating span lengths (text first unless told otherwise)."""
    rng = np.random.default_rng([seed, 1 << 20])
    seqlens, spans, mus, sinks, buds, taus = [], [], [], [], [], []
    for b, lens in enumerate(span_lengths):
        sp = _alternating_spans(lens, first_mod)
        L = int(sum(lens))
        seqlens.append(L)
        spans.append(sp)
        mus.append([(float(rng.uniform(0.0, 1.0)) if random_mu else 0.5) if m == IMAGE else 0.0
                    for (_, _, m) in sp])
        n_sink = int(round(0.01 * L))
        hi = max(L - window, 1)
        n_sink = min(n_sink, hi)
        sinks.append(np.sort(rng.choice(hi, size=n_sink, replace=False)).astype(np.int64))
        B = int(budgets[b]) if budgets is not None else budget_tokens(L, int(budget_pct[b]), window)
        buds.append(B)
        taus.append(float(tau_factor / B))
    return Workload(name=name, dtype=dtype, seed=seed, n_layers=n_layers, n_q_heads=n_q_heads,
                    n_kv_heads=n_kv_heads, head_dim=head_dim, window=window, seqlens=seqlens,
                    budgets=buds, spans=spans, span_mu=mus, sinks=sinks, theta=theta, tau=taus)


def config(i: int, n_layers: int | None = None) -> Workload:
    """The five benchmark configurations; `n_layers` overrides the depth (tests use fewer layers)."""
    if i == 0:
        return make_workload("tiny_f32", "f32", 0, n_layers or 1, 4, 4, 64, 16,
                             [[32, 256, 32]], [20])
    if i == 1:
        return make_workload("llava15_7b_shaped", "bf16", 1, n_layers or 32, 32, 32, 128, 32,
                             [[35, 576, 64]], [10])
    if i == 2:
        return make_workload("qwen2vl_7b_shaped_gqa", "bf16", 2, n_layers or 28, 28, 4, 128, 32,
                             [[248, 3600, 248]], [10])
    if i == 3:
        lens = []
        for j in range(8):
            lens += [398, 1600]
        lens += [400]
        return make_workload("long_multi_image_16k", "bf16", 3, n_layers or 32, 32, 8, 128, 64,
                             [lens], [5], random_mu=True)
    if i == 4:
        rng = np.random.default_rng([4, 1 << 21])
        span_lengths, pcts = [], []
        for _ in range(8):
            L = int(rng.integers(2048, 8193))
            f = float(rng.uniform(0.6, 0.9))
            n_img = int(round(f * L))
            n_txt = L - n_img
            span_lengths.append([n_txt // 2, n_img, n_txt - n_txt // 2])
            pcts.append(int(rng.choice([5, 10, 20])))
        return make_workload("ragged_batch8_qwen2vl", "bf16", 4, n_layers or 28, 28, 4, 128, 32,
                             span_lengths, pcts)
    raise ValueError(f"no config {i}")
