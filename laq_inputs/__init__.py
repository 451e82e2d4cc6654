"""Seeded synthetic inputs for the LAQ re-eviction hot path.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It holds *no* arithmetic of the method (no logits, no
softmax, no pooling, no selection): it only draws the tensors the method
consumes -- the cached lookahead queries (Q-cache, Sec. 4.2), the prefill key
and value caches (Sec. 4.3) and the per-layer budgets -- with the shapes of
the GQA models the paper evaluates (Sec. 5.1 "Setup": 32 query / 8 KV heads,
head size 128, 32 layers, contexts 4K-32K, windows of 8 / 8+8 queries,
budgets 128-512, PyramidKV-style per-layer budgets).

The paper's prompts come from LongBench / Needle-in-a-Haystack / RULER run
through trained models; neither the datasets nor the weights exist here, so
these tensors stand in for the *shape and structure* of that workload:
planted heavy keys (keys aligned with the mean window query, the structure an
importance score is meant to find), attention-sink rows at the first
positions, clustered keys, heavy-tailed query norms.

All draws come from ``torch.Generator`` seeded from (config, sequence, layer);
a CPU generator and a GPU generator give different bits for the same seed, so
a test always draws once and hands the same tensors to both sides.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import torch

__all__ = [
    "LaqConfig", "CONFIGS", "get_config", "budgets_for", "instance_seed",
    "make_instance", "make_batch", "pyramid_budget",
]


@dataclasses.dataclass(frozen=True)
class LaqConfig:
    """One synthetic workload (shapes follow the paper's Sec. 5.1 set-up)."""
    name: str
    cfg_id: int
    dtype: str          # "f32" | "bf16"
    n_seq: int          # independent sequences
    n_layer: int        # layers per sequence
    Hq: int
    Hkv: int
    d: int
    L: int              # rows of K handed in (prefix P = L - W, then the W window tokens)
    W: int              # cached lookahead queries per query head
    pool: int           # pooling kernel (odd)
    budget: str         # "uniform:<B>" | "pyramid:<hi>:<lo>"
    kind: str           # generator recipe, see make_instance
    planted_frac: float = 0.0
    planted_count: int = 0
    planted_amp: float = 4.0
    n_sink: int = 0

    @property
    def n_inst(self) -> int:
        return self.n_seq * self.n_layer

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def R(self) -> int:
        return self.G * self.W

    @property
    def P(self) -> int:
        return self.L - self.W

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


CONFIGS: Dict[int, LaqConfig] = {
    1: LaqConfig("tiny-f32", 1, "f32", 1, 1, 4, 2, 64, 512, 8, 7, "uniform:64",
                 "planted_spaced", planted_count=8),
    2: LaqConfig("llama3-8b-1layer-4k", 2, "bf16", 1, 1, 32, 8, 128, 4096, 8, 7,
                 "uniform:128", "planted", planted_frac=0.01),
    3: LaqConfig("llama3-8b-32layer-16k", 3, "bf16", 1, 32, 32, 8, 128, 16384, 16, 7,
                 "uniform:512", "planted", planted_frac=0.005, n_sink=4),
    4: LaqConfig("mistral-7b-32layer-32k-pyramid", 4, "bf16", 1, 32, 32, 8, 128, 32768, 32, 7,
                 "pyramid:2048:128", "clusters"),
    5: LaqConfig("batch8-32layer-32k-heavytail", 5, "bf16", 8, 32, 32, 8, 128, 32768, 16, 7,
                 "uniform:256", "student_t"),
}


def get_config(cfg_id: int) -> LaqConfig:
    return CONFIGS[int(cfg_id)]


def pyramid_budget(layer: int, n_layer: int, hi: int, lo: int) -> int:
    """Linearly decreasing integer budget hi -> lo over the layers (layer 0 gets hi)."""
    if n_layer <= 1:
        return hi
    span = hi - lo
    return hi - (span * layer + (n_layer - 1) // 2) // (n_layer - 1)


def budgets_for(cfg: LaqConfig) -> List[int]:
    """Per-instance budgets, instance index = seq * n_layer + layer."""
    parts = cfg.budget.split(":")
    out: List[int] = []
    for _seq in range(cfg.n_seq):
        for layer in range(cfg.n_layer):
            if parts[0] == "uniform":
                out.append(int(parts[1]))
            elif parts[0] == "pyramid":
                out.append(pyramid_budget(layer, cfg.n_layer, int(parts[1]), int(parts[2])))
            else:
                raise ValueError(cfg.budget)
    return out


def instance_seed(cfg_id: int, seq: int, layer: int) -> int:
    """Distinct 63-bit seed per (config, sequence, layer) from a splitmix-style integer mix."""
    x = (cfg_id * 0x9E3779B97F4A7C15 + seq * 0xBF58476D1CE4E5B9 + layer * 0x94D049BB133111EB
         + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def _mean_window_query_unit(q: torch.Tensor, Hkv: int) -> torch.Tensor:
    """Unit vector along the mean of the G*W window queries of each KV head: [Hkv, d] fp32."""
    Hq, W, d = q.shape
    m = q.float().reshape(Hkv, (Hq // Hkv) * W, d).mean(dim=1)
    return m / m.norm(dim=1, keepdim=True).clamp_min(1e-20)


def _spaced_positions(gen: torch.Generator, count: int, P: int, gap: int, margin: int,
                      device) -> torch.Tensor:
    """`count` positions in [margin, P-margin), pairwise at least `gap` apart (one per stratum)."""
    lo, hi = margin, P - margin
    stride = (hi - lo) // count
    if stride < gap:
        raise ValueError("prefix too short for spaced planting")
    jitter = torch.randint(0, stride - gap + 1, (count,), generator=gen, device=device)
    base = lo + stride * torch.arange(count, device=device)
    return base + jitter


def make_instance(cfg: LaqConfig, seq: int = 0, layer: int = 0, device="cpu",
                  want_v: bool = True
                  ) -> Tuple[torch.Tensor, torch.Tensor, Optional[torch.Tensor], dict]:
    """Draw one (sequence, layer) instance.

    Returns q_win [Hq, W, d], k [Hkv, L, d], v [Hkv, L, d] (or None) in the
    config's storage dtype, and a dict with the structure that was planted
    (``planted``: LongTensor [Hkv, n] of prefix positions, ``sinks``: int).
    Values are drawn in fp32 and rounded once (round-to-nearest-even) to the
    storage dtype; both consumers see exactly those rounded values.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(instance_seed(cfg.cfg_id, seq, layer))
    Hq, Hkv, d, L, W, P = cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.W, cfg.P
    meta: dict = {"planted": None, "sinks": cfg.n_sink}

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32)

    q = randn(Hq, W, d)
    if cfg.kind == "student_t":
        # heavy-tailed query norms: each query row scaled by |t|, t ~ Student-t(nu=3)
        n = randn(Hq, W, 4)
        t = n[..., 0] / torch.sqrt((n[..., 1:] ** 2).sum(-1) / 3.0)
        q = q * t.abs().unsqueeze(-1)

    if cfg.kind == "clusters":
        centres = randn(Hkv, 64, d)
        which = torch.randint(0, 64, (Hkv, L), generator=gen, device=dev)
        k = torch.gather(centres, 1, which.unsqueeze(-1).expand(Hkv, L, d))
        k = k + 0.5 * randn(Hkv, L, d)
    else:
        k = randn(Hkv, L, d)

    if cfg.kind in ("planted", "planted_spaced"):
        # the direction is taken from the queries *as stored* so that both consumers agree on it
        u = _mean_window_query_unit(q.to(cfg.torch_dtype), Hkv)            # [Hkv, d]
        if cfg.kind == "planted_spaced":
            n_pl = cfg.planted_count
            pos = torch.stack([_spaced_positions(gen, n_pl, P, cfg.pool + 1, cfg.pool // 2 + 1, dev)
                               for _ in range(Hkv)])
        else:
            n_pl = int(round(cfg.planted_frac * P))
            pos = torch.stack([torch.randperm(P - cfg.n_sink, generator=gen, device=dev)[:n_pl]
                               + cfg.n_sink for _ in range(Hkv)])
        noise = randn(Hkv, n_pl, d)
        rows = cfg.planted_amp * u.unsqueeze(1) + noise
        k.scatter_(1, pos.unsqueeze(-1).expand(Hkv, n_pl, d), rows)
        meta["planted"] = pos
        if cfg.n_sink:
            k[:, :cfg.n_sink, :] = 8.0 * u.unsqueeze(1) + randn(Hkv, cfg.n_sink, d)

    v = randn(Hkv, L, d) if want_v else None
    dt = cfg.torch_dtype
    return q.to(dt), k.to(dt), (v.to(dt) if v is not None else None), meta


def make_batch(cfg: LaqConfig, device="cpu", want_v: bool = True, instances=None):
    """Draw several instances into dense batched tensors.

    Returns q_win [n, Hq, W, d], k [n, Hkv, L, d], v [n, Hkv, L, d] or None,
    budgets (list of int, one per instance) and the per-instance meta dicts.
    ``instances`` selects a subset of instance indices (seq * n_layer + layer).
    """
    ids = list(range(cfg.n_inst)) if instances is None else list(instances)
    dev = torch.device(device)
    dt = cfg.torch_dtype
    n = len(ids)
    q = torch.empty(n, cfg.Hq, cfg.W, cfg.d, dtype=dt, device=dev)
    k = torch.empty(n, cfg.Hkv, cfg.L, cfg.d, dtype=dt, device=dev)
    v = torch.empty(n, cfg.Hkv, cfg.L, cfg.d, dtype=dt, device=dev) if want_v else None
    metas = []
    all_budgets = budgets_for(cfg)
    for slot, inst in enumerate(ids):
        seq, layer = divmod(inst, cfg.n_layer)
        qi, ki, vi, meta = make_instance(cfg, seq, layer, device=dev, want_v=want_v)
        q[slot].copy_(qi)
        k[slot].copy_(ki)
        if want_v:
            v[slot].copy_(vi)
        metas.append(meta)
    return q, k, v, [all_budgets[i] for i in ids], metas


def scaled(cfg: LaqConfig, **overrides) -> LaqConfig:
    """A copy of a config with some fields replaced (used for reduced-size parity cases)."""
    return dataclasses.replace(cfg, **overrides)
