"""Synthetic STS workloads: shapes, value distributions and planted attention structure.

The paper times on NarrativeQA / LongBench / SWE-bench traces with Llama-3.1 8B/70B targets
and a Llama-3.2 1B draft (Section 6.1, 6.2). None of those are available offline, so the
inputs here take the attention *shapes* and context lengths of those workloads and plant
the attention-mass structure the paper describes (sink tokens, a recent window, a few
scattered heavy tokens; Section 6.4) synthetically. Everything is seeded.

All tensors are made with plain torch ops on the requested device, so the same recipe
serves small CPU cases (tests) and full-size GPU cases (benchmark).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    B: int            # batch
    N: int            # cached tokens (context length)
    Hq: int           # target query heads
    Hkv: int          # target KV heads
    d: int            # head dim
    Tq: int           # query rows of the speculative block (gamma + 1)
    Hd: int           # draft heads feeding this layer
    budget: float     # fraction of N kept per head
    heavy_frac: float = 0.02   # fraction of positions per KV head planted as heavy
    zipf_s: float = 1.1        # exponent of the rank distribution of heavy positions
    sinks: int = 4             # leading positions planted
    recent: int = 64           # trailing positions planted
    noise: float = 0.5         # std of the logit noise between target and draft
    gain: float = 3.0          # planted keys get gain * q_hat added
    clustered: bool = False    # heavy positions: rank r sits at N - r (recency-clustered) instead of scattered
    kv_std: float = 0.5
    layers: int = 1            # distinct resident layers (bench only)
    # draft attention layer of its own (70B-shaped config): query heads Hd, these extras
    draft_Hkv: int = 0
    draft_d: int = 0
    draft_key_noise: float = 0.3


CONFIGS: Dict[str, WorkloadConfig] = {
    # single layer, 4K context, 8B-shaped heads: the case the oracle finishes in seconds
    "c1": WorkloadConfig("c1", B=1, N=4096, Hq=32, Hkv=8, d=128, Tq=5, Hd=16, budget=0.10),
    "c2": WorkloadConfig("c2", B=1, N=32768, Hq=32, Hkv=8, d=128, Tq=5, Hd=16, budget=0.10),
    # headline: 128K context, batch 4, 10% budget (5% and 20% by override)
    "c3": WorkloadConfig("c3", B=4, N=131072, Hq=32, Hkv=8, d=128, Tq=5, Hd=16, budget=0.10,
                         heavy_frac=0.01, zipf_s=1.2, noise=0.7),
    "c4": WorkloadConfig("c4", B=1, N=1048576, Hq=32, Hkv=8, d=128, Tq=5, Hd=16, budget=0.10,
                         recent=256, layers=32),
    "c5": WorkloadConfig("c5", B=8, N=131072, Hq=64, Hkv=8, d=128, Tq=8, Hd=32, budget=0.10,
                         heavy_frac=0.01, zipf_s=1.2, draft_Hkv=8, draft_d=64),
}


def budget_tokens(cfg: WorkloadConfig, frac: Optional[float] = None) -> int:
    """Token budget from a fraction: k = ceil(frac * N) (410 at N=4096, 10%)."""
    f = cfg.budget if frac is None else frac
    # guard the product against binary representation error before the ceiling
    return int(math.ceil(round(f * cfg.N, 6)))


def default_head_map(Hq: int, Hd: int) -> torch.Tensor:
    """Target head t -> draft head floor(t * Hd / Hq): neighbours share a draft head."""
    return (torch.arange(Hq, dtype=torch.int64) * Hd // Hq).to(torch.int32)


@dataclass
class Workload:
    cfg: WorkloadConfig
    q: torch.Tensor          # [B,Tq,Hq,d] bf16
    k: torch.Tensor          # [B,Hkv,N,d] bf16
    v: torch.Tensor          # [B,Hkv,N,d] bf16
    head_map: torch.Tensor   # [Hq] int32 (CPU)
    scores: Optional[torch.Tensor]  # [B,Hd,Tq,N] fp32 draft probabilities (None if not asked)
    scale: float
    k_budget: int
    extras: dict = field(default_factory=dict)


def _heavy_positions(N: int, count: int, s: float, gen: torch.Generator, device,
                     clustered: bool = False) -> torch.Tensor:
    """`count` distinct positions whose ranks follow a truncated Zipf(s), scattered by a
    seeded permutation (the worst case for gather locality), or, `clustered`, rank r at
    position N - r. Sequential weighted draws without replacement are realised with Gumbel
    perturbations of the log-weights (same distribution, one pass)."""
    ranks = torch.arange(1, N + 1, device=device, dtype=torch.float32)
    u = torch.rand(N, generator=gen, device=device, dtype=torch.float32).clamp_(1e-12, 1 - 1e-7)
    keyed = -s * torch.log(ranks) - torch.log(-torch.log(u))
    chosen = torch.topk(keyed, count).indices
    perm = torch.randperm(N, generator=gen, device=device)     # drawn in both modes: same stream of numbers after it
    return (N - 1 - chosen) if clustered else perm[chosen]


def make_workload(cfg: WorkloadConfig, seed: int = 20251127, device="cpu", with_scores: bool = True,
                  head_map: Optional[torch.Tensor] = None, budget: Optional[float] = None) -> Workload:
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    B, N, Hq, Hkv, d, Tq, Hd = cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.d, cfg.Tq, cfg.Hd
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(d)
    hm = default_head_map(Hq, Hd) if head_map is None else head_map.to(torch.int32).cpu()

    q32 = torch.randn(B, Tq, Hq, d, generator=gen, device=dev, dtype=torch.float32)
    q = q32.to(torch.bfloat16)
    k = torch.empty(B, Hkv, N, d, device=dev, dtype=torch.bfloat16)
    v = torch.empty(B, Hkv, N, d, device=dev, dtype=torch.bfloat16)
    n_heavy = int(math.ceil(cfg.heavy_frac * N))
    fixed = torch.cat([torch.arange(0, min(cfg.sinks, N), device=dev),
                       torch.arange(max(N - cfg.recent, 0), N, device=dev)])
    for b in range(B):
        kb = torch.randn(Hkv, N, d, generator=gen, device=dev, dtype=torch.float32) * cfg.kv_std
        # unit vector along the sum of the query vectors that read each KV head
        qsum = q[b].float().reshape(Tq, Hkv, G, d).sum(dim=(0, 2))
        qhat = qsum / qsum.norm(dim=-1, keepdim=True).clamp_min(1e-20)
        for g in range(Hkv):
            pos = torch.unique(torch.cat([fixed, _heavy_positions(N, n_heavy, cfg.zipf_s, gen, dev, cfg.clustered)]))
            kb[g, pos] += cfg.gain * qhat[g]
        k[b] = kb.to(torch.bfloat16)
        del kb
        v[b] = (torch.randn(Hkv, N, d, generator=gen, device=dev, dtype=torch.float32)
                * cfg.kv_std).to(torch.bfloat16)

    scores = None
    if with_scores:
        scores = torch.empty(B, Hd, Tq, N, device=dev, dtype=torch.float32)
        hm_dev = hm.to(dev).long()
        for b in range(B):
            # target scaled logits per query head, from the rounded bf16 tensors
            kt = k[b].float().repeat_interleave(G, dim=0)                  # [Hq,N,d]
            lt = torch.einsum("ihe,hne->hin", q[b].float(), kt) * scale      # [Hq,Tq,N]
            del kt
            ld = torch.zeros(Hd, Tq, N, device=dev, dtype=torch.float32)
            ld.index_add_(0, hm_dev, lt)
            cnt = torch.bincount(hm_dev, minlength=Hd).clamp_min(1).to(torch.float32)
            ld /= cnt.view(Hd, 1, 1)
            del lt
            ld += cfg.noise * torch.randn(Hd, Tq, N, generator=gen, device=dev, dtype=torch.float32)
            scores[b] = torch.softmax(ld, dim=-1)
            del ld
    return Workload(cfg=cfg, q=q, k=k, v=v, head_map=hm, scores=scores, scale=scale,
                    k_budget=budget_tokens(cfg, budget))


def make_draft_layer(w: Workload, seed: int = 777):
    """Draft attention layer for the 70B-shaped config: draft keys are a random linear
    projection of the target keys plus noise, draft queries the same projection of the mean
    target query of the heads mapped to each draft head. Returns dict(q,k,v,scale)."""
    cfg = w.cfg
    assert cfg.draft_d > 0 and cfg.draft_Hkv == cfg.Hkv
    dev = w.k.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    B, N, Hd, dd, Tq = cfg.B, cfg.N, cfg.Hd, cfg.draft_d, cfg.Tq
    R = torch.randn(cfg.d, dd, generator=gen, device=dev, dtype=torch.float32) / math.sqrt(dd)
    kd = torch.empty(B, cfg.draft_Hkv, N, dd, device=dev, dtype=torch.bfloat16)
    vd = torch.empty_like(kd)
    for b in range(B):
        kd[b] = (w.k[b].float() @ R + cfg.draft_key_noise
                 * torch.randn(cfg.draft_Hkv, N, dd, generator=gen, device=dev)).to(torch.bfloat16)
        vd[b] = (cfg.kv_std * torch.randn(cfg.draft_Hkv, N, dd, generator=gen, device=dev)
                 ).to(torch.bfloat16)
    hm_dev = w.head_map.to(dev).long()
    qm = torch.zeros(B, Tq, Hd, cfg.d, device=dev, dtype=torch.float32)
    qm.index_add_(2, hm_dev, w.q.float())
    cnt = torch.bincount(hm_dev, minlength=Hd).clamp_min(1).to(torch.float32)
    qm /= cnt.view(1, 1, Hd, 1)
    qd = (qm @ R).to(torch.bfloat16)
    # q.k of the projected pair approximates the target's q.k (E[R R^T] = I), so the draft is
    # scaled like the target to keep its logits correlated with the target's
    return {"q": qd, "k": kd, "v": vd, "scale": 1.0 / math.sqrt(cfg.d)}


def small(cfg: WorkloadConfig, **kw) -> WorkloadConfig:
    return replace(cfg, **kw)
