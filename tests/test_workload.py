"""The synthetic input recipe: shapes, determinism, planted structure."""
from dataclasses import replace

import numpy as np
import torch

from workload import CONFIGS, budget_tokens, default_head_map, make_draft_layer, make_workload


def test_budget_rule_is_ceiling():
    assert budget_tokens(CONFIGS["c1"]) == 410
    assert budget_tokens(CONFIGS["c2"]) == 3277
    assert [budget_tokens(CONFIGS["c3"], f) for f in (0.05, 0.10, 0.20)] == [6554, 13108, 26215]
    assert [budget_tokens(CONFIGS["c4"], f) for f in (0.02, 0.10)] == [20972, 104858]


def test_default_head_map_pairs_neighbours():
    hm = default_head_map(32, 16)
    assert hm.tolist() == [t // 2 for t in range(32)]


def test_small_workload_shapes_and_determinism():
    cfg = replace(CONFIGS["c1"], N=512)
    a = make_workload(cfg, seed=5)
    b = make_workload(cfg, seed=5)
    c = make_workload(cfg, seed=6)
    assert a.q.shape == (1, 5, 32, 128) and a.k.shape == (1, 8, 512, 128) and a.scores.shape == (1, 16, 5, 512)
    assert a.q.dtype == torch.bfloat16 and a.scores.dtype == torch.float32
    assert torch.equal(a.k, b.k) and torch.equal(a.scores, b.scores)
    assert not torch.equal(a.k, c.k)
    np.testing.assert_allclose(a.scores.sum(-1).numpy(), 1.0, rtol=1e-5)
    assert a.k_budget == 52


def test_planted_tokens_carry_more_draft_mass():
    cfg = replace(CONFIGS["c1"], N=1024)
    w = make_workload(cfg, seed=1)
    mass = w.scores.sum(2)[0]                 # [Hd,N]
    planted = torch.cat([torch.arange(4), torch.arange(1024 - 64, 1024)])
    rest = torch.ones(1024, dtype=torch.bool)
    rest[planted] = False
    assert mass[:, planted].mean() > 1.3 * mass[:, rest].mean()


def test_draft_layer_shapes():
    cfg = replace(CONFIGS["c5"], B=1, N=256)
    w = make_workload(cfg, seed=2, with_scores=False)
    dl = make_draft_layer(w)
    assert dl["q"].shape == (1, 8, 32, 64) and dl["k"].shape == (1, 8, 256, 64)
    # draft logits correlate with the mean target logits of the mapped heads
    G = 8
    lt = torch.einsum("ihe,hne->hin", w.q[0].float(), w.k[0].float().repeat_interleave(G, 0))
    ld = torch.einsum("ihe,hne->hin", dl["q"][0].float(), dl["k"][0].float().repeat_interleave(4, 0))
    ltm = lt.reshape(32, 2, 8, 256).mean(1)
    corr = torch.corrcoef(torch.stack([ltm.flatten(), ld.flatten()]))[0, 1]
    assert corr > 0.5
