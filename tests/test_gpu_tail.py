"""GPU parity for the fused verification tail: the speculative block's own keys/values are
appended (causally) after the cached keys inside the combine step. Against the CPU oracle,
through the C ABI."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(seed, B, Tq, Hq, Hkv, d, N):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    kn = (torch.randn(B, Tq, Hkv, d, generator=g) * 0.5).to(torch.bfloat16)
    vn = (torch.randn(B, Tq, Hkv, d, generator=g) * 0.5).to(torch.bfloat16)
    return q, k, v, kn, vn


@pytest.mark.parametrize("B,Tq,Hq,Hkv,d,N,kk,causal", [
    (2, 5, 8, 2, 128, 1000, 100, True),
    (2, 5, 8, 2, 128, 1000, 100, False),
    (1, 8, 16, 2, 128, 700, 64, True),       # 16 rows per unit
    (2, 5, 8, 2, 64, 333, 40, True),         # head dim 64
    (1, 1, 4, 4, 128, 50, 5, True),          # a single candidate
    (1, 16, 4, 2, 64, 200, 20, True),        # 16 candidates
])
def test_sparse_with_block_tail(B, Tq, Hq, Hkv, d, N, kk, causal):
    q, k, v, kn, vn = make(1, B, Tq, Hq, Hkv, d, N)
    rng = np.random.default_rng(2)
    hm = [t // 2 for t in range(Hq)]
    idx = np.empty((B, Hq, kk), np.int32)
    for b in range(B):
        rows = {}
        for t in range(Hq):
            rows.setdefault(hm[t], np.sort(rng.choice(N, kk, replace=False)))
            idx[b, t] = rows[hm[t]]
    counts = np.full((B, Hq), kk, np.int32)
    counts[0, :2] = 0                          # a set with an empty index row: tail only
    scale = 1.0 / math.sqrt(d)
    ref = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), scale, idx, counts,
                      k_new=oracle.bf16_bits(kn), v_new=oracle.bf16_bits(vn), causal=causal)
    out, lse = sts.sts_sparse_attn(q.to(DEV), k.to(DEV), v.to(DEV), torch.from_numpy(idx).to(DEV), scale,
                                   counts=torch.from_numpy(counts).to(DEV), head_map=hm,
                                   out_dtype=torch.float32, k_new=kn.to(DEV), v_new=vn.to(DEV), causal=causal)
    check_attn(out, lse, ref, what="sparse + tail")


@pytest.mark.parametrize("d", [128, 64])
def test_dense_with_block_tail_and_lengths(d):
    B, Tq, Hq, Hkv, N = 3, 5, 8, 2, 600
    q, k, v, kn, vn = make(3, B, Tq, Hq, Hkv, d, N)
    lens = torch.tensor([600, 77, 0], dtype=torch.int32)      # the last sequence has no cache yet
    ref = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), 0.1, seq_lens=lens.numpy(),
                      k_new=oracle.bf16_bits(kn), v_new=oracle.bf16_bits(vn), causal=True)
    out, lse, _ = sts.sts_dense_attn(q.to(DEV), k.to(DEV), v.to(DEV), 0.1, seq_lens=lens.to(DEV),
                                     out_dtype=torch.float32, k_new=kn.to(DEV), v_new=vn.to(DEV))
    check_attn(out, lse, ref, what="dense + tail")
    out16, lse16, _ = sts.sts_dense_attn(q.to(DEV), k.to(DEV), v.to(DEV), 0.1, seq_lens=lens.to(DEV),
                                         k_new=kn.to(DEV), v_new=vn.to(DEV))
    check_attn(out16, lse16, ref, what="dense + tail bf16")


def test_tail_equals_caller_side_merge_with_lse():
    """Fusing the tail must equal what a caller gets by merging the cached part and the block's
    own causal part with the returned log-sum-exp values."""
    B, Tq, Hq, Hkv, d, N, kk = 1, 5, 8, 2, 128, 500, 50
    q, k, v, kn, vn = make(4, B, Tq, Hq, Hkv, d, N)
    idx = torch.from_numpy(np.sort(np.random.default_rng(0).choice(N, (B, Hq, kk)), -1).astype(np.int32))
    fused, lse_f = sts.sts_sparse_attn(q.to(DEV), k.to(DEV), v.to(DEV), idx.to(DEV), 0.09, out_dtype=torch.float32,
                                       k_new=kn.to(DEV), v_new=vn.to(DEV))
    part, lse_p = sts.sts_sparse_attn(q.to(DEV), k.to(DEV), v.to(DEV), idx.to(DEV), 0.09, out_dtype=torch.float32)
    G = Hq // Hkv
    s = torch.einsum("bihe,bjhe->bhij", q.float(), kn.float().repeat_interleave(G, 2)) * 0.09     # [B,Hq,Tq,Tq]
    s = s.masked_fill(~torch.tril(torch.ones(Tq, Tq, dtype=torch.bool)), float("-inf"))
    lse_t = torch.logsumexp(s, -1)                                                                # [B,Hq,Tq]
    o_t = torch.einsum("bhij,bjhe->bihe", torch.softmax(s, -1), vn.float().repeat_interleave(G, 2))
    lp = lse_p.cpu()
    lw = torch.logaddexp(lp, lse_t)
    wa = torch.exp(lp - lw).permute(0, 2, 1)[..., None]
    wb = torch.exp(lse_t - lw).permute(0, 2, 1)[..., None]
    merged = wa * part.cpu() + wb * o_t
    assert (merged - fused.cpu()).abs().max() < 2e-3
    assert (lw - lse_f.cpu()).abs().max() < 1e-3
