"""Sparse prefill masks (Section 4.2: during prefill every query token gets its own mask, a
two-dimensional pattern per head). Expressed with the existing entry points as a batch of
single-row queries that all read the same cache (kv_stride_b = 0), with a per-row visible
length for causality. Selection and attention against the oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_prefill_rows_as_a_stride_zero_batch():
    g = torch.Generator().manual_seed(0)
    R, P0, Hq, Hkv, Hd, d, k = 24, 300, 8, 2, 4, 128, 48      # rows P0..P0+R-1 of a prompt
    N = P0 + R
    q = torch.randn(R, 1, Hq, d, generator=g).to(torch.bfloat16)          # one query row per "batch"
    kc = (torch.randn(1, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    vc = (torch.randn(1, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    hm = [t // 2 for t in range(Hq)]
    lens = torch.arange(P0 + 1, P0 + R + 1, dtype=torch.int32)            # row r sees tokens 0..P0+r
    # draft probabilities per row: causal softmax of random logits
    logits = torch.randn(R, Hd, 1, N, generator=g) * 2
    for r in range(R):
        logits[r, :, :, lens[r]:] = float("-inf")
    scores = torch.softmax(logits, dim=-1)
    idx, cnt, _ = sts.sts_select(scores.to(DEV), hm, k, seq_lens=lens.to(DEV))
    o_idx, o_cnt, _ = oracle.select_indices(scores.numpy(), np.asarray(hm, np.int32), k, seq_lens=lens.numpy())
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    assert all((o_idx[r] < lens[r].item()).all() for r in range(R))        # masks respect causality
    # attention: every row reads the one shared cache
    k_exp, v_exp = kc.to(DEV).expand(R, Hkv, N, d), vc.to(DEV).expand(R, Hkv, N, d)
    assert k_exp.stride(0) == 0
    out, lse = sts.sts_sparse_attn(q.to(DEV), k_exp, v_exp, idx, 1 / math.sqrt(d), counts=cnt, head_map=hm,
                                   out_dtype=torch.float32)
    ref = oracle.attn(oracle.bf16_bits(q), oracle.bf16_bits(kc.expand(R, Hkv, N, d).contiguous()),
                      oracle.bf16_bits(vc.expand(R, Hkv, N, d).contiguous()), 1 / math.sqrt(d), o_idx, o_cnt)
    check_attn(out, lse, ref, what="prefill rows")
