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


def test_chunked_prefill_in_blocks_of_16_rows():
    """A prefill chunk of R new tokens after P0 cached ones, processed as R/16 query blocks.
    Block j is one "batch element": it reads the one shared cache (kv_stride_b = 0) up to its own
    start (seq_lens / counts), gets its own mask from the draft scores of its 16 rows, and adds
    its own 16 tokens causally (k_new / v_new). Draft side, selection and target side all run
    through the library; every stage is checked against the oracle, and with a budget that keeps
    everything the result is pinned to plain causal attention over the whole prompt (torch)."""
    g = torch.Generator().manual_seed(3)
    P0, R, T, Hq, Hkv, Hd, d, dd = 200, 64, 16, 8, 2, 4, 128, 64
    nblk, N = R // T, P0 + R
    hm = [t // 2 for t in range(Hq)]
    scale, dscale = 1 / math.sqrt(d), 1 / math.sqrt(dd)
    mk = lambda *s: (torch.randn(*s, generator=g) * 0.5).to(torch.bfloat16)
    q, kc, vc = torch.randn(R, Hq, d, generator=g).to(torch.bfloat16), mk(1, Hkv, N, d), mk(1, Hkv, N, d)
    qd, kd, vd = torch.randn(R, Hd, dd, generator=g).to(torch.bfloat16), mk(1, Hkv, N, dd), mk(1, Hkv, N, dd)
    starts = torch.tensor([P0 + T * j for j in range(nblk)], dtype=torch.int32)       # cached tokens each block sees

    def blocks(x):            # [R, H, e] -> [nblk, T, H, e]
        return x.view(nblk, T, x.shape[1], x.shape[2]).contiguous()

    def own(c):               # the block's own rows of the cache as [nblk, T, Hkv, e]
        return torch.stack([c[0, :, P0 + T * j:P0 + T * (j + 1)].permute(1, 0, 2) for j in range(nblk)]).contiguous()

    def shared(c):            # one cache for every block
        return c.to(DEV).expand(nblk, -1, -1, -1)

    # draft layer: dense attention per block with the query-key products dumped
    _, d_lse, d_logits = sts.sts_dense_attn(blocks(qd).to(DEV), shared(kd), shared(vd), dscale, seq_lens=starts.to(DEV),
                                            want_logits=True, k_new=own(kd).to(DEV), v_new=own(vd).to(DEV))
    # the dump covers the cached keys; its normaliser for the mask is the LSE over those keys only
    lse_cached = torch.stack([torch.logsumexp(d_logits[j, :, :, :starts[j]], dim=-1) for j in range(nblk)])
    for k in (48, N):
        idx, cnt, agg = sts.sts_select(d_logits, hm, k, lse=lse_cached, seq_lens=starts.to(DEV),
                                       kind=sts.STS_SCORES_LOGITS_LSE, want_agg=True)
        sel, c = oracle.select(agg.cpu().numpy(), k, starts.numpy())
        o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
        np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
        np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
        out, lse = sts.sts_sparse_attn(blocks(q).to(DEV), shared(kc), shared(vc), idx, scale, counts=cnt, head_map=hm,
                                       out_dtype=torch.float32, k_new=own(kc).to(DEV), v_new=own(vc).to(DEV))
        ref = oracle.attn(oracle.bf16_bits(blocks(q)), oracle.bf16_bits(kc.expand(nblk, -1, -1, -1).contiguous()),
                          oracle.bf16_bits(vc.expand(nblk, -1, -1, -1).contiguous()), scale, o_idx, o_cnt,
                          k_new=oracle.bf16_bits(own(kc)), v_new=oracle.bf16_bits(own(vc)), causal=True)
        check_attn(out, lse, ref, what=f"chunked prefill k={k}")
    # k >= N kept every cached token: plain causal attention of rows P0.. over the whole prompt
    G = Hq // Hkv
    qf = q.float().permute(1, 0, 2)                                         # [Hq, R, d]
    kf = kc[0].float().repeat_interleave(G, dim=0)                          # [Hq, N, d]
    vf = vc[0].float().repeat_interleave(G, dim=0)
    mask = torch.arange(N)[None, :] <= (P0 + torch.arange(R))[:, None]      # row r sees tokens 0..P0+r
    full = torch.nn.functional.scaled_dot_product_attention(qf[None], kf[None], vf[None], attn_mask=mask[None, None],
                                                            scale=scale)[0].permute(1, 0, 2)      # [R, Hq, d]
    got = out.cpu().view(R, Hq, d)
    assert (got - full).abs().max().item() < 1e-2
