"""Seeded random sweeps over shapes and option combinations, every case against the oracle.
Complements the hand-picked cases: page sizes, page tables, head maps, ragged counts, lengths,
the fused tail, output types and both head dims get combined at random."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn, stored_agg
from test_gpu_blocks import paged_copy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("seed", range(24))
def test_random_attention_case(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    Tq = int(rng.integers(1, 17))
    B = int(rng.integers(1, 4))
    N = int(rng.integers(1, 2500))
    page = int(rng.choice([1, 1, 2, 4, 8, 16, 32]))
    paged = bool(rng.integers(0, 2))
    sparse = bool(rng.integers(0, 4) > 0)
    tail = bool(rng.integers(0, 2))
    causal = bool(rng.integers(0, 2))
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    kn = vn = None
    if tail:
        kn = (torch.randn(B, Tq, Hkv, d, generator=g) * 0.5).to(torch.bfloat16)
        vn = (torch.randn(B, Tq, Hkv, d, generator=g) * 0.5).to(torch.bfloat16)
    scale = float(rng.uniform(0.05, 0.3))
    nblk = (N + page - 1) // page
    kw = dict(page_size=page)
    kd, vd = k.to(DEV), v.to(DEV)
    if paged:
        kp, vp, table = paged_copy(k, v, page, seed)
        kd, vd = kp.to(DEV), vp.to(DEV)
        kw.update(block_table=table.to(DEV), N=N)
    if tail:
        kw.update(k_new=kn.to(DEV), v_new=vn.to(DEV), causal=causal)
    okw = dict(k_new=None if kn is None else oracle.bf16_bits(kn), v_new=None if vn is None else oracle.bf16_bits(vn),
               causal=causal)
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    out_dtype = torch.float32 if rng.integers(0, 2) else torch.bfloat16
    what = f"seed {seed}: d{d} Hkv{Hkv} G{G} Tq{Tq} B{B} N{N} p{page} paged{paged} sparse{sparse} tail{tail}"
    if sparse:
        hm = rng.integers(0, max(1, Hq // 2), size=Hq).tolist() if rng.integers(0, 2) else None
        kbk = int(rng.integers(1, nblk + 1))
        idx = np.empty((B, Hq, kbk), np.int32)
        counts = np.empty((B, Hq), np.int32)
        for b in range(B):
            rows, cnts = {}, {}
            for t in range(Hq):
                key = (t // G, hm[t]) if hm is not None else t
                if key not in rows:
                    rows[key] = np.sort(rng.choice(nblk, kbk, replace=False))
                    cnts[key] = int(rng.integers(0, kbk + 1)) if rng.integers(0, 3) == 0 else kbk
                idx[b, t], counts[b, t] = rows[key], cnts[key]
        tok, tcnt = oracle.expand_blocks(idx, counts, page, N)
        ref = oracle.attn(qb, kb, vb, scale, tok, tcnt, **okw)
        out, lse = sts.sts_sparse_attn(q.to(DEV), kd, vd, torch.from_numpy(idx).to(DEV), scale,
                                       counts=torch.from_numpy(counts).to(DEV), head_map=hm, out_dtype=out_dtype, **kw)
    else:
        lens = torch.from_numpy(rng.integers(0, N + 1, size=B).astype(np.int32)) if rng.integers(0, 2) else None
        ref = oracle.attn(qb, kb, vb, scale, seq_lens=None if lens is None else lens.numpy(), **okw)
        out, lse, _ = sts.sts_dense_attn(q.to(DEV), kd, vd, scale, seq_lens=None if lens is None else lens.to(DEV),
                                         out_dtype=out_dtype, **kw)
    check_attn(out, lse, ref, what=what)


@pytest.mark.parametrize("seed", range(16))
def test_random_select_case(seed):
    rng = np.random.default_rng(2000 + seed)
    B = int(rng.integers(1, 4))
    Hd = int(rng.integers(1, 7))
    Hq = int(rng.integers(1, 13))
    Tq = int(rng.integers(1, 10))
    N = int(rng.integers(1, 30000))
    page = int(rng.choice([1, 1, 1, 3, 8, 16, 64]))
    nunits = (N + page - 1) // page
    k = int(rng.integers(1, nunits + 3))
    reduce = int(rng.integers(0, 2))
    hm = rng.integers(0, Hd, size=Hq).tolist()
    g = torch.Generator().manual_seed(seed)
    style = seed % 4
    if style == 0:
        scores = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 3, dim=-1)
    elif style == 1:
        scores = torch.randint(0, 5, (B, Hd, Tq, N), generator=g).float() / 4          # massive ties
    elif style == 2:
        scores = torch.randn(B, Hd, Tq, N, generator=g)                                # signed
    else:
        scores = torch.rand(B, Hd, Tq, N, generator=g) * 1e-30                          # tiny / denormal sums
    lens = torch.from_numpy(rng.integers(0, N + 1, size=B).astype(np.int32)) if rng.integers(0, 2) else None
    idx, cnt, agg = sts.sts_select(scores.to(DEV), hm, k, seq_lens=None if lens is None else lens.to(DEV),
                                   reduce=reduce, want_agg=True, page_size=page)
    torch.cuda.synchronize()
    o_idx, o_cnt, o_agg = oracle.select_indices(scores.numpy(), np.asarray(hm, np.int32), k, reduce=reduce,
                                                seq_lens=None if lens is None else lens.numpy(), page=page)
    what = f"seed {seed}: B{B} Hd{Hd} Hq{Hq} Tq{Tq} N{N} k{k} p{page} reduce{reduce} style{style}"
    np.testing.assert_array_equal(agg.cpu().numpy().view(np.uint32), stored_agg(o_agg, lens).view(np.uint32), err_msg=what)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt, err_msg=what)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx, err_msg=what)


@pytest.mark.parametrize("seed", range(30))
def test_random_selection_case(seed):
    """Random shapes and options of sts_select: row lengths on both sides of every path switch
    (one workgroup per row, chunk-local top-k + pool, histogram pipeline, vector and scalar
    loads), budgets from 1 to beyond N, ragged lengths, per-head budgets, block granularity,
    both score kinds and reductions, fp32 and bf16 scores, quantised scores (ties)."""
    rng = np.random.default_rng(5000 + seed)
    B = int(rng.integers(1, 4))
    Hd = int(rng.integers(1, 6))
    Hq = int(rng.integers(1, 9))
    Tq = int(rng.choice([1, 2, 5, 8, 11]))
    N = int(rng.choice([rng.integers(1, 9000), rng.integers(9000, 40000), rng.integers(40000, 120000)]))
    if rng.integers(0, 3):
        N = max(4, N - N % 4)                                  # mostly the vector paths
    page = int(rng.choice([1, 1, 1, 4, 8, 16]))
    nunits = (N + page - 1) // page
    k = int(rng.choice([1, rng.integers(1, 64), rng.integers(1, max(2, nunits // 8)), rng.integers(1, nunits + 50)]))
    kind = int(rng.integers(0, 2))
    reduce = int(rng.integers(0, 2)) if kind == 0 else 0
    bf16 = bool(rng.integers(0, 3) == 0)
    ties = bool(rng.integers(0, 4) == 0)
    g = torch.Generator().manual_seed(seed)
    logits = torch.randn(B, Hd, Tq, N, generator=g) * 2.0
    if ties:
        logits = torch.round(logits)
    if bf16:
        logits = logits.to(torch.bfloat16).float()
    lse = torch.logsumexp(logits, dim=-1)
    scores = logits if kind == 1 else torch.softmax(logits, dim=-1)
    if bf16:
        scores = scores.to(torch.bfloat16)
    hm = rng.integers(0, Hd, size=Hq).tolist()
    lens = None
    if rng.integers(0, 2):
        lens = torch.tensor([int(rng.integers(0, N + 1)) for _ in range(B)], dtype=torch.int32)
    kh = None
    if rng.integers(0, 2):
        kh = [int(x) for x in rng.integers(1, k + 1, Hd)]
    what = f"seed {seed}: B{B} Hd{Hd} Hq{Hq} Tq{Tq} N{N} k{k} page{page} kind{kind} reduce{reduce} bf16{bf16} ties{ties}"
    idx, cnt, agg = sts.sts_select(scores.to(DEV), hm, k, lse=lse.to(DEV) if kind == 1 else None,
                                   seq_lens=None if lens is None else lens.to(DEV), kind=kind, reduce=reduce,
                                   want_agg=True, page_size=page, k_head=kh)
    torch.cuda.synchronize()
    agg = agg.cpu().numpy()
    o_agg = stored_agg(oracle.aggregate(scores.float().numpy(), lse.numpy() if kind == 1 else None, kind, reduce), lens)
    if kind == 0:
        np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32), err_msg=what)
    else:
        np.testing.assert_allclose(agg, o_agg, rtol=1e-5, atol=1e-12, err_msg=what)
    # stage-wise: the ranking is checked on the GPU's own aggregate
    lens_np = None if lens is None else lens.numpy()
    if page > 1:
        src = oracle.block_scores(agg, page, lens_np)
        l2 = None if lens_np is None else ((lens_np.astype(np.int64) + page - 1) // page).astype(np.int32)
    else:
        src, l2 = agg, lens_np
    sel, c = oracle.select(src, k, l2) if kh is None else oracle.select_per_head(src, k, kh, l2)
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt, err_msg=what)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx, err_msg=what)


@pytest.mark.parametrize("seed", range(20))
def test_random_summed_weights_case(seed):
    """The draft layer's summed attention weights over random shapes (query rows 1..16, groups
    1..16, both head dims, strided caches, ragged lengths): bit for bit what the logits dump and
    the selection's aggregation give, the same index sets, and within the dump's tolerance of the
    oracle's aggregate of its own logits."""
    rng = np.random.default_rng(3000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
    Hq = Hkv * G
    Tq = int(rng.integers(1, 17))
    B = int(rng.integers(1, 4))
    N = int(rng.integers(1, 3000))
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    scale = float(rng.uniform(0.05, 0.3))
    if rng.integers(0, 2):     # interleaved K/V cache: row stride 2d
        kv = torch.stack([k, v], dim=3).contiguous().to(DEV)
        kd, vd = kv[:, :, :, 0], kv[:, :, :, 1]
    else:
        kd, vd = k.to(DEV), v.to(DEV)
    lens = torch.from_numpy(rng.integers(0, N + 1, size=B).astype(np.int32)) if rng.integers(0, 2) else None
    ld = None if lens is None else lens.to(DEV)
    A = torch.full((B, Hq, N), -3.0, dtype=torch.float32, device=DEV)
    _, lse, logits = sts.sts_dense_attn(q.to(DEV), kd, vd, scale, seq_lens=ld, want_logits=True, weights_sum_out=A)
    kk = int(rng.integers(1, N + 1))
    hm = list(range(Hq))
    idx_d, cnt_d, agg_d = sts.sts_select(logits, hm, kk, lse=lse, seq_lens=ld, kind=sts.STS_SCORES_LOGITS_LSE,
                                         want_agg=True)
    idx_a, cnt_a, _ = sts.sts_select(A.view(B, Hq, 1, N), hm, kk, seq_lens=ld)
    what = f"seed {seed}: d{d} Hkv{Hkv} G{G} Tq{Tq} B{B} N{N} k{kk}"
    assert torch.equal(idx_a, idx_d) and torch.equal(cnt_a, cnt_d), what
    ref = oracle.attn(oracle.bf16_bits(q), oracle.bf16_bits(k), oracle.bf16_bits(v), scale,
                      seq_lens=None if lens is None else lens.numpy(), want_logits=True)
    got = A.cpu().numpy()
    for b in range(B):
        n = N if lens is None else int(lens[b])
        assert torch.equal(A[b, :, :n], agg_d[b, :, :n]), what
        assert (A[b, :, n:] == 0).all(), what
        if n > 0:
            ref_A = oracle.aggregate(ref["logits"][b:b + 1, :, :, :n].copy(), ref["lse"][b:b + 1], kind=oracle.LOGITS_LSE)[0]
            assert (np.abs(got[b, :, :n] - ref_A) <= 3e-5 * ref_A + 1e-10).all(), what
