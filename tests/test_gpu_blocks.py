"""GPU parity for block-granular selection and attention, and for paged KV caches
(Section 4.2: top-k over blocks; Section 5: block granularity over scattered KV blocks;
Section 6.3: page size p_s), through the C ABI against the CPU oracle."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn, check_logits, oracle_attn, stored_agg
from workload import CONFIGS, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_qkv(seed, B, Tq, Hq, Hkv, d, N):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    return q, k, v


def random_blocks(seed, B, Hq, nblocks, kb, head_map, force_last=True):
    rng = np.random.default_rng(seed)
    idx = np.empty((B, Hq, kb), np.int32)
    for b in range(B):
        rows = {}
        for t in range(Hq):
            key = head_map[t]
            if key not in rows:
                r = rng.choice(nblocks, kb, replace=False)
                if force_last and (nblocks - 1) not in r:
                    r[0] = nblocks - 1          # the (possibly partial) last block is exercised
                rows[key] = np.sort(r)
            idx[b, t] = rows[key]
    return idx


def paged_copy(k, v, page, seed):
    """Scatter a logical cache [B,Hkv,N,d] into a pool [P,Hkv,page,d] through a random page
    table. The unfilled tail of each sequence's last page holds NaN-free garbage (large values)
    so that reading it by mistake would show."""
    B, Hkv, N, d = k.shape
    nblk = (N + page - 1) // page
    P = B * nblk + 3
    rng = np.random.default_rng(seed)
    table = rng.permutation(P)[:B * nblk].reshape(B, nblk).astype(np.int32)
    kp = torch.full((P, Hkv, page, d), 50.0, dtype=torch.bfloat16)
    vp = torch.full((P, Hkv, page, d), -50.0, dtype=torch.bfloat16)
    pad = nblk * page - N
    kpad = torch.nn.functional.pad(k, (0, 0, 0, pad), value=50.0).reshape(B, Hkv, nblk, page, d)
    vpad = torch.nn.functional.pad(v, (0, 0, 0, pad), value=-50.0).reshape(B, Hkv, nblk, page, d)
    for b in range(B):
        kp[table[b]] = kpad[b].permute(1, 0, 2, 3)
        vp[table[b]] = vpad[b].permute(1, 0, 2, 3)
    return kp, vp, torch.from_numpy(table)


@pytest.mark.parametrize("page,N,k", [(2, 1000, 77), (8, 4096, 51), (8, 20001, 300), (16, 333, 21),
                                      (7, 500, 10), (32, 9000, 282), (8, 100, 20),
                                      # shapes that take the coalesced block-sum kernel
                                      (4, 1000, 100), (16, 4096, 30), (32, 8256, 17), (64, 2560, 5),
                                      (8, 16392, 205)])
def test_block_select_bit_exact(page, N, k):
    g = torch.Generator().manual_seed(page * 1000 + N)
    B, Hd, Tq, Hq = 2, 4, 5, 8
    scores = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1)
    hm = [t // 2 for t in range(Hq)]
    lens = torch.tensor([N, max(1, N // 3)], dtype=torch.int32)
    for sl in (None, lens):
        idx, cnt, agg = sts.sts_select(scores.to(DEV), hm, k, seq_lens=None if sl is None else sl.to(DEV),
                                       want_agg=True, page_size=page)
        torch.cuda.synchronize()
        o_idx, o_cnt, o_agg = oracle.select_indices(scores.numpy(), np.asarray(hm, np.int32), k,
                                                    seq_lens=None if sl is None else sl.numpy(), page=page)
        np.testing.assert_array_equal(agg.cpu().numpy().view(np.uint32), stored_agg(o_agg, sl).view(np.uint32))
        np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
        np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)


@pytest.mark.parametrize("page", [2, 4, 8, 16, 32])
@pytest.mark.parametrize("d", [128, 64])
def test_block_sparse_attention(page, d):
    B, Tq, Hq, Hkv, N = 2, 5, 8, 2, 1003            # the last block is partial for every page size
    q, k, v = make_qkv(page + d, B, Tq, Hq, Hkv, d, N)
    hm = [t // 2 for t in range(Hq)]
    nblk = (N + page - 1) // page
    kb = max(2, nblk // 6)
    blocks = random_blocks(page, B, Hq, nblk, kb, hm)
    counts = np.full((B, Hq), kb, np.int32)
    counts[1, :2] = kb - 1                            # one set with a shorter list
    tok, tcnt = oracle.expand_blocks(blocks, counts, page, N)
    scale = 1.0 / math.sqrt(d)
    ref = oracle.attn(oracle.bf16_bits(q), oracle.bf16_bits(k), oracle.bf16_bits(v), scale, tok, tcnt)
    out, lse = sts.sts_sparse_attn(q.to(DEV), k.to(DEV), v.to(DEV), torch.from_numpy(blocks).to(DEV), scale,
                                   counts=torch.from_numpy(counts).to(DEV), head_map=hm,
                                   out_dtype=torch.float32, page_size=page)
    check_attn(out, lse, ref, what=f"block sparse p{page} d{d}")


@pytest.mark.parametrize("page", [1, 8, 16])
def test_paged_cache_sparse_and_dense(page):
    B, Tq, Hq, Hkv, d, N = 3, 5, 8, 2, 128, 777
    q, k, v = make_qkv(40 + page, B, Tq, Hq, Hkv, d, N)
    kp, vp, table = paged_copy(k, v, page, seed=page)
    hm = [t // 2 for t in range(Hq)]
    nblk = (N + page - 1) // page
    kb = max(2, nblk // 5)
    blocks = random_blocks(7, B, Hq, nblk, kb, hm)
    tok, tcnt = oracle.expand_blocks(blocks, None, page, N)
    qb, kb_, vb = oracle.bf16_bits(q), oracle.bf16_bits(k), oracle.bf16_bits(v)
    ref = oracle.attn(qb, kb_, vb, 0.09, tok, tcnt)
    out, lse = sts.sts_sparse_attn(q.to(DEV), kp.to(DEV), vp.to(DEV), torch.from_numpy(blocks).to(DEV), 0.09,
                                   head_map=hm, out_dtype=torch.float32, page_size=page,
                                   block_table=table.to(DEV), N=N)
    check_attn(out, lse, ref, what=f"paged sparse p{page}")
    # dense over the paged cache, with per-batch lengths and the logits dump
    lens = torch.tensor([N, 300, 1], dtype=torch.int32)
    dref = oracle.attn(qb, kb_, vb, 0.09, seq_lens=lens.numpy(), want_logits=True)
    dout, dlse, dlog = sts.sts_dense_attn(q.to(DEV), kp.to(DEV), vp.to(DEV), 0.09, seq_lens=lens.to(DEV),
                                          out_dtype=torch.float32, want_logits=True, page_size=page,
                                          block_table=table.to(DEV), N=N)
    check_attn(dout, dlse, dref, what=f"paged dense p{page}")
    lg = dlog.cpu().numpy()
    for b, n in enumerate(lens.tolist()):
        check_logits(lg[b, :, :, :n], dref["logits"][b, :, :, :n], what=f"batch {b}")


def test_block_chain_select_then_attention_on_the_4k_configuration():
    page = 8
    w = make_workload(CONFIGS["c1"], seed=3)
    kb = math.ceil(w.k_budget / page)                 # same token budget, in blocks of 8
    q, k, v, scores = w.q.to(DEV), w.k.to(DEV), w.v.to(DEV), w.scores.to(DEV)
    idx, cnt, _ = sts.sts_select(scores, w.head_map, kb, page_size=page)
    out, lse = sts.sts_sparse_attn(q, k, v, idx, w.scale, counts=cnt, head_map=w.head_map,
                                   out_dtype=torch.float32, page_size=page)
    torch.cuda.synchronize()
    o_idx, o_cnt, _ = oracle.select_indices(w.scores.numpy(), w.head_map.numpy(), kb, page=page)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    tok, tcnt = oracle.expand_blocks(o_idx, o_cnt, page, w.cfg.N)
    ref = oracle_attn(q, k, v, w.scale, torch.from_numpy(tok), torch.from_numpy(tcnt))
    check_attn(out, lse, ref, what="block chain")


def test_page_arguments_are_validated():
    q, k, v = make_qkv(1, 1, 5, 8, 2, 128, 256)
    idx = torch.zeros(1, 8, 4, dtype=torch.int32, device=DEV)
    with pytest.raises(sts.StsError):
        sts.sts_sparse_attn(q.to(DEV), k.to(DEV), v.to(DEV), idx, 0.09, page_size=3)
    with pytest.raises(sts.StsError):
        sts.sts_sparse_attn(q.to(DEV), k.to(DEV), v.to(DEV), idx, 0.09, page_size=64)


@pytest.mark.parametrize("page,N,k,kind,bf16", [
    (8, 65536, 700, 0, False),       # 8192 blocks per row: fused aggregation + ranking out of LDS
    (16, 262144, 1600, 0, False),    # 16384 blocks per row: the limit of that path
    (8, 262144, 3000, 0, False),     # 32768 blocks per row: fused aggregation + histogram pipeline
    (8, 65536, 700, 1, True),        # scaled logits stored as bf16
    (8, 65528, 700, 0, False),       # N % page == 0 but a ragged last chunk
    (8, 65532, 700, 0, False),       # N % page != 0: separate aggregation and block kernels
])
def test_block_select_fused_paths(page, N, k, kind, bf16):
    """Block-granular selection through its launch sequences, with and without the per-token
    aggregate on request, per-head budgets and ragged lengths; stage-wise against the oracle."""
    from test_gpu_select import launched
    g = torch.Generator().manual_seed(N + page + kind)
    B, Hd, Tq, Hq = 2, 3, 2, 6
    logits = torch.randn(B, Hd, Tq, N, generator=g) * 2
    if bf16:
        logits = logits.to(torch.bfloat16).float()
    lse = torch.logsumexp(logits, dim=-1)
    scores = logits if kind == 1 else torch.softmax(logits, dim=-1)
    sd = (scores.to(torch.bfloat16) if bf16 else scores).to(DEV)
    hm = [2, 0, 0, 1, 2, 1]
    kh = [k, 3, max(1, k // 2)]
    lens = torch.tensor([N, N // 2 + 3], dtype=torch.int32)
    got = {}
    def call(want_agg):
        got["r"] = sts.sts_select(sd, hm, k, lse=lse.to(DEV) if kind == 1 else None, seq_lens=lens.to(DEV), kind=kind,
                                  want_agg=want_agg, page_size=page, k_head=kh)
    kinds = launched(lambda: call(True))
    nblk = (N + page - 1) // page
    if N % page:
        assert "select_block" in kinds
    elif nblk <= 16384:
        assert kinds == {"select_agg", "select_small"}
    else:
        assert kinds == {"select_clear", "select_agg", "select_hist", "select_write"}
    idx, cnt, agg = got["r"]
    agg = agg.cpu().numpy()
    o_agg = stored_agg(oracle.aggregate(scores.numpy(), lse.numpy() if kind == 1 else None, kind, 0), lens)
    if kind == 0:
        np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    else:
        np.testing.assert_allclose(agg, o_agg, rtol=1e-5, atol=1e-12)
    blk = oracle.block_scores(agg, page, lens.numpy())
    l2 = ((lens.numpy().astype(np.int64) + page - 1) // page).astype(np.int32)
    sel, c = oracle.select_per_head(blk, k, kh, l2)
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    call(False)                                            # the lists do not depend on the optional output
    assert torch.equal(got["r"][0], idx) and torch.equal(got["r"][1], cnt)


@pytest.mark.parametrize("N,page,nb", [(64, 8, 43), (40000, 16, 39989), (300000, 8, 299995)])
def test_partial_last_block_is_ranked_on_the_gpu(N, page, nb):
    """The planted case of the oracle's pin on every selection path (one workgroup per row, fused
    block sums + LDS ranking, the multi-workgroup pipeline): the best score sits in the partial
    last block of a ragged length, a larger one just past the length must not count."""
    B, Hd, Tq = 1, 2, 2
    P = torch.full((B, Hd, Tq, N), 0.01)
    P[0, :, :, nb - 1] = 5.0
    if nb < N:
        P[0, :, :, nb] = 50.0
    lens = torch.tensor([nb], dtype=torch.int32)
    last = (nb - 1) // page
    for k in (1, 3):
        idx, cnt, _ = sts.sts_select(P.to(DEV), [0, 1], k, seq_lens=lens.to(DEV), page_size=page)
        o_idx, o_cnt, _ = oracle.select_indices(P.numpy(), np.asarray([0, 1], np.int32), k, seq_lens=lens.numpy(), page=page)
        np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
        np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
        assert last in o_idx[0, 0].tolist()
