"""GPU parity for the two-dimensional masks of prefill (Section 4.2: every query token of a head
has an index set of its own): per-row selection, the union of a block's row sets with its row
bits (sts_union_rows), and attention that gathers the union once and lets row i see only the
entries whose word has bit i set (row_mask). Integer work bit-exact, attention within the
tolerance of the other attention tests, all against the oracle's definitions."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def random_rows(seed, B, Hd, Tq, N, k, ragged=True, sort=True):
    rng = np.random.default_rng(seed)
    sel = np.full((B, Hd, Tq, k), -1, np.int32)
    cnt = np.zeros((B, Hd, Tq), np.int32)
    for b in range(B):
        for j in range(Hd):
            hot = rng.choice(N, min(N, 3 * k), replace=False)        # rows of a block share most of their tokens
            for i in range(Tq):
                c = int(rng.integers(0, k + 1)) if ragged else k
                row = rng.choice(hot, min(c, len(hot)), replace=False)
                c = len(row)
                sel[b, j, i, :c] = np.sort(row) if sort else row
                cnt[b, j, i] = c
    return sel, cnt


@pytest.mark.parametrize("B,Hd,Hq,Tq,N,k", [
    (2, 3, 6, 5, 1000, 40),          # one chunk
    (1, 2, 4, 16, 70000, 900),       # three chunks, 16 rows
    (2, 4, 4, 1, 33000, 100),        # a single row: the union is the row
    (1, 1, 2, 7, 32768, 5000),       # exactly one chunk, long lists
])
def test_union_of_rows_bit_exact(B, Hd, Hq, Tq, N, k):
    sel, cnt = random_rows(N + k, B, Hd, Tq, N, k)
    hm = [(t * Hd) // Hq for t in range(Hq)]
    idx, mask, ucnt = sts.sts_union_rows(torch.from_numpy(sel).to(DEV), torch.from_numpy(cnt).to(DEV), hm, N)
    torch.cuda.synchronize()
    o_idx, o_mask, o_cnt = oracle.union_rows(sel, cnt, hm, pitch=idx.shape[2])
    np.testing.assert_array_equal(ucnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(mask.cpu().numpy().view(np.uint16), o_mask)


def test_union_unsorted_rows_no_counts_and_a_short_pitch():
    B, Hd, Hq, Tq, N, k = 1, 2, 3, 4, 5000, 64
    sel, _ = random_rows(7, B, Hd, Tq, N, k, ragged=False, sort=False)
    hm = [1, 0, 1]
    idx, mask, ucnt = sts.sts_union_rows(torch.from_numpy(sel).to(DEV), None, hm, N)
    o_idx, o_mask, o_cnt = oracle.union_rows(sel, None, hm, pitch=idx.shape[2])
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(mask.cpu().numpy().view(np.uint16), o_mask)
    np.testing.assert_array_equal(ucnt.cpu().numpy(), o_cnt)
    # a pitch below the union's size keeps its first entries and says so in the counts
    short = int(o_cnt.min()) - 5
    idx2, mask2, cnt2 = sts.sts_union_rows(torch.from_numpy(sel).to(DEV), None, hm, N, pitch=short)
    np.testing.assert_array_equal(idx2.cpu().numpy(), o_idx[:, :, :short])
    np.testing.assert_array_equal(mask2.cpu().numpy().view(np.uint16), o_mask[:, :, :short])
    assert (cnt2.cpu().numpy() == short).all()


@pytest.mark.parametrize("B,Hd,Tq,N,k,lens", [(2, 4, 8, 3000, 100, None), (2, 2, 16, 40000, 700, [40000, 12345]),
                                             (1, 16, 16, 9000, 64, None)])
def test_per_row_selection_bit_exact(B, Hd, Tq, N, k, lens):
    g = torch.Generator().manual_seed(N)
    scores = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1)
    ln = None if lens is None else torch.tensor(lens, dtype=torch.int32)
    ridx, rcnt = sts.sts_select_rows(scores.to(DEV), k, seq_lens=None if ln is None else ln.to(DEV))
    torch.cuda.synchronize()
    o_sel, o_cnt = oracle.select_rows(scores.numpy(), k, seq_lens=None if ln is None else ln.numpy())
    np.testing.assert_array_equal(rcnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(ridx.cpu().numpy(), o_sel)


@pytest.mark.parametrize("swap", ["whole list shuffled", "two entries swapped across chunks", "ascending"])
def test_union_over_several_chunks_does_not_depend_on_the_order_inside_a_list(swap):
    """Long contexts are walked in chunks of 32768 tokens, each chunk reading its own segment of
    every (ascending) list; a list in any other order must give the same union (the kernel notices
    and reads every entry for every chunk instead)."""
    B, Hd, Hq, Tq, N, k = 2, 2, 4, 9, 150000, 3000
    sel, cnt = random_rows(91, B, Hd, Tq, N, k)
    rng = np.random.default_rng(5)
    if swap == "whole list shuffled":
        for b in range(B):
            for j in range(Hd):
                for i in range(Tq):
                    c = cnt[b, j, i]
                    sel[b, j, i, :c] = rng.permutation(sel[b, j, i, :c])
    elif swap == "two entries swapped across chunks":
        c = cnt[1, 1, 3]
        assert c > 10 and sel[1, 1, 3, 0] < 32768 <= sel[1, 1, 3, c - 1]
        sel[1, 1, 3, [0, c - 1]] = sel[1, 1, 3, [c - 1, 0]]
    hm = [0, 1, 1, 0]
    idx, mask, ucnt = sts.sts_union_rows(torch.from_numpy(sel).to(DEV), torch.from_numpy(cnt).to(DEV), hm, N)
    torch.cuda.synchronize()
    o_idx, o_mask, o_cnt = oracle.union_rows(sel, cnt, hm, pitch=idx.shape[2])
    np.testing.assert_array_equal(ucnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(mask.cpu().numpy().view(np.uint16), o_mask)


def make_qkv(seed, B, Tq, Hq, Hkv, d, N):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    return q, k, v


@pytest.mark.parametrize("B,Tq,Hq,Hkv,d,N,k,shared", [
    (2, 5, 8, 2, 128, 2000, 60, 2),      # pairs of heads share the rows' lists: one query tile
    (1, 16, 4, 2, 128, 3000, 200, 1),    # 16 rows, every head on its own
    (1, 16, 8, 2, 128, 9000, 900, 2),    # 32 query rows per unit (two query tiles), lists long enough to be split
    (1, 8, 8, 1, 64, 2500, 120, 8),      # 64 query rows per unit (four query tiles), head size 64
    (2, 3, 4, 2, 64, 600, 30, 1),
])
def test_attention_with_a_list_per_query_row(B, Tq, Hq, Hkv, d, N, k, shared):
    q, kc, vc = make_qkv(Tq * 100 + N, B, Tq, Hq, Hkv, d, N)
    Hd = Hq // shared
    hm = [t // shared for t in range(Hq)]
    sel, cnt = random_rows(N + d, B, Hd, Tq, N, k)
    cnt[0, 0, 0] = 0                                   # a row that keeps nothing: out 0, lse -inf
    sel[0, 0, 0] = -1
    scale = 1 / math.sqrt(d)
    idx, mask, ucnt = sts.sts_union_rows(torch.from_numpy(sel).to(DEV), torch.from_numpy(cnt).to(DEV), hm, N)
    out, lse = sts.sts_sparse_attn(q.to(DEV), kc.to(DEV), vc.to(DEV), idx, scale, counts=ucnt, head_map=hm,
                                   row_mask=mask, out_dtype=torch.float32)
    torch.cuda.synchronize()
    rows = np.stack([sel[:, j] for j in hm], axis=1)               # [B,Hq,Tq,k]
    rcnt = np.stack([cnt[:, j] for j in hm], axis=1)
    ref = oracle.attn_rows(oracle.bf16_bits(q), oracle.bf16_bits(kc), oracle.bf16_bits(vc), scale, rows, rcnt)
    check_attn(out, lse, ref, what="list per row")
    assert np.isneginf(lse.cpu().numpy()[0, 0:shared, 0]).all() and (out.cpu().numpy()[0, 0, 0:shared] == 0).all()
    # without the hint every head is a unit of its own: same answer; and in bf16
    out2, lse2 = sts.sts_sparse_attn(q.to(DEV), kc.to(DEV), vc.to(DEV), idx, scale, counts=ucnt, row_mask=mask)
    check_attn(out2, lse2, ref, what="list per row, unhinted, bf16")
    # all bits set is the plain shared list
    full = torch.full_like(mask, -1)
    out3, lse3 = sts.sts_sparse_attn(q.to(DEV), kc.to(DEV), vc.to(DEV), idx, scale, counts=ucnt, head_map=hm, row_mask=full,
                                     out_dtype=torch.float32)
    out4, lse4 = sts.sts_sparse_attn(q.to(DEV), kc.to(DEV), vc.to(DEV), idx, scale, counts=ucnt, head_map=hm,
                                     out_dtype=torch.float32)
    assert torch.equal(out3, out4) and torch.equal(lse3, lse4)


def test_prefill_block_chain_scores_to_attention_with_own_tokens():
    """A 16-row prefill block end to end: per-row selection from the draft scores (causal visible
    lengths per block), union + row bits, attention over the shared cache with the block's own
    tokens appended causally; against the oracle's row-by-row definition on a cache that holds the
    block's own tokens as ordinary rows."""
    g = torch.Generator().manual_seed(11)
    NB, T, Hq, Hkv, Hd, d, P0, k = 3, 16, 8, 2, 4, 128, 700, 80
    N = P0 + T * NB
    hm = [t // 2 for t in range(Hq)]
    scale = 1 / math.sqrt(d)
    q = torch.randn(NB, T, Hq, d, generator=g).to(torch.bfloat16)
    kc = (torch.randn(1, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    vc = (torch.randn(1, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    starts = torch.tensor([P0 + T * j for j in range(NB)], dtype=torch.int32)          # cached tokens block j sees
    logits = torch.randn(NB, Hd, T, N, generator=g) * 2
    for j in range(NB):
        logits[j, :, :, starts[j]:] = float("-inf")
    scores = torch.softmax(logits, dim=-1)
    ridx, rcnt = sts.sts_select_rows(scores.to(DEV), k, seq_lens=starts.to(DEV))
    idx, mask, ucnt = sts.sts_union_rows(ridx, rcnt, hm, N)
    own = lambda c: torch.stack([c[0, :, P0 + T * j:P0 + T * (j + 1)].permute(1, 0, 2) for j in range(NB)]).contiguous()
    out, lse = sts.sts_sparse_attn(q.to(DEV), kc.to(DEV).expand(NB, -1, -1, -1), vc.to(DEV).expand(NB, -1, -1, -1), idx, scale,
                                   counts=ucnt, head_map=hm, row_mask=mask, out_dtype=torch.float32,
                                   k_new=own(kc).to(DEV), v_new=own(vc).to(DEV), causal=True)
    torch.cuda.synchronize()
    o_sel, o_cnt = oracle.select_rows(scores.numpy(), k, seq_lens=starts.numpy())
    np.testing.assert_array_equal(ridx.cpu().numpy(), o_sel)
    o_idx, o_mask, o_ucnt = oracle.union_rows(o_sel, o_cnt, hm, pitch=idx.shape[2])
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(mask.cpu().numpy().view(np.uint16), o_mask)
    # oracle: row i of block j attends to its own list plus tokens starts[j] .. starts[j] + i of the cache
    rows = np.full((NB, Hq, T, k + T), -1, np.int32)
    rc = np.zeros((NB, Hq, T), np.int32)
    for j in range(NB):
        for t in range(Hq):
            for i in range(T):
                c = int(o_cnt[j, hm[t], i])
                mine = list(o_sel[j, hm[t], i, :c]) + list(range(int(starts[j]), int(starts[j]) + i + 1))
                rows[j, t, i, :len(mine)] = mine
                rc[j, t, i] = len(mine)
    kx = oracle.bf16_bits(kc.expand(NB, -1, -1, -1).contiguous())
    vx = oracle.bf16_bits(vc.expand(NB, -1, -1, -1).contiguous())
    ref = oracle.attn_rows(oracle.bf16_bits(q), kx, vx, scale, rows, rc)
    check_attn(out, lse, ref, what="prefill block with a mask per row")
