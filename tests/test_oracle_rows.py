"""Pins of the oracle's per-row (two-dimensional) masks (Section 4.2: during prefill every query
token has an index set of its own): the union of a block's row sets with its row bits, and
attention with one index set per query row."""
import numpy as np
import torch

import oracle


def _rows(rng, B, Hd, Tq, N, k, ragged=True):
    sel = np.full((B, Hd, Tq, k), -1, np.int32)
    cnt = np.zeros((B, Hd, Tq), np.int32)
    for b in range(B):
        for j in range(Hd):
            for i in range(Tq):
                c = int(rng.integers(0, k + 1)) if ragged else k
                sel[b, j, i, :c] = np.sort(rng.choice(N, c, replace=False))
                cnt[b, j, i] = c
    return sel, cnt


def test_union_is_the_set_union_and_the_bits_say_who_keeps_what():
    rng = np.random.default_rng(0)
    B, Hd, Tq, N, k = 2, 3, 5, 60, 9
    sel, cnt = _rows(rng, B, Hd, Tq, N, k)
    hm = [2, 0, 0, 1]
    union, mask, ucnt = oracle.union_rows(sel, cnt, hm)
    for b in range(B):
        for t, j in enumerate(hm):
            sets = [set(sel[b, j, i, :cnt[b, j, i]].tolist()) for i in range(Tq)]
            want = sorted(set().union(*sets))
            c = ucnt[b, t]
            assert union[b, t, :c].tolist() == want and (union[b, t, c:] == -1).all() and (mask[b, t, c:] == 0).all()
            for p, n in enumerate(want):
                assert mask[b, t, p] == sum(1 << i for i in range(Tq) if n in sets[i])
    # heads mapped to the same draft head get the same union
    np.testing.assert_array_equal(union[:, 1], union[:, 2])
    # and the way back gives every row its own list again
    rows, rc = oracle.rows_of_union(union, mask, ucnt, Tq, k)
    for t, j in enumerate(hm):
        np.testing.assert_array_equal(rc[:, t], cnt[:, j])
        np.testing.assert_array_equal(rows[:, t], sel[:, j])


def test_union_closed_forms():
    # identical rows: the union is the row, every bit set; disjoint rows: concatenation, one bit each
    row = np.array([3, 7, 20, 21], np.int32)
    sel = np.tile(row, (1, 1, 4, 1))
    union, mask, cnt = oracle.union_rows(sel, None, [0])
    assert cnt[0, 0] == 4 and union[0, 0].tolist() == row.tolist() and (mask[0, 0] == 0b1111).all()
    sel = np.arange(12, dtype=np.int32).reshape(1, 1, 3, 4)
    union, mask, cnt = oracle.union_rows(sel, None, [0])
    assert cnt[0, 0] == 12 and union[0, 0].tolist() == list(range(12))
    assert mask[0, 0].tolist() == [1] * 4 + [2] * 4 + [4] * 4
    # an empty block
    union, mask, cnt = oracle.union_rows(np.full((1, 1, 2, 3), -1, np.int32), np.zeros((1, 1, 2), np.int32), [0], pitch=5)
    assert cnt[0, 0] == 0 and (union == -1).all() and union.shape[2] == 5


def test_select_rows_is_the_single_row_selection_of_every_row():
    g = torch.Generator().manual_seed(1)
    B, Hd, Tq, N, k = 2, 2, 4, 200, 17
    scores = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1).numpy()
    lens = np.array([200, 77], np.int32)
    sel, cnt = oracle.select_rows(scores, k, seq_lens=lens)
    for i in range(Tq):
        idx, c, _ = oracle.select_indices(scores[:, :, i:i + 1], np.arange(Hd, dtype=np.int32), k, seq_lens=lens)
        np.testing.assert_array_equal(sel[:, :, i], idx)
        np.testing.assert_array_equal(cnt[:, :, i], c)
    # against torch.topk on a tie-free input: same sets
    top = torch.topk(torch.from_numpy(scores[0]), k, dim=-1).indices.sort(dim=-1).values.numpy()
    np.testing.assert_array_equal(sel[0], top)


def test_rows_with_one_shared_list_equal_the_shared_list_result_bit_for_bit():
    g = torch.Generator().manual_seed(2)
    B, Tq, Hq, Hkv, d, N, k = 1, 3, 4, 2, 64, 90, 20
    q = oracle.bf16_bits(torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16))
    kk = oracle.bf16_bits((torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16))
    vv = oracle.bf16_bits((torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16))
    rng = np.random.default_rng(3)
    idx = np.stack([np.sort(rng.choice(N, k, replace=False)) for _ in range(B * Hq)]).reshape(B, Hq, k).astype(np.int32)
    shared = oracle.attn(q, kk, vv, 0.2, idx)
    rows = oracle.attn_rows(q, kk, vv, 0.2, np.repeat(idx[:, :, None, :], Tq, axis=2))
    np.testing.assert_array_equal(rows["out"], shared["out"])
    np.testing.assert_array_equal(rows["lse"], shared["lse"])


def test_attention_per_row_equals_masked_full_softmax():
    """Brute force (torch, fp64): full softmax over all N keys with -inf wherever the row does not
    keep the key equals attention over the row's own list."""
    g = torch.Generator().manual_seed(4)
    B, Tq, Hq, Hkv, d, N, k = 2, 4, 4, 2, 32, 50, 11
    qt = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    kt = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    vt = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16)
    rng = np.random.default_rng(5)
    sel, cnt = _rows(rng, B, Hq, Tq, N, k)
    cnt = np.maximum(cnt, 1)                              # at least one key per row
    for b in range(B):
        for t in range(Hq):
            for i in range(Tq):
                sel[b, t, i, :cnt[b, t, i]] = np.sort(rng.choice(N, cnt[b, t, i], replace=False))
    got = oracle.attn_rows(oracle.bf16_bits(qt), oracle.bf16_bits(kt), oracle.bf16_bits(vt), 0.3, sel, cnt)
    G = Hq // Hkv
    for b in range(B):
        for t in range(Hq):
            for i in range(Tq):
                s = (kt[b, t // G].double() @ qt[b, i, t].double()) * 0.3
                keep = torch.zeros(N, dtype=torch.bool)
                keep[torch.from_numpy(sel[b, t, i, :cnt[b, t, i]].astype(np.int64))] = True
                s = s.masked_fill(~keep, float("-inf"))
                p = torch.softmax(s, dim=0)
                want = p @ vt[b, t // G].double()
                assert np.abs(got["out"][b, i, t] - want.numpy()).max() < 1e-6
                assert abs(got["lse"][b, t, i] - torch.logsumexp(s, 0).item()) < 1e-5
