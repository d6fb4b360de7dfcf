"""Pins for the selection half of the oracle (aggregate, top-k with ties, remap).

The paper prints no worked numeric example for these steps (Section 4.2 states the
operation only), so the oracle is pinned by: the O(N^2) counting definition of "k largest,
ties to the lower index", closed-form special cases, invariants, torch.topk value
multisets, and hand-computed fixtures under tests/golden/.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_select(a: np.ndarray, c: int):
    """n is kept iff #{m: a[m] > a[n]} + #{m < n: a[m] == a[n]} < c (counting definition)."""
    n = a.shape[0]
    keep = []
    for i in range(n):
        rank = int(np.sum(a > a[i])) + int(np.sum(a[:i] == a[i]))
        if rank < c:
            keep.append(i)
    return np.array(keep, np.int32)


# ------------------------------------------------------------------ aggregate


def test_aggregate_sum_is_left_to_right_fp32():
    # 2^24 + 1 + 1: fp32 left-to-right gives 2^24 (each +1 is lost); any other order or a
    # wider accumulator gives 2^24 + 2.
    P = np.zeros((1, 1, 3, 2), np.float32)
    P[0, 0, :, 0] = [16777216.0, 1.0, 1.0]
    P[0, 0, :, 1] = [1.0, 1.0, 16777216.0]
    A = oracle.aggregate(P)
    assert A[0, 0, 0] == np.float32(16777216.0)
    assert A[0, 0, 1] == np.float32(16777218.0)


def test_aggregate_matches_sequential_numpy_fp32():
    rng = np.random.default_rng(1)
    P = rng.random((2, 3, 5, 257), dtype=np.float32)
    acc = P[:, :, 0, :].copy()
    for i in range(1, 5):
        acc = (acc + P[:, :, i, :]).astype(np.float32)
    np.testing.assert_array_equal(oracle.aggregate(P), acc)
    np.testing.assert_array_equal(oracle.aggregate(P, reduce=oracle.MAX), P.max(axis=2))


def test_aggregate_single_row_is_identity():
    rng = np.random.default_rng(2)
    P = rng.standard_normal((1, 2, 1, 33)).astype(np.float32)
    np.testing.assert_array_equal(oracle.aggregate(P)[:, :, :], P[:, :, 0, :])


def test_aggregate_logits_lse_recovers_softmax():
    rng = np.random.default_rng(3)
    S = rng.standard_normal((2, 2, 4, 100)).astype(np.float32) * 3
    lse = torch.logsumexp(torch.from_numpy(S).double(), dim=-1).float().numpy()
    A = oracle.aggregate(S, lse, kind=oracle.LOGITS_LSE)
    ref = torch.softmax(torch.from_numpy(S).double(), dim=-1).sum(dim=2).numpy()
    np.testing.assert_allclose(A, ref, rtol=2e-6, atol=1e-9)
    # every row of probabilities sums to one, so the aggregate sums to Tq
    np.testing.assert_allclose(A.sum(-1), 4.0, rtol=1e-5)


# --------------------------------------------------------------------- select


@pytest.mark.parametrize("seed", range(6))
def test_select_matches_counting_definition_random(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(1, 300))
    k = int(rng.integers(1, N + 3))
    A = rng.standard_normal((2, 3, N)).astype(np.float32)
    sel, cnt = oracle.select(A, k)
    c = min(k, N)
    assert (cnt == c).all()
    for b in range(2):
        for j in range(3):
            np.testing.assert_array_equal(sel[b, j, :c], brute_select(A[b, j], c))
            assert (sel[b, j, c:] == -1).all()


@pytest.mark.parametrize("levels", [1, 2, 4])
def test_select_ties_go_to_lower_index(levels):
    rng = np.random.default_rng(10 + levels)
    N = 200
    A = rng.integers(0, levels, size=(1, 4, N)).astype(np.float32)
    for k in (1, 7, 64, 199, 200):
        sel, _ = oracle.select(A, k)
        for j in range(4):
            np.testing.assert_array_equal(sel[0, j, :k], brute_select(A[0, j], k))


def test_select_special_cases():
    N, k = 97, 13
    const = np.full((1, 1, N), 0.25, np.float32)
    dec = np.arange(N, 0, -1, dtype=np.float32).reshape(1, 1, N)
    inc = np.arange(N, dtype=np.float32).reshape(1, 1, N)
    np.testing.assert_array_equal(oracle.select(const, k)[0][0, 0], np.arange(k))
    np.testing.assert_array_equal(oracle.select(dec, k)[0][0, 0], np.arange(k))
    np.testing.assert_array_equal(oracle.select(inc, k)[0][0, 0], np.arange(N - k, N))
    np.testing.assert_array_equal(oracle.select(inc, N)[0][0, 0], np.arange(N))
    # k = 1 is the first argmax
    a = np.array([[[1, 5, 3, 5, 2]]], np.float32)
    assert oracle.select(a, 1)[0][0, 0, 0] == 1
    # k > N pads with -1
    sel, cnt = oracle.select(a, 8)
    np.testing.assert_array_equal(sel[0, 0], [0, 1, 2, 3, 4, -1, -1, -1])
    assert cnt[0, 0] == 5


def test_select_signed_zero_denormal_negative():
    a = np.array([[[-0.0, 0.0, 1e-45, -1e-45, -3.0, 0.0, -0.0, 2.0]]], np.float32)
    # order: 2.0(7), 1e-45(2), zeros by index (0,1,5,6), -1e-45(3), -3(4)
    for k, want in [(1, [7]), (2, [2, 7]), (3, [0, 2, 7]), (4, [0, 1, 2, 7]), (5, [0, 1, 2, 5, 7]),
                    (6, [0, 1, 2, 5, 6, 7]), (7, [0, 1, 2, 3, 5, 6, 7])]:
        np.testing.assert_array_equal(oracle.select(a, k)[0][0, 0], want)
        np.testing.assert_array_equal(brute_select(a[0, 0], k), want)


def test_select_value_multiset_matches_torch_topk():
    rng = np.random.default_rng(5)
    A = rng.standard_normal((2, 4, 4096)).astype(np.float32)
    k = 410
    sel, _ = oracle.select(A, k)
    tv, ti = torch.topk(torch.from_numpy(A), k, dim=-1)
    got = np.take_along_axis(A, sel, axis=-1)
    np.testing.assert_array_equal(np.sort(got, -1), np.sort(tv.numpy(), -1))
    # tie-free input: the index sets agree as well
    np.testing.assert_array_equal(sel, np.sort(ti.numpy(), -1))
    # invariants: ascending, every kept score >= every dropped score
    assert (np.diff(sel, axis=-1) > 0).all()
    for b in range(2):
        for j in range(4):
            mask = np.ones(4096, bool)
            mask[sel[b, j]] = False
            assert A[b, j][sel[b, j]].min() >= A[b, j][mask].max()


def test_select_seq_lens():
    rng = np.random.default_rng(6)
    A = rng.standard_normal((3, 2, 50)).astype(np.float32)
    lens = np.array([50, 7, 0], np.int32)
    sel, cnt = oracle.select(A, 10, lens)
    np.testing.assert_array_equal(cnt, [[10, 10], [7, 7], [0, 0]])
    np.testing.assert_array_equal(sel[1, 0, :7], np.arange(7))
    assert (sel[1, :, 7:] == -1).all() and (sel[2] == -1).all()
    np.testing.assert_array_equal(sel[0, 1], brute_select(A[0, 1], 10))


def test_per_head_budgets_are_nested_prefixes_of_the_ranking():
    """With the deterministic tie rule the c best tokens contain the c' < c best ones, so the
    list of a head with a smaller budget is the larger list filtered; budgets equal to k change
    nothing; each head is checked against the counting definition by brute force."""
    rng = np.random.default_rng(12)
    A = np.round(rng.standard_normal((2, 3, 200)) * 2).astype(np.float32) / 2    # many ties
    lens = np.array([200, 37], np.int32)
    k, kh = 40, [40, 1, 13]
    full, cfull = oracle.select(A, k, lens)
    sel, cnt = oracle.select_per_head(A, k, kh, lens)
    np.testing.assert_array_equal(cnt, np.minimum(np.array(kh)[None, :], lens[:, None]))
    np.testing.assert_array_equal(sel[:, 0], full[:, 0])
    for b in range(2):
        for j in range(3):
            c = cnt[b, j]
            want = brute_select(A[b, j, :lens[b]], kh[j])
            np.testing.assert_array_equal(sel[b, j, :c], want)
            assert (sel[b, j, c:] == -1).all()
            assert set(sel[b, j, :c]) <= set(full[b, j, :cfull[b, j]])
    idx, counts, _ = oracle.select_indices(np.repeat(A[:, :, None, :], 1, axis=2), np.array([2, 0, 1, 2], np.int32),
                                           k, seq_lens=lens, k_head=kh)
    np.testing.assert_array_equal(idx[:, 0], sel[:, 2])
    np.testing.assert_array_equal(idx[:, 3], sel[:, 2])
    np.testing.assert_array_equal(counts[:, 1], cnt[:, 0])


def test_select_rejects_nan():
    a = np.array([[[0.0, np.nan, 1.0]]], np.float32)
    with pytest.raises(ValueError):
        oracle.select(a, 2)


def test_select_golden_fixture():
    with open(os.path.join(GOLDEN, "select_handworked.json")) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        P = np.array(case["probs"], np.float32)[None]          # [1,Hd,Tq,N]
        hm = np.array(case["head_map"], np.int32)
        idx, cnt, A = oracle.select_indices(P, hm, case["k"], page=case.get("page", 1), k_head=case.get("k_head"))
        np.testing.assert_array_equal(idx[0], np.array(case["indices"], np.int32))
        np.testing.assert_allclose(A[0], np.array(case["agg"], np.float32), rtol=0, atol=1e-7)
        if "counts" in case:
            np.testing.assert_array_equal(cnt[0], np.array(case["counts"], np.int32))
        if "block_scores" in case:
            np.testing.assert_array_equal(oracle.block_scores(A, case["page"])[0],
                                          np.array(case["block_scores"], np.float32))


# ---------------------------------------------------------------------- remap


def test_remap_rows_follow_head_map():
    rng = np.random.default_rng(7)
    A = rng.standard_normal((2, 4, 64)).astype(np.float32)
    sel, cnt = oracle.select(A, 9)
    hm = np.array([0, 0, 3, 1, 1, 1, 2, 0], np.int32)
    idx, counts = oracle.remap(sel, cnt, hm)
    for t, j in enumerate(hm):
        np.testing.assert_array_equal(idx[:, t], sel[:, j])
        np.testing.assert_array_equal(counts[:, t], cnt[:, j])
    perm = rng.permutation(8)
    idx2, _ = oracle.remap(sel, cnt, hm[perm])
    np.testing.assert_array_equal(idx2, idx[:, perm])
    with pytest.raises(ValueError):
        oracle.remap(sel, cnt, np.array([0, 4], np.int32))


def test_reduction_switch_reaches_the_selection():
    """Sum and maximum over the query rows rank differently; the whole selection follows the switch."""
    P = np.zeros((1, 1, 3, 4), np.float32)
    P[0, 0, :, 0] = [0.3, 0.3, 0.3]         # sum 0.9, max 0.3
    P[0, 0, :, 1] = [0.8, 0.0, 0.0]         # sum 0.8, max 0.8
    P[0, 0, :, 2] = [0.1, 0.1, 0.1]
    hm = np.array([0], np.int32)
    i_sum, _, a_sum = oracle.select_indices(P, hm, 1, reduce=oracle.SUM)
    i_max, _, a_max = oracle.select_indices(P, hm, 1, reduce=oracle.MAX)
    assert i_sum[0, 0, 0] == 0 and i_max[0, 0, 0] == 1
    assert a_max[0, 0].tolist() == [np.float32(0.3), np.float32(0.8), np.float32(0.1), 0.0]
