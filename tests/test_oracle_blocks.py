"""Pins for block-granular selection in the oracle (Section 4.2: top-k over blocks; Section 6.3:
page size p_s). The paper names no block operator and prints no example; the oracle sums the
aggregated scores of a block's tokens left to right in fp32. Pins: reshape-sum on exactly
representable values, page 1 identity, truncation at the valid length, rounding order, brute
force block top-k, and block expansion feeding the (already pinned) attention."""
import math

import numpy as np
import torch

import oracle
from test_oracle_select import brute_select


def test_block_scores_match_reshape_sum_on_exact_values():
    rng = np.random.default_rng(0)
    A = (rng.integers(0, 64, size=(2, 3, 96)) / 64.0).astype(np.float32)     # dyadic: sums exact
    for page in (1, 2, 4, 8, 16, 32):
        got = oracle.block_scores(A, page)
        np.testing.assert_array_equal(got, A.reshape(2, 3, 96 // page, page).sum(-1))
    np.testing.assert_array_equal(oracle.block_scores(A, 1), A)


def test_block_scores_partial_last_block_and_seq_lens():
    A = np.arange(1, 11, dtype=np.float32).reshape(1, 1, 10)
    np.testing.assert_array_equal(oracle.block_scores(A, 4)[0, 0], [10, 26, 19])
    np.testing.assert_array_equal(oracle.block_scores(A, 4, np.array([6], np.int32))[0, 0], [10, 11, 0])
    np.testing.assert_array_equal(oracle.block_scores(A, 4, np.array([0], np.int32))[0, 0], [0, 0, 0])


def test_block_scores_add_left_to_right_in_fp32():
    A = np.array([[[16777216.0, 1.0, 1.0, 0.0, 1.0, 1.0, 16777216.0, 0.0]]], np.float32)
    got = oracle.block_scores(A, 4)[0, 0]
    assert got[0] == np.float32(16777216.0) and got[1] == np.float32(16777218.0)


def test_block_selection_matches_brute_force_and_expansion():
    rng = np.random.default_rng(1)
    B, Hd, Tq, N, page, kb = 2, 3, 4, 203, 8, 5
    P = rng.random((B, Hd, Tq, N), dtype=np.float32)
    hm = np.array([2, 0, 0, 1], np.int32)
    lens = np.array([203, 150], np.int32)
    idx, cnt, A = oracle.select_indices(P, hm, kb, seq_lens=lens, page=page)
    blk = oracle.block_scores(A, page, lens)
    for b in range(B):
        nbb = (lens[b] + page - 1) // page
        for t, j in enumerate(hm):
            np.testing.assert_array_equal(idx[b, t], brute_select(blk[b, j, :nbb], kb))
    tok, tcnt = oracle.expand_blocks(idx, cnt, page, N)
    for b in range(B):
        for t in range(4):
            row = tok[b, t, :tcnt[b, t]]
            assert (np.diff(row) > 0).all() and row.max() < N
            # every token of a chosen block, and only those (clipped at N)
            want = np.concatenate([np.arange(m * page, min((m + 1) * page, N)) for m in idx[b, t]])
            np.testing.assert_array_equal(row, want)
    # the last block (id 25) holds 3 tokens only
    t2, c2 = oracle.expand_blocks(np.array([[[0, 25]]], np.int32), None, page, N)
    assert c2[0, 0] == 11 and t2[0, 0, :11].tolist() == list(range(8)) + [200, 201, 202]
    # counts cut the block list: only the first counts[b, t] entries stand for tokens, the rest
    # of the row (here a valid-looking block id and the -1 padding) is ignored
    t3, c3 = oracle.expand_blocks(np.array([[[1, 3, 7, -1]]], np.int32), np.array([[2]], np.int32), page, N)
    assert c3[0, 0] == 16 and t3[0, 0, :16].tolist() == list(range(8, 16)) + list(range(24, 32))
    assert (t3[0, 0, 16:] == -1).all()
    t4, c4 = oracle.expand_blocks(np.array([[[5, 6]]], np.int32), np.array([[0]], np.int32), page, N)
    assert c4[0, 0] == 0 and (t4 == -1).all()


def test_block_attention_equals_token_attention_on_expanded_rows():
    g = torch.Generator().manual_seed(3)
    B, Tq, Hq, Hkv, d, N, page = 1, 2, 4, 2, 16, 45, 4
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, N, d, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, N, d, generator=g).to(torch.bfloat16)
    blocks = np.array([[[0, 3, 11], [1, 2, 11], [4, 5, 6], [0, 10, 11]]], np.int32)   # 11 is partial (1 token)
    tok, cnt = oracle.expand_blocks(blocks, None, page, N)
    r = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), 0.25, tok, cnt)
    for t in range(Hq):
        rows = torch.from_numpy(tok[0, t, :cnt[0, t]]).long()
        s = (q[0, :, t].double() @ k[0, t // 2].double()[rows].T) * 0.25
        ref = torch.softmax(s, -1) @ v[0, t // 2].double()[rows]
        np.testing.assert_allclose(r["out"][0, :, t], ref.numpy(), rtol=1e-6, atol=1e-7)
    assert cnt.tolist() == [[9, 9, 12, 9]]


def test_partial_last_block_of_a_ragged_length_is_ranked():
    """A valid length that is no multiple of the page: the last, partial block is a candidate like
    any other (ceil(N_b / page) blocks), and tokens past the length do not count towards it."""
    B, Hd, Tq, N, page = 1, 1, 2, 64, 8
    P = np.full((B, Hd, Tq, N), 0.01, np.float32)
    P[0, 0, :, 42] = 5.0                    # block 5 holds tokens 40..47; the valid length is 43
    P[0, 0, :, 44] = 50.0                   # past the valid length: must not help block 5 ... nor hurt
    lens = np.array([43], np.int32)
    idx, cnt, A = oracle.select_indices(P, np.array([0], np.int32), 1, seq_lens=lens, page=page)
    assert cnt[0, 0] == 1 and idx[0, 0, 0] == 5
    blk = oracle.block_scores(A, page, lens)
    assert blk[0, 0, 5] == np.float32(0.02 + 0.02 + 10.0)        # tokens 40, 41, 42 only
    idx6, cnt6, _ = oracle.select_indices(P, np.array([0], np.int32), 8, seq_lens=lens, page=page)
    assert cnt6[0, 0] == 6 and idx6[0, 0, :6].tolist() == [0, 1, 2, 3, 4, 5] and (idx6[0, 0, 6:] == -1).all()
