"""Pins for the attention half of the oracle (sparse = softmax restricted to an index set).

Section 2.3 / 4.2 of the paper define the result (attention over a selected subset of a
full, kept cache); no numbers are printed. Pins: mask-restricted full softmax by brute
force, budget == N equals dense bit for bit, closed forms, invariants, split/merge
invariance (the definition of the combine step) and torch's scaled_dot_product_attention.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def rand_case(seed, B=2, Tq=3, Hq=4, Hkv=2, d=16, N=37, kv_std=0.5):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * kv_std).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * kv_std).to(torch.bfloat16)
    return q, k, v


def rand_indices(seed, B, Hq, N, kk):
    rng = np.random.default_rng(seed)
    idx = np.stack([[np.sort(rng.choice(N, kk, replace=False)) for _ in range(Hq)] for _ in range(B)])
    return idx.astype(np.int32)


def masked_softmax_ref(q, k, v, scale, idx, counts=None):
    """Full softmax over all N positions with -inf on positions not in the index set (fp64)."""
    B, Tq, Hq, d = q.shape
    Hkv, N = k.shape[1], k.shape[2]
    G = Hq // Hkv
    qf, kf, vf = q.double(), k.double(), v.double()
    out = torch.zeros(B, Tq, Hq, d, dtype=torch.float64)
    lse = torch.zeros(B, Hq, Tq, dtype=torch.float64)
    for b in range(B):
        for t in range(Hq):
            c = idx.shape[2] if counts is None else int(counts[b, t])
            mask = torch.full((N,), -math.inf, dtype=torch.float64)
            mask[torch.from_numpy(idx[b, t, :c]).long()] = 0.0
            s = (qf[b, :, t, :] @ kf[b, t // G].T) * scale + mask          # [Tq,N]
            p = torch.softmax(s, dim=-1)
            out[b, :, t, :] = p @ vf[b, t // G]
            lse[b, t] = torch.logsumexp(s, dim=-1)
    return out.numpy(), lse.numpy()


@pytest.mark.parametrize("seed", range(4))
def test_sparse_equals_mask_restricted_full_softmax(seed):
    q, k, v = rand_case(seed)
    B, Tq, Hq, d = q.shape
    N = k.shape[2]
    idx = rand_indices(seed, B, Hq, N, 11)
    scale = 1.0 / math.sqrt(d)
    r = oracle.attn(oracle.bf16_bits(q), oracle.bf16_bits(k), oracle.bf16_bits(v), scale, idx)
    ref_o, ref_l = masked_softmax_ref(q, k, v, scale, idx)
    np.testing.assert_allclose(r["out"], ref_o, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(r["lse"], ref_l, rtol=1e-6, atol=1e-6)


def test_full_budget_equals_dense_bitwise_and_sdpa():
    q, k, v = rand_case(11, N=53)
    B, Tq, Hq, d = q.shape
    Hkv, N = k.shape[1], k.shape[2]
    scale = 0.2
    idx = np.broadcast_to(np.arange(N, dtype=np.int32), (B, Hq, N)).copy()
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    sp = oracle.attn(qb, kb, vb, scale, idx)
    de = oracle.attn(qb, kb, vb, scale, want_logits=True)
    np.testing.assert_array_equal(sp["out"], de["out"])
    np.testing.assert_array_equal(sp["lse"], de["lse"])
    # library cross-check: torch SDPA in fp32 with K/V repeated over the GQA group
    G = Hq // Hkv
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.float().permute(0, 2, 1, 3), k.float().repeat_interleave(G, 1),
        v.float().repeat_interleave(G, 1), scale=scale).permute(0, 2, 1, 3)
    np.testing.assert_allclose(de["out"], ref.numpy(), rtol=2e-5, atol=2e-6)
    # the dumped logits are the pre-softmax scaled products
    lg = torch.einsum("bihe,bhne->bhin", q.double(), k.double().repeat_interleave(G, 1)) * scale
    np.testing.assert_allclose(de["logits"], lg.numpy(), rtol=1e-6, atol=1e-7)


def test_sdpa_with_boolean_mask():
    q, k, v = rand_case(12, B=1, Tq=2, Hq=4, Hkv=2, d=32, N=64)
    idx = rand_indices(12, 1, 4, 64, 9)
    scale = 1.0 / math.sqrt(32)
    r = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), scale, idx)
    mask = torch.zeros(1, 4, 1, 64, dtype=torch.bool)
    for t in range(4):
        mask[0, t, 0, torch.from_numpy(idx[0, t]).long()] = True
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.float().permute(0, 2, 1, 3), k.float().repeat_interleave(2, 1),
        v.float().repeat_interleave(2, 1), attn_mask=mask, scale=scale).permute(0, 2, 1, 3)
    np.testing.assert_allclose(r["out"], ref.numpy(), rtol=2e-5, atol=2e-6)


def test_gqa_head_uses_its_group_kv():
    # two KV heads with constant, different V: every query head must return its group's constant
    B, Tq, Hq, Hkv, d, N = 1, 2, 6, 2, 8, 10
    q, k, _ = rand_case(13, B, Tq, Hq, Hkv, d, N)
    v = torch.zeros(B, Hkv, N, d)
    v[:, 0] = 1.5
    v[:, 1] = -2.0
    v = v.to(torch.bfloat16)
    r = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), 0.3)
    np.testing.assert_allclose(r["out"][:, :, :3], 1.5, rtol=1e-6)
    np.testing.assert_allclose(r["out"][:, :, 3:], -2.0, rtol=1e-6)


def test_zero_query_gives_mean_of_selected_values_and_log_count():
    q, k, v = rand_case(14)
    q = torch.zeros_like(q)
    B, Tq, Hq, d = q.shape
    idx = rand_indices(14, B, Hq, k.shape[2], 7)
    r = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), 0.7, idx)
    G = Hq // k.shape[1]
    for b in range(B):
        for t in range(Hq):
            mean = v[b, t // G].double()[torch.from_numpy(idx[b, t]).long()].mean(0).numpy()
            for i in range(Tq):
                np.testing.assert_allclose(r["out"][b, i, t], mean, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(r["lse"], math.log(7), rtol=1e-6)


def test_dominant_key_returns_its_value_row():
    q, k, v = rand_case(15, B=1, Tq=1, Hq=2, Hkv=1, d=8, N=20)
    q = torch.ones_like(q)
    k = torch.zeros_like(k)
    k[0, 0, 13] = 64.0       # logit 8*64*scale far above the zeros
    idx = np.array([[[2, 13, 17], [13, 14, 15]]], np.int32)
    r = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), 1.0, idx)
    np.testing.assert_allclose(r["out"][0, 0, 0], v[0, 0, 13].float().numpy(), rtol=1e-6, atol=1e-30)
    np.testing.assert_allclose(r["out"][0, 0, 1], v[0, 0, 13].float().numpy(), rtol=1e-6, atol=1e-30)
    np.testing.assert_allclose(r["lse"], 512.0, rtol=1e-6)


def test_output_bounded_by_selected_values_and_permutation_invariant():
    q, k, v = rand_case(16)
    B, Tq, Hq, d = q.shape
    N = k.shape[2]
    idx = rand_indices(16, B, Hq, N, 9)
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    r = oracle.attn(qb, kb, vb, 0.25, idx)
    G = Hq // k.shape[1]
    for b in range(B):
        for t in range(Hq):
            rows = v[b, t // G].float()[torch.from_numpy(idx[b, t]).long()].numpy()
            assert (r["out"][b, :, t] <= rows.max(0) + 1e-6).all()
            assert (r["out"][b, :, t] >= rows.min(0) - 1e-6).all()
    rng = np.random.default_rng(0)
    shuffled = np.take_along_axis(idx, rng.permuted(np.tile(np.arange(9), (B, Hq, 1)), axis=-1), -1)
    r2 = oracle.attn(qb, kb, vb, 0.25, shuffled)
    np.testing.assert_allclose(r2["out"], r["out"], rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(r2["lse"], r["lse"], rtol=1e-6, atol=1e-7)


def test_split_merge_invariance():
    """Attention over two halves merged with log-sum-exp weights equals attention over the
    whole index set: the definition the split/combine kernels implement (split-K, Section 5)."""
    q, k, v = rand_case(17, N=64)
    B, Tq, Hq, d = q.shape
    idx = rand_indices(17, B, Hq, 64, 20)
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    whole = oracle.attn(qb, kb, vb, 0.3, idx)
    a = oracle.attn(qb, kb, vb, 0.3, np.ascontiguousarray(idx[:, :, :8]))
    b = oracle.attn(qb, kb, vb, 0.3, np.ascontiguousarray(idx[:, :, 8:]))
    la, lb = a["lse"].astype(np.float64), b["lse"].astype(np.float64)
    lw = np.logaddexp(la, lb)
    wa = np.exp(la - lw).transpose(0, 2, 1)[..., None]
    wb = np.exp(lb - lw).transpose(0, 2, 1)[..., None]
    np.testing.assert_allclose(wa * a["out"] + wb * b["out"], whole["out"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(lw, whole["lse"], rtol=1e-6, atol=1e-6)


def test_counts_seq_lens_strides_and_empty_rows():
    q, k, v = rand_case(18, B=2, N=30)
    B, Tq, Hq, d = q.shape
    idx = rand_indices(18, B, Hq, 30, 12)
    counts = np.array([[12, 5, 0, 1], [3, 12, 7, 0]], np.int32)
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    r = oracle.attn(qb, kb, vb, 0.3, idx, counts)
    ref_o, ref_l = masked_softmax_ref(q, k, v, 0.3, idx, counts)
    for b in range(B):
        for t in range(Hq):
            if counts[b, t] == 0:
                assert (r["out"][b, :, t] == 0).all() and np.isneginf(r["lse"][b, t]).all()
            else:
                np.testing.assert_allclose(r["out"][b, :, t], ref_o[b, :, t], rtol=1e-6, atol=1e-7)
                np.testing.assert_allclose(r["lse"][b, t], ref_l[b, t], rtol=1e-6, atol=1e-6)
    # dense with seq_lens equals dense on the truncated cache
    lens = np.array([30, 17], np.int32)
    de = oracle.attn(qb, kb, vb, 0.3, seq_lens=lens)
    tr = oracle.attn(qb[1:], np.ascontiguousarray(kb[1:, :, :17]), np.ascontiguousarray(vb[1:, :, :17]), 0.3)
    np.testing.assert_array_equal(de["out"][1], tr["out"][0])
    # a strided (interleaved K/V) cache gives the same result as a packed one
    kv = torch.stack([k, v], dim=3)                  # [B,Hkv,N,2,d]
    ks, vs = kv[:, :, :, 0], kv[:, :, :, 1]
    rs = oracle.attn(qb, oracle.bf16_bits(ks), oracle.bf16_bits(vs), 0.3, idx, counts)
    np.testing.assert_array_equal(rs["out"], r["out"])
    # out-of-range index is an error
    bad = idx.copy()
    bad[0, 0, 0] = 30
    with pytest.raises(ValueError):
        oracle.attn(qb, kb, vb, 0.3, bad)


def test_logit_shift_changes_only_lse():
    # adding c*q/|q|^2-aligned constant is awkward; scale the scores by using duplicated keys:
    # duplicating every selected index doubles l and leaves out unchanged (each occurrence counted)
    q, k, v = rand_case(19)
    B, Tq, Hq, d = q.shape
    idx = rand_indices(19, B, Hq, k.shape[2], 6)
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    r1 = oracle.attn(qb, kb, vb, 0.3, idx)
    r2 = oracle.attn(qb, kb, vb, 0.3, np.concatenate([idx, idx], -1))
    np.testing.assert_allclose(r2["out"], r1["out"], rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(r2["lse"], r1["lse"] + math.log(2), rtol=1e-6, atol=1e-6)


def test_sampling_ranges_touch_only_requested_heads():
    q, k, v = rand_case(20)
    qb, kb, vb = map(oracle.bf16_bits, (q, k, v))
    full = oracle.attn(qb, kb, vb, 0.3)
    part = oracle.attn(qb, kb, vb, 0.3, batches=range(1, 2), heads=range(1, 3))
    np.testing.assert_array_equal(part["out"][1, :, 1:3], full["out"][1, :, 1:3])
    assert (part["out"][0] == 0).all() and (part["out"][1, :, 0] == 0).all()


# ---------------------------------------------------------- the block's own causal keys


def _tail_case(seed, B=2, Tq=4, Hq=4, Hkv=2, d=16, N=29):
    q, k, v = rand_case(seed, B, Tq, Hq, Hkv, d, N)
    g = torch.Generator().manual_seed(seed + 100)
    kn = torch.randn(B, Tq, Hkv, d, generator=g).to(torch.bfloat16)
    vn = torch.randn(B, Tq, Hkv, d, generator=g).to(torch.bfloat16)
    return q, k, v, kn, vn


@pytest.mark.parametrize("causal", [True, False])
def test_block_tail_matches_sdpa_on_the_concatenated_cache(causal):
    """Verification attends to the cached prefix (restricted to the index set) plus the
    speculative block's own tokens, candidate i seeing candidates 0..i (Section 2.1: all
    candidates are verified in one parallel step). Pin: torch SDPA over [K; K_new] with the
    explicit boolean mask."""
    q, k, v, kn, vn = _tail_case(31)
    B, Tq, Hq, d = q.shape
    Hkv, N = k.shape[1], k.shape[2]
    G = Hq // Hkv
    idx = rand_indices(31, B, Hq, N, 7)
    r = oracle.attn(*map(oracle.bf16_bits, (q, k, v)), 0.3, idx,
                    k_new=oracle.bf16_bits(kn), v_new=oracle.bf16_bits(vn), causal=causal)
    kc = torch.cat([k, kn.permute(0, 2, 1, 3)], dim=2).float().repeat_interleave(G, 1)   # [B,Hq,N+Tq,d]
    vc = torch.cat([v, vn.permute(0, 2, 1, 3)], dim=2).float().repeat_interleave(G, 1)
    mask = torch.zeros(B, Hq, Tq, N + Tq, dtype=torch.bool)
    for b in range(B):
        for t in range(Hq):
            mask[b, t, :, torch.from_numpy(idx[b, t]).long()] = True
    for i in range(Tq):
        mask[:, :, i, N:N + (i + 1 if causal else Tq)] = True
    ref = torch.nn.functional.scaled_dot_product_attention(q.float().permute(0, 2, 1, 3), kc, vc,
                                                           attn_mask=mask, scale=0.3).permute(0, 2, 1, 3)
    np.testing.assert_allclose(r["out"], ref.numpy(), rtol=2e-5, atol=2e-6)


def test_block_tail_non_causal_equals_dense_over_longer_cache_and_empty_prefix():
    q, k, v, kn, vn = _tail_case(32)
    B, Tq, Hq, d = q.shape
    N = k.shape[2]
    qb, kb, vb, knb, vnb = map(oracle.bf16_bits, (q, k, v, kn, vn))
    r = oracle.attn(qb, kb, vb, 0.3, k_new=knb, v_new=vnb, causal=False)
    kc = torch.cat([k, kn.permute(0, 2, 1, 3)], dim=2).contiguous()
    vc = torch.cat([v, vn.permute(0, 2, 1, 3)], dim=2).contiguous()
    d2 = oracle.attn(qb, oracle.bf16_bits(kc), oracle.bf16_bits(vc), 0.3)
    np.testing.assert_allclose(r["out"], d2["out"], rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(r["lse"], d2["lse"], rtol=1e-6, atol=1e-6)
    # empty index rows: candidate 0 sees only itself -> its own value row and its own logit
    idx = np.zeros((B, Hq, 1), np.int32)
    cnt = np.zeros((B, Hq), np.int32)
    e = oracle.attn(qb, kb, vb, 0.3, idx, cnt, k_new=knb, v_new=vnb, causal=True)
    G = Hq // k.shape[1]
    for t in range(Hq):
        np.testing.assert_allclose(e["out"][:, 0, t], vn[:, 0, t // G].float().numpy(), rtol=1e-6, atol=1e-30)
        s00 = 0.3 * (q[:, 0, t].double() * kn[:, 0, t // G].double()).sum(-1)
        np.testing.assert_allclose(e["lse"][:, t, 0], s00.numpy(), rtol=1e-6, atol=1e-6)
