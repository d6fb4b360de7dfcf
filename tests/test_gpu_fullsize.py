"""GPU parity at the benchmark's full size and launch configuration (128K context, batch 4,
10% budget): selection is checked bit-exact on whole rows, the sparse attention of the headline
layer on every output, the dense attention on one whole batch element and on sampled (batch,
head) outputs elsewhere."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn, check_logits, oracle_attn
from workload import CONFIGS, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def c3():
    w = make_workload(CONFIGS["c3"], seed=20251127, device=DEV)
    torch.cuda.synchronize()
    return w


def test_c3_select_rows_bit_exact(c3):
    w = c3
    idx, cnt, agg = sts.sts_select(w.scores, w.head_map, w.k_budget, want_agg=True)
    torch.cuda.synchronize()
    assert w.k_budget == 13108
    # whole rows of two batch elements (the oracle sorts 131072 scores per row)
    for b in (0, 3):
        sc = w.scores[b:b + 1].cpu().numpy()
        o_idx, o_cnt, o_agg = oracle.select_indices(sc, w.head_map.numpy(), w.k_budget)
        np.testing.assert_array_equal(agg[b:b + 1].cpu().numpy().view(np.uint32), o_agg.view(np.uint32))
        np.testing.assert_array_equal(idx[b:b + 1].cpu().numpy(), o_idx)
        np.testing.assert_array_equal(cnt[b:b + 1].cpu().numpy(), o_cnt)
    # properties on every row: ascending, in range, equal-mapped heads identical
    i = idx.cpu().numpy()
    assert (np.diff(i, axis=-1) > 0).all() and i.min() >= 0 and i.max() < w.cfg.N
    hm = w.head_map.numpy()
    for t in range(1, len(hm)):
        if hm[t] == hm[t - 1]:
            np.testing.assert_array_equal(i[:, t], i[:, t - 1])


def test_c3_whole_sparse_layer_and_a_dense_batch_element(c3):
    """The headline layer as a whole: the sparse result for every (batch, head, query row) of the
    128K, batch-4, 10% configuration against the oracle, and the dense result for every head of one
    batch element (the oracle needs about 0.2 s for the first and 0.7 s for the second)."""
    w = c3
    idx, cnt, _ = sts.sts_select(w.scores, w.head_map, w.k_budget)
    out, lse = sts.sts_sparse_attn(w.q, w.k, w.v, idx, w.scale, counts=cnt, head_map=w.head_map)
    dout, dlse, _ = sts.sts_dense_attn(w.q, w.k, w.v, w.scale)
    torch.cuda.synchronize()
    ref = oracle_attn(w.q, w.k, w.v, w.scale, idx, cnt)
    check_attn(out, lse, ref, what="c3 sparse, whole layer")
    b = 1
    dref = oracle_attn(w.q[b:b + 1], w.k[b:b + 1], w.v[b:b + 1], w.scale)
    check_attn(dout[b:b + 1], dlse[b:b + 1], dref, what=f"c3 dense, batch element {b}, every head")
    # sampled heads of the other batch elements
    _sample_heads(w, None, None, None, None, [(0, 0), (2, 6), (3, 31)], "c3", dense=(dout, dlse))
    assert torch.isfinite(out.float()).all() and torch.isfinite(dout.float()).all()


@pytest.mark.parametrize("frac,want_k", [(0.05, 6554), (0.20, 26215)])
def test_c3_budget_sweep(c3, frac, want_k):
    """The other two points of the 128K budget sweep: whole selection rows of one batch element
    bit-exact, sparse attention on sampled (batch, head) pairs."""
    from workload import budget_tokens
    w = c3
    kb = budget_tokens(w.cfg, frac)
    assert kb == want_k
    idx, cnt, _ = sts.sts_select(w.scores, w.head_map, kb)
    out, lse = sts.sts_sparse_attn(w.q, w.k, w.v, idx, w.scale, counts=cnt, head_map=w.head_map)
    torch.cuda.synchronize()
    b = 2
    o_idx, o_cnt, _ = oracle.select_indices(w.scores[b:b + 1].cpu().numpy(), w.head_map.numpy(), kb)
    np.testing.assert_array_equal(idx[b:b + 1].cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt[b:b + 1].cpu().numpy(), o_cnt)
    _sample_heads(w, idx, cnt, out, lse, [(0, 7), (3, 20)], f"c3 {frac:.0%}")


def _sample_heads(w, idx, cnt, out, lse, samples, tag, dense=None):
    G = w.cfg.Hq // w.cfg.Hkv
    for b, t in samples:
        g = t // G
        qg = w.q[b:b + 1, :, g * G:(g + 1) * G].contiguous().cpu()
        kb, vb = w.k[b:b + 1, g:g + 1].cpu(), w.v[b:b + 1, g:g + 1].cpu()
        hs = range(t - g * G, t - g * G + 1)
        sl = (slice(0, 1), slice(t - g * G, t - g * G + 1))
        if idx is not None:
            ig = idx[b:b + 1, g * G:(g + 1) * G].cpu().contiguous()
            cg = cnt[b:b + 1, g * G:(g + 1) * G].cpu().contiguous()
            ref = oracle_attn(qg, kb, vb, w.scale, ig, cg, heads=hs)
            check_attn(out[b:b + 1, :, g * G:(g + 1) * G], lse[b:b + 1, g * G:(g + 1) * G], ref, sel=sl,
                       what=f"{tag} sparse b{b} h{t}")
        if dense is not None:
            dref = oracle_attn(qg, kb, vb, w.scale, heads=hs)
            check_attn(dense[0][b:b + 1, :, g * G:(g + 1) * G], dense[1][b:b + 1, g * G:(g + 1) * G], dref,
                       sel=sl, what=f"{tag} dense b{b} h{t}")


def test_c2_whole_configuration():
    """The 32K configuration as a whole (batch 1, 10%: k = 3277): every selection row bit-exact,
    every head of the sparse and the dense attention against the oracle, and the budget sweep
    of the 128K configuration's fractions on the same tensors."""
    from workload import budget_tokens
    w = make_workload(CONFIGS["c2"], seed=2, device=DEV)
    assert w.k_budget == 3277
    for frac in (0.05, 0.10, 0.20):
        kb = budget_tokens(w.cfg, frac)
        idx, cnt, agg = sts.sts_select(w.scores, w.head_map, kb, want_agg=True)
        out, lse = sts.sts_sparse_attn(w.q, w.k, w.v, idx, w.scale, counts=cnt, head_map=w.head_map,
                                       out_dtype=torch.float32)
        torch.cuda.synchronize()
        o_idx, o_cnt, o_agg = oracle.select_indices(w.scores.cpu().numpy(), w.head_map.numpy(), kb)
        np.testing.assert_array_equal(agg.cpu().numpy().view(np.uint32), o_agg.view(np.uint32))
        np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
        np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
        ref = oracle_attn(w.q.cpu(), w.k.cpu(), w.v.cpu(), w.scale, idx.cpu(), cnt.cpu())
        check_attn(out, lse, ref, what=f"c2 sparse {frac:.0%}")
    dout, dlse, _ = sts.sts_dense_attn(w.q, w.k, w.v, w.scale, out_dtype=torch.float32)
    dref = oracle_attn(w.q.cpu(), w.k.cpu(), w.v.cpu(), w.scale, heads=range(0, 8))
    check_attn(dout, dlse, dref, sel=(slice(0, 1), slice(0, 8)), what="c2 dense heads 0-7")


def test_c4_one_layer_of_the_1m_context_configuration():
    """One full layer of the 1M-token configuration (4 GiB of KV): byte offsets beyond 2^32,
    selection bit-exact on whole rows at both budgets, attention on sampled heads."""
    w = make_workload(CONFIGS["c4"], seed=4, device=DEV)
    torch.cuda.synchronize()
    for frac, want_k in ((0.02, 20972), (0.10, 104858)):
        from workload import budget_tokens
        kb = budget_tokens(w.cfg, frac)
        assert kb == want_k
        idx, cnt, agg = sts.sts_select(w.scores, w.head_map, kb, want_agg=True)
        out, lse = sts.sts_sparse_attn(w.q, w.k, w.v, idx, w.scale, counts=cnt, head_map=w.head_map)
        torch.cuda.synchronize()
        o_idx, o_cnt, o_agg = oracle.select_indices(w.scores.cpu().numpy(), w.head_map.numpy(), kb)
        np.testing.assert_array_equal(agg.cpu().numpy().view(np.uint32), o_agg.view(np.uint32))
        np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
        np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
        _sample_heads(w, idx, cnt, out, lse, [(0, 5), (0, 30)], f"c4 {frac:.0%}")
    dout, dlse, _ = sts.sts_dense_attn(w.q, w.k, w.v, w.scale)
    torch.cuda.synchronize()
    _sample_heads(w, None, None, None, None, [(0, 31)], "c4", dense=(dout, dlse))


def test_c5_two_batch_elements_of_the_70b_shaped_chain():
    """The 70B-shaped configuration at full context (128K), two batch elements: draft dense
    attention with logits dump -> selection -> sparse target attention."""
    from dataclasses import replace
    from workload import make_draft_layer

    cfg = replace(CONFIGS["c5"], B=2)
    w = make_workload(cfg, seed=5, device=DEV, with_scores=False)
    dl = make_draft_layer(w)
    kb = w.k_budget
    d_out, d_lse, d_logits = sts.sts_dense_attn(dl["q"], dl["k"], dl["v"], dl["scale"], want_logits=True)
    idx, cnt, agg = sts.sts_select(d_logits, w.head_map, kb, lse=d_lse, kind=sts.STS_SCORES_LOGITS_LSE,
                                   want_agg=True)
    out, lse = sts.sts_sparse_attn(w.q, w.k, w.v, idx, w.scale, counts=cnt, head_map=w.head_map)
    torch.cuda.synchronize()
    # draft logits of one sampled draft head against the oracle (the QK^T dump)
    j, b = 9, 1
    gd = j // (cfg.Hd // cfg.draft_Hkv)
    Gd = cfg.Hd // cfg.draft_Hkv
    ref_d = oracle_attn(dl["q"][b:b + 1, :, gd * Gd:(gd + 1) * Gd].contiguous().cpu(), dl["k"][b:b + 1, gd:gd + 1].cpu(),
                        dl["v"][b:b + 1, gd:gd + 1].cpu(), dl["scale"], want_logits=True,
                        heads=range(j - gd * Gd, j - gd * Gd + 1))
    got = d_logits[b, j].cpu().numpy()
    check_logits(got, ref_d["logits"][0, j - gd * Gd], what="c5 draft logits")
    # selection: bit-exact on the GPU's own aggregate
    a = agg.cpu().numpy()
    sel, c = oracle.select(a, kb)
    o_idx, o_cnt = oracle.remap(sel, c, w.head_map.numpy())
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    o_agg = oracle.aggregate(d_logits[:1, :4].cpu().numpy(), d_lse[:1, :4].cpu().numpy(), kind=oracle.LOGITS_LSE)
    np.testing.assert_allclose(a[:1, :4], o_agg, rtol=1e-5, atol=1e-12)
    _sample_heads(w, idx, cnt, out, lse, [(0, 3), (1, 40), (1, 63)], "c5")
    # the other route: the draft layer sums its attention weights itself (second pass over K)
    # and the selection ranks that tensor in place: same aggregate bit for bit, same index sets;
    # one sampled head against the oracle's aggregate of its own logits
    A = torch.empty(cfg.B, cfg.Hd, cfg.N, dtype=torch.float32, device=DEV)
    sts.sts_dense_attn(dl["q"], dl["k"], dl["v"], dl["scale"], logits_out=d_logits, lse_out=d_lse,
                       weights_sum_out=A)
    assert torch.equal(A, agg)
    idx2, cnt2, _ = sts.sts_select(A.view(cfg.B, cfg.Hd, 1, cfg.N), w.head_map, kb)
    assert torch.equal(idx2, idx) and torch.equal(cnt2, cnt)
    ref_A = oracle.aggregate(ref_d["logits"][:, j - gd * Gd:j - gd * Gd + 1],
                             ref_d["lse"][:, j - gd * Gd:j - gd * Gd + 1], kind=oracle.LOGITS_LSE)[0, 0]
    got_A = A[b, j].cpu().numpy()
    assert (np.abs(got_A - ref_A) <= 3e-5 * ref_A + 1e-10).all()


@pytest.mark.parametrize("B,Hd,Tq,dtype,kind", [
    (8, 32, 8, torch.float32, "logits"),       # the 70B-shaped layer's dump as the benchmark selects from it
    (8, 32, 1, torch.float32, "probs"),        # its summed weights
    (32, 16, 16, torch.bfloat16, "probs"),     # block masks of chunked prefill: 512 rows of 16 bf16 scores per token
])
def test_full_batches_of_128k_rows_take_the_one_pass_selection(B, Hd, Tq, dtype, kind):
    """The shapes the benchmark times with at least a row per compute unit, at their full sizes
    and under the library's own routing: one workgroup per row, one pass. Whole rows, sampled over
    the batch, bit for bit against the oracle (scaled-logit input: stage-wise, the oracle ranks
    the GPU's own aggregate of the row and checks that aggregate to rounding)."""
    N, k = 131072, 13108
    g = torch.Generator(device=DEV)
    g.manual_seed(B * Tq)
    scores = torch.empty(B, Hd, Tq, N, dtype=dtype, device=DEV)
    lse = torch.empty(B, Hd, Tq, dtype=torch.float32, device=DEV) if kind == "logits" else None
    lens = torch.full((B,), N, dtype=torch.int32, device=DEV)
    lens[B - 1] = N - 4097
    for b in range(B):
        lg = torch.randn(Hd, Tq, N, generator=g, device=DEV) * 2
        lg[:, :, int(lens[b]):] = float("-inf") if kind == "probs" else 0.0
        if kind == "logits":
            scores[b] = lg
            lse[b] = torch.logsumexp(lg[:, :, :int(lens[b])], dim=-1)
        else:
            scores[b] = torch.softmax(lg, dim=-1).to(dtype)
        del lg
    hm = list(range(Hd))
    sts.prof_enable(True)
    sts.prof_reset()
    try:
        idx, cnt, agg = sts.sts_select(scores, hm, k, lse=lse, seq_lens=lens, want_agg=(kind == "logits"),
                                       kind=sts.STS_SCORES_LOGITS_LSE if kind == "logits" else sts.STS_SCORES_PROBS)
        torch.cuda.synchronize()
        kinds = {name for name, (n, _) in sts.prof_read().items() if n}
    finally:
        sts.prof_enable(False)
    assert kinds == {"select_band"}
    assert (cnt.cpu().numpy() == np.minimum(k, lens.cpu().numpy())[:, None]).all()
    for b, j in [(0, 0), (B // 2, Hd - 1), (B - 1, Hd // 2)]:
        ln = lens[b:b + 1].cpu().numpy()
        if kind == "logits":
            a = agg[b:b + 1, j:j + 1].cpu().numpy()
            o_agg = oracle.aggregate(scores[b:b + 1, j:j + 1].cpu().numpy(), lse[b:b + 1, j:j + 1].cpu().numpy(),
                                     kind=oracle.LOGITS_LSE)
            n = int(ln[0])
            np.testing.assert_allclose(a[..., :n], o_agg[..., :n], rtol=1e-5, atol=1e-12)
            sel, c = oracle.select_per_head(a, k, [k], ln)
        else:
            o_idx, o_cnt, _ = oracle.select_indices(scores[b:b + 1, j:j + 1].float().cpu().numpy(), np.zeros(1, np.int32), k,
                                                    seq_lens=ln)
            sel, c = o_idx, o_cnt
        np.testing.assert_array_equal(cnt[b, j].cpu().numpy(), np.asarray(c).reshape(-1)[0])
        np.testing.assert_array_equal(idx[b, j].cpu().numpy(), np.asarray(sel).reshape(-1, k)[0])


def test_summed_weights_at_a_million_tokens():
    """The second pass over K on a 1M-token draft cache (32768 key tiles, 64-bit row offsets):
    bit for bit the aggregate of the dump, zero past the valid length, same index sets."""
    B, Tq, Hq, Hkv, d, N = 1, 5, 16, 4, 64, 1 << 20
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    q = torch.randn(B, Tq, Hq, d, generator=g, device=DEV).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g, device=DEV) * 0.5).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g, device=DEV) * 0.5).to(torch.bfloat16)
    lens = torch.tensor([N - 12345], dtype=torch.int32, device=DEV)
    A = torch.full((B, Hq, N), 7.0, device=DEV)
    _, lse, logits = sts.sts_dense_attn(q, k, v, 0.125, seq_lens=lens, want_logits=True, weights_sum_out=A)
    hm, kk, n = list(range(Hq)), 50000, int(lens[0])
    idx_d, cnt_d, agg_d = sts.sts_select(logits, hm, kk, lse=lse, seq_lens=lens, kind=sts.STS_SCORES_LOGITS_LSE,
                                         want_agg=True)
    idx_a, cnt_a, _ = sts.sts_select(A.view(B, Hq, 1, N), hm, kk, seq_lens=lens)
    assert torch.equal(A[0, :, :n], agg_d[0, :, :n]) and (A[0, :, n:] == 0).all()
    assert torch.equal(idx_a, idx_d) and torch.equal(cnt_a, cnt_d)
    assert torch.allclose(A[0, :, :n].double().sum(-1), torch.full((Hq,), float(Tq), dtype=torch.float64, device=DEV),
                          atol=1e-4)
