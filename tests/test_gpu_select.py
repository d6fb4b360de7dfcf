"""GPU parity: sts_select (through the C ABI) against the CPU oracle. Index sets, counts and
the aggregated scores must match bit for bit on identical score tensors."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import stored_agg
from workload import CONFIGS, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True, params=[0, 2, 3, 5],
                ids=["auto", "pipeline-or-pool", "one-launch-wherever-possible", "one-workgroup-per-row-wherever-possible"])
def select_path(request):
    """Every case runs several times: under the library's own routing (long rows take the
    one-launch selection), with that path switched off, so that the histogram pipeline and the
    chunk-local top-k + pool, which the same shapes took before and block-granular calls still
    take, stay covered, and with every call whose shape allows it ranked by one workgroup per row
    in one pass (which the library's rule takes only from one row per second compute unit on)."""
    sts.set_knob("select_path", request.param)
    yield request.param
    sts.set_knob("select_path", None)


def run_both(scores, head_map, k, lse=None, seq_lens=None, kind=0, reduce=0):
    sd = scores.to(DEV)
    idx, cnt, agg = sts.sts_select(sd, head_map, k, lse=None if lse is None else lse.to(DEV),
                                   seq_lens=None if seq_lens is None else seq_lens.to(DEV),
                                   kind=kind, reduce=reduce, want_agg=True)
    torch.cuda.synchronize()
    o_idx, o_cnt, o_agg = oracle.select_indices(
        scores.numpy(), np.asarray(head_map, np.int32), k, lse=None if lse is None else lse.numpy(),
        kind=kind, reduce=reduce, seq_lens=None if seq_lens is None else seq_lens.numpy())
    return (idx.cpu().numpy(), cnt.cpu().numpy(), agg.cpu().numpy()), (o_idx, o_cnt, stored_agg(o_agg, seq_lens))


def run_both_budgets(scores, head_map, k, k_head, seq_lens=None, page=1):
    idx, cnt, _ = sts.sts_select(scores.to(DEV), head_map, k, k_head=k_head, page_size=page,
                                 seq_lens=None if seq_lens is None else seq_lens.to(DEV))
    torch.cuda.synchronize()
    o_idx, o_cnt, _ = oracle.select_indices(scores.numpy(), np.asarray(head_map, np.int32), k, k_head=k_head,
                                            page=page, seq_lens=None if seq_lens is None else seq_lens.numpy())
    return (idx.cpu().numpy(), cnt.cpu().numpy()), (o_idx, o_cnt)


def softmax_scores(seed, B, Hd, Tq, N, temp=2.0):
    g = torch.Generator().manual_seed(seed)
    return torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * temp, dim=-1)


@pytest.mark.parametrize("B,Hd,Tq,N,Hq,k", [
    (1, 16, 5, 4096, 32, 410),        # the 4K configuration's shape
    (2, 3, 5, 20000, 6, 2000),        # several chunks per row, ragged last chunk (pool path)
    (1, 2, 1, 8192, 4, 1),            # single query row, k = 1
    (2, 4, 8, 1001, 8, 100),          # N % 4 != 0: scalar path
    (1, 2, 5, 50, 2, 50),             # k = N
    (1, 2, 5, 50, 3, 80),             # k > N: tail padded with -1
    (1, 1, 64, 300, 1, 7),            # many query rows
    # rows longer than 32768 tokens take the multi-workgroup path (global histograms)
    (2, 3, 5, 40000, 6, 4000),
    (1, 2, 3, 70001, 4, 123),         # and its scalar variant (N % 4 != 0)
    (1, 4, 5, 8192, 8, 819),          # the longest row that always takes the single-workgroup path
    (1, 2, 5, 8196, 4, 819),          # the shortest that does not (few rows): chunk-local top-k + pool
    (16, 16, 2, 20000, 16, 500),      # 256 rows: the single-workgroup path up to its LDS limit
    (16, 16, 1, 32768, 16, 77),
])
def test_select_bit_exact_random(B, Hd, Tq, N, Hq, k):
    scores = softmax_scores(1, B, Hd, Tq, N)
    hm = [(t * Hd) // Hq for t in range(Hq)]
    (idx, cnt, agg), (o_idx, o_cnt, o_agg) = run_both(scores, hm, k)
    np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    np.testing.assert_array_equal(cnt, o_cnt)
    np.testing.assert_array_equal(idx, o_idx)


@pytest.mark.parametrize("levels", [1, 2, 4, 37])
def test_select_heavy_ties(levels):
    g = torch.Generator().manual_seed(levels)
    B, Hd, Tq, Hq = 2, 4, 3, 8
    hm = [3, 3, 0, 1, 2, 2, 0, 1]
    for N, k in ((30000, 1), (30000, 999), (30000, 8192), (30000, 29999), (50000, 7777), (50000, 49999)):
        scores = torch.randint(0, levels, (B, Hd, Tq, N), generator=g).float() / 8.0
        (idx, cnt, _), (o_idx, o_cnt, _) = run_both(scores, hm, k)
        np.testing.assert_array_equal(idx, o_idx)
        np.testing.assert_array_equal(cnt, o_cnt)


def test_select_without_agg_output_matches_with():
    # the single-workgroup path keeps the aggregate in LDS unless it is asked for
    scores = softmax_scores(21, 2, 3, 5, 9000).to(DEV)
    hm = [0, 1, 2, 2]
    a_idx, a_cnt, _ = sts.sts_select(scores, hm, 700, want_agg=False)
    b_idx, b_cnt, _ = sts.sts_select(scores, hm, 700, want_agg=True)
    assert torch.equal(a_idx, b_idx) and torch.equal(a_cnt, b_cnt)


def test_select_signed_zero_negative_denormal_inf():
    N = 5000
    g = torch.Generator().manual_seed(5)
    base = torch.randn(1, 2, 1, N, generator=g)
    base[0, 0, 0, ::7] = 0.0
    base[0, 0, 0, 3::7] = -0.0
    base[0, 0, 0, 5::11] = 1e-42
    base[0, 0, 0, 6::13] = -1e-42
    base[0, 1, 0, 100] = float("inf")
    base[0, 1, 0, 200] = float("-inf")
    for k in (1, 700, 2500, 4999):
        (idx, _, agg), (o_idx, _, o_agg) = run_both(base, [0, 1], k)
        np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
        np.testing.assert_array_equal(idx, o_idx)


def test_select_seq_lens_and_unmapped_draft_heads():
    B, Hd, Tq, N, Hq, k = 3, 4, 5, 9000, 5, 600
    scores = softmax_scores(6, B, Hd, Tq, N)
    lens = torch.tensor([9000, 333, 0], dtype=torch.int32)
    hm = [0, 0, 3, 3, 0]                      # draft heads 1 and 2 feed nobody
    (idx, cnt, _), (o_idx, o_cnt, _) = run_both(scores, hm, k, seq_lens=lens)
    np.testing.assert_array_equal(cnt, o_cnt)
    np.testing.assert_array_equal(idx, o_idx)
    assert (idx[2] == -1).all() and (cnt[1] == 333).all()


def test_select_max_reduction():
    scores = softmax_scores(7, 1, 4, 5, 6000)
    hm = [0, 1, 2, 3]
    (idx, _, agg), (o_idx, _, o_agg) = run_both(scores, hm, 512, reduce=sts.STS_REDUCE_MAX)
    np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    np.testing.assert_array_equal(idx, o_idx)


def test_select_logits_lse_stagewise():
    """expf differs between libm and the device, so the aggregate is compared within a
    relative tolerance and the selection is then checked bit-exact on the GPU's own
    aggregate fed to the oracle (identical score tensors on both sides)."""
    g = torch.Generator().manual_seed(8)
    B, Hd, Tq, N, Hq, k = 2, 4, 5, 12000, 8, 1200
    logits = torch.randn(B, Hd, Tq, N, generator=g) * 2.0
    lse = torch.logsumexp(logits.double(), dim=-1).float()
    hm = [t // 2 for t in range(Hq)]
    (idx, cnt, agg), (_, _, o_agg) = run_both(logits, hm, k, lse=lse, kind=sts.STS_SCORES_LOGITS_LSE)
    np.testing.assert_allclose(agg, o_agg, rtol=1e-5, atol=1e-12)
    sel, c = oracle.select(agg, k)
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
    np.testing.assert_array_equal(idx, o_idx)
    np.testing.assert_array_equal(cnt, o_cnt)


def test_select_then_sparse_attention_on_the_4k_configuration():
    """The whole path on the small configuration: planted workload, selection bit-exact,
    sparse attention within tolerance, everything against the oracle."""
    from gpu_util import check_attn, check_logits, oracle_attn

    w = make_workload(CONFIGS["c1"], seed=20251127)
    q, k, v, scores = w.q.to(DEV), w.k.to(DEV), w.v.to(DEV), w.scores.to(DEV)
    idx, cnt, _ = sts.sts_select(scores, w.head_map, w.k_budget)
    out, lse = sts.sts_sparse_attn(q, k, v, idx, w.scale, counts=cnt, head_map=w.head_map,
                                   out_dtype=torch.float32)
    torch.cuda.synchronize()
    o_idx, o_cnt, _ = oracle.select_indices(w.scores.numpy(), w.head_map.numpy(), w.k_budget)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    assert w.k_budget == 410 and (o_cnt == 410).all()
    ref = oracle_attn(q, k, v, w.scale, torch.from_numpy(o_idx), torch.from_numpy(o_cnt))
    check_attn(out, lse, ref, what="c1 chain")
    # planted sink / recent positions are kept far more often than the 10% base rate
    planted = np.concatenate([np.arange(4), np.arange(4096 - 64, 4096)])
    assert min(np.isin(planted, o_idx[0, t]).mean() for t in range(32)) > 0.4


def test_draft_attention_to_selection_to_sparse_attention_chain():
    """70B-shaped chain at a small context: the draft layer's dense attention dumps scaled
    logits and LSE, selection consumes them (LOGITS_LSE), the target attends sparsely.
    Checked stage by stage against the oracle."""
    from dataclasses import replace

    from gpu_util import check_attn, check_logits, oracle_attn
    from workload import make_draft_layer

    cfg = replace(CONFIGS["c5"], B=2, N=3000)
    w = make_workload(cfg, seed=11, with_scores=False)
    dl = make_draft_layer(w)
    q, k, v = w.q.to(DEV), w.k.to(DEV), w.v.to(DEV)
    qd, kd, vd = dl["q"].to(DEV), dl["k"].to(DEV), dl["v"].to(DEV)
    kb = w.k_budget
    # stage a0: draft dense attention with logits + LSE
    d_out, d_lse, d_logits = sts.sts_dense_attn(qd, kd, vd, dl["scale"], want_logits=True, out_dtype=torch.float32)
    ref_d = oracle_attn(qd, kd, vd, dl["scale"], want_logits=True)
    check_attn(d_out, d_lse, ref_d, what="draft dense")
    check_logits(d_logits.cpu().numpy(), ref_d["logits"], what="draft logits")
    # stage a1-a3 on the GPU's own logits (identical score tensors on both sides)
    idx, cnt, agg = sts.sts_select(d_logits, w.head_map, kb, lse=d_lse, kind=sts.STS_SCORES_LOGITS_LSE,
                                   want_agg=True)
    torch.cuda.synchronize()
    o_agg = oracle.aggregate(d_logits.cpu().numpy(), d_lse.cpu().numpy(), kind=oracle.LOGITS_LSE)
    np.testing.assert_allclose(agg.cpu().numpy(), o_agg, rtol=1e-5, atol=1e-12)
    sel, c = oracle.select(agg.cpu().numpy(), kb)
    o_idx, o_cnt = oracle.remap(sel, c, w.head_map.numpy())
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    # stage a4-a5
    out, lse = sts.sts_sparse_attn(q, k, v, idx, w.scale, counts=cnt, head_map=w.head_map,
                                   out_dtype=torch.float32)
    ref = oracle_attn(q, k, v, w.scale, idx, cnt)
    check_attn(out, lse, ref, what="c5 chain sparse")
    # the draft's selection captures more of the target's attention mass than a random set
    dense = oracle_attn(q, k, v, w.scale)
    mass = np.exp(ref["lse"].astype(np.float64) - dense["lse"].astype(np.float64))
    assert mass.mean() > 1.1 * kb / cfg.N


def test_select_maximum_head_counts():
    g = torch.Generator().manual_seed(31)
    B, Hd, Hq, Tq, N, k = 1, 256, 256, 2, 3000, 300
    scores = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1)
    hm = torch.randint(0, Hd, (Hq,), generator=g).tolist()
    (idx, cnt, agg), (o_idx, o_cnt, o_agg) = run_both(scores, hm, k)
    np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    np.testing.assert_array_equal(idx, o_idx)
    np.testing.assert_array_equal(cnt, o_cnt)
    # more heads than the tables carry is refused, not truncated
    with pytest.raises(sts.StsError):
        sts.sts_select(torch.zeros(1, 257, 1, 64, device=DEV), list(range(257)), 4)


@pytest.mark.parametrize("B,Hd,Tq,N,Hq,k,page", [
    (2, 4, 5, 4096, 8, 410, 1),        # single-workgroup path
    (2, 4, 5, 50000, 8, 5000, 1),      # multi-workgroup path, ragged last chunk
    (1, 3, 2, 70001, 6, 900, 1),       # scalar variant
    (2, 4, 5, 65536, 8, 512, 8),       # block granularity: budgets count blocks
])
def test_select_per_head_budgets(B, Hd, Tq, N, Hq, k, page):
    """Section 6.4: budgets differ per layer (the k of the call) and, here, per draft head."""
    scores = softmax_scores(21, B, Hd, Tq, N)
    hm = [(t * Hd) // Hq for t in range(Hq)]
    rng = np.random.default_rng(5)
    kh = [int(x) for x in rng.integers(1, k + 1, Hd)]
    kh[0], kh[-1] = k, 1                                  # both ends of the allowed range
    lens = torch.tensor([N] + [max(1, N // 3)] * (B - 1), dtype=torch.int32)
    (idx, cnt), (o_idx, o_cnt) = run_both_budgets(scores, hm, k, kh, seq_lens=lens, page=page)
    np.testing.assert_array_equal(cnt, o_cnt)
    np.testing.assert_array_equal(idx, o_idx)
    # equal budgets are the same as none
    (idx2, cnt2), _ = run_both_budgets(scores, hm, k, [k] * Hd, seq_lens=lens, page=page)
    ref, rcnt, _ = sts.sts_select(scores.to(DEV), hm, k, seq_lens=lens.to(DEV), page_size=page)
    np.testing.assert_array_equal(idx2, ref.cpu().numpy())
    np.testing.assert_array_equal(cnt2, rcnt.cpu().numpy())


def test_per_head_budgets_feed_sparse_attention():
    """Lists of different lengths in one call: counts carry each head's own length."""
    cfg = replace(CONFIGS["c1"], N=6000)
    w = make_workload(cfg, seed=9)
    k = w.k_budget
    kh = [max(1, (k * (j + 1)) // w.scores.shape[1]) for j in range(w.scores.shape[1])]
    idx, cnt, _ = sts.sts_select(w.scores.to(DEV), w.head_map, k, k_head=kh)
    out, lse = sts.sts_sparse_attn(w.q.to(DEV), w.k.to(DEV), w.v.to(DEV), idx, w.scale, counts=cnt,
                                   head_map=w.head_map, out_dtype=torch.float32)
    torch.cuda.synchronize()
    o_idx, o_cnt, _ = oracle.select_indices(w.scores.numpy(), np.asarray(w.head_map, np.int32), k, k_head=kh)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    ref = oracle.attn(oracle.bf16_bits(w.q), oracle.bf16_bits(w.k), oracle.bf16_bits(w.v), w.scale,
                      indices=o_idx, counts=o_cnt)
    from gpu_util import check_attn
    check_attn(out, lse, ref, what="per-head budgets")


@pytest.mark.parametrize("spin_limit", ["0", "3"])
def test_lookback_recount_path(spin_limit):
    """Workgroups that read what other workgroups of their row publish (the parts' histograms in
    the one-launch selection) wait a bounded number of polls; what does not show up is recomputed
    by the waiting workgroup. A tiny limit (set from the host) forces that path; the result must
    not change."""
    sts.set_knob("select_spin_limit", int(spin_limit))
    try:
        _lookback_cases()
    finally:
        sts.set_knob("select_spin_limit", None)


def _lookback_cases():
    hm = [0, 1, 1, 2]
    for N, k, levels in ((200000, 20000, 0), (70001, 7000, 0), (100000, 50000, 3)):
        if levels:
            g = torch.Generator().manual_seed(N)
            scores = torch.randint(0, levels, (2, 3, 2, N), generator=g).float() / 4.0
        else:
            scores = softmax_scores(N, 2, 3, 2, N)
        lens = torch.tensor([N, N - 12345], dtype=torch.int32)
        (idx, cnt, _), (o_idx, o_cnt, _) = run_both(scores, hm, k, seq_lens=lens)
        np.testing.assert_array_equal(cnt, o_cnt)
        np.testing.assert_array_equal(idx, o_idx)


def launched(fn):
    """Kernel kinds launched by fn(), from the library's own launch records."""
    sts.prof_enable(True)
    sts.prof_reset()
    try:
        fn()
        torch.cuda.synchronize()
        return {k for k, (n, _) in sts.prof_read().items() if n}
    finally:
        sts.prof_enable(False)


FUSED = {"select_clear", "select_fused"}
BAND = {"select_band"}


def test_each_selection_path_is_taken_where_expected(select_path):
    """Ways through sts_select, chosen from the shape: one workgroup per row (short rows); for
    long rows the one-launch selection, or, with that switched off, chunk-local top-k + pool
    (small budgets) and the histogram pipeline (the rest)."""
    def run(B, Hd, N, k):
        s = softmax_scores(3, B, Hd, 2, N).to(DEV)
        return launched(lambda: sts.sts_select(s, list(range(Hd)), k))
    pipeline = {"select_clear", "select_agg", "select_hist", "select_write"}
    pool = {"select_local", "select_pool"}
    if select_path == 5:
        assert run(1, 4, 8192, 100) == {"select_band"} and run(1, 4, 65536, 512) == {"select_band"}
        assert run(1, 4, 65532 + 2, 512) == FUSED                           # N % 4 != 0: not its shape
        assert run(1, 1, 4096 * 300, 100) == {"select_clear", "select_agg", "select_hist", "select_write"}   # beyond its bitmap
        return
    assert run(1, 4, 8192, 100) == {"select_small"}
    assert run(16, 16, 20000, 100) == {"select_small"}                      # 256 rows
    if select_path == 3:
        assert run(1, 2, 32768 * 40, 100) == FUSED                          # 40 parts per row
        return
    if select_path == 0:
        assert run(1, 4, 8196, 100) == FUSED
        assert run(1, 4, 65536, 512) == FUSED
        assert run(16, 4, 65536, 4097) == FUSED
        assert run(1, 4, 65532 + 2, 512) == FUSED                           # N % 4 != 0: scalar variant
        assert run(2, 4, 262144, 100) == FUSED                              # 8 parts of 32768: the limit
        assert run(2, 4, 262144 + 4, 100) == pool                           # beyond it: the earlier paths
        assert run(1, 1, 4096 * 300, 100) == pipeline
        return
    assert run(1, 4, 65536, 512) == pool                                    # 8 chunks of 8192 x 512
    assert run(1, 4, 65536, 1024) == pool                                   # 8192 pooled pairs: the limit
    assert run(1, 4, 65536, 4096) == pipeline                               # 2 chunks of 32768: 8 workgroups only
    assert run(16, 4, 65536, 4096) == pool                                  # 64 rows x 2 chunks of 32768 x 4096
    assert run(16, 4, 65536, 4097) == pipeline
    assert run(1, 4, 65532 + 2, 512) == pipeline                            # N % 4 != 0
    assert run(8, 16, 65536, 2048) == pool                                  # 16384 pooled, 8M scores
    assert run(8, 16, 65536, 8192) == pool                                  # 2 x 8192 pooled, 8M scores
    assert run(8, 16, 65536, 8193) == pipeline


@pytest.mark.parametrize("kind,reduce", [(0, 0), (0, 1), (1, 0)])
def test_pool_path_options(kind, reduce, select_path):
    """Chunk-local top-k + pool with every option of the call: scaled-logit input, maximum
    reduction, ragged lengths (one ending inside the first chunk, one between chunks, one
    empty), per-head budgets, a draft head nobody reads, and the aggregate on request."""
    B, Hd, Tq, N, k = 4, 4, 3, 40000, 700
    g = torch.Generator().manual_seed(17 + kind + 2 * reduce)
    logits = torch.randn(B, Hd, Tq, N, generator=g) * 2.0
    lse = torch.logsumexp(logits, dim=-1)
    scores = logits if kind == 1 else torch.softmax(logits, dim=-1)
    hm = [0, 0, 2, 3, 3, 2]                                # draft head 1 is not read
    kh = [700, 5, 1, 333]
    lens = torch.tensor([N, 5000, 16384, 0], dtype=torch.int32)
    sd = scores.to(DEV)
    got = {}
    def call():
        got["r"] = sts.sts_select(sd, hm, k, lse=lse.to(DEV) if kind == 1 else None, seq_lens=lens.to(DEV),
                                  kind=kind, reduce=reduce, want_agg=True, k_head=kh)
    assert launched(call) == ({"select_local", "select_pool"} if select_path == 2 else BAND if select_path == 5 else FUSED)
    idx, cnt, agg = got["r"]
    agg = agg.cpu().numpy()
    o_agg = stored_agg(oracle.aggregate(scores.numpy(), lse.numpy() if kind == 1 else None, kind, reduce), lens)
    if kind == 0:
        np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    else:
        np.testing.assert_allclose(agg, o_agg, rtol=1e-5, atol=1e-12)
    # stage-wise: rank the GPU's own aggregate with the oracle
    sel, c = oracle.select_per_head(agg, k, kh, lens.numpy())
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    # without the aggregate output the lists are the same
    idx2, cnt2, _ = sts.sts_select(sd, hm, k, lse=lse.to(DEV) if kind == 1 else None, seq_lens=lens.to(DEV),
                                   kind=kind, reduce=reduce, k_head=kh)
    assert torch.equal(idx2, idx) and torch.equal(cnt2, cnt)


@pytest.mark.parametrize("levels", [1, 2, 5])
def test_pool_path_ties_across_chunks(levels):
    """Equal scores in different chunks: the lower token must win, whichever chunk holds it."""
    B, Hd, Tq, N = 2, 3, 2, 81920                           # 10 chunks
    g = torch.Generator().manual_seed(levels)
    scores = torch.randint(0, levels, (B, Hd, Tq, N), generator=g).float() / 4.0
    for k in (1, 7, 300, 819):
        (idx, cnt, _), (o_idx, o_cnt, _) = run_both(scores, [0, 1, 2, 1], k)
        np.testing.assert_array_equal(cnt, o_cnt)
        np.testing.assert_array_equal(idx, o_idx)


@pytest.mark.parametrize("B,Hd,Tq,N,Hq,k", [
    (1, 16, 5, 4096, 32, 410),        # one workgroup per row
    (2, 3, 5, 20000, 6, 2000),        # chunk-local top-k + pool
    (2, 3, 5, 40000, 6, 4000),        # histogram pipeline
    (1, 2, 3, 70001, 4, 123),         # its scalar variant (N % 4 != 0)
    (1, 2, 9, 1001, 2, 100),          # scalar, more than one group of eight rows
])
@pytest.mark.parametrize("kind", [0, 1])
def test_select_bf16_scores(B, Hd, Tq, N, Hq, k, kind):
    """Scores stored as bf16 (half the bytes): the result equals that of the same call on the
    widened tensor, which is what the oracle gets."""
    g = torch.Generator().manual_seed(N + kind)
    logits = (torch.randn(B, Hd, Tq, N, generator=g) * 2.0).to(torch.bfloat16)
    lse = torch.logsumexp(logits.float(), dim=-1)
    scores = logits if kind == 1 else torch.softmax(logits.float(), dim=-1).to(torch.bfloat16)
    hm = [(t * Hd) // Hq for t in range(Hq)]
    idx, cnt, agg = sts.sts_select(scores.to(DEV), hm, k, lse=lse.to(DEV) if kind == 1 else None, kind=kind,
                                   want_agg=True)
    torch.cuda.synchronize()
    wide = scores.float().numpy()
    o_agg = oracle.aggregate(wide, lse.numpy() if kind == 1 else None, kind, 0)
    agg = agg.cpu().numpy()
    if kind == 0:
        np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    else:
        np.testing.assert_allclose(agg, o_agg, rtol=1e-5, atol=1e-12)
    sel, c = oracle.select(agg, k)
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    # the same call on the widened tensor gives the same lists
    idx32, cnt32, _ = sts.sts_select(scores.float().to(DEV), hm, k, lse=lse.to(DEV) if kind == 1 else None, kind=kind)
    assert torch.equal(idx32, idx) and torch.equal(cnt32, cnt)


def test_bf16_dump_feeds_selection():
    """Draft attention dumps bf16 logits + fp32 LSE; the selection reads them as they are."""
    cfg = replace(CONFIGS["c5"], B=1, N=20000, Hq=16, Hkv=2, Tq=4, Hd=8, draft_Hkv=2)
    from workload import make_draft_layer
    w = make_workload(cfg, seed=4)
    dl = make_draft_layer(w)
    dq, dk, dv = dl["q"].to(DEV), dl["k"].to(DEV), dl["v"].to(DEV)
    _, d_lse, d_logits = sts.sts_dense_attn(dq, dk, dv, dl["scale"], want_logits=torch.bfloat16)
    assert d_logits.dtype == torch.bfloat16
    k = 1500
    idx, cnt, agg = sts.sts_select(d_logits, w.head_map, k, lse=d_lse, kind=sts.STS_SCORES_LOGITS_LSE, want_agg=True)
    torch.cuda.synchronize()
    o_agg = oracle.aggregate(d_logits.float().cpu().numpy(), d_lse.cpu().numpy(), 1, 0)
    np.testing.assert_allclose(agg.cpu().numpy(), o_agg, rtol=1e-5, atol=1e-12)
    sel, c = oracle.select(agg.cpu().numpy(), k)
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(w.head_map, np.int32))
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)


def test_misaligned_scores_fall_back_to_the_pipeline(select_path):
    """A pool-shaped call whose score pointer is not 16-byte aligned runs the histogram pipeline
    (scalar loads) inside the same workspace, with the same result; the one-launch selection takes
    its scalar variant."""
    B, Hd, Tq, N, k = 1, 3, 2, 40000, 500
    base = torch.zeros(B * Hd * Tq * N + 1, dtype=torch.float32)
    scores = base[1:].view(B, Hd, Tq, N)
    scores.copy_(softmax_scores(8, B, Hd, Tq, N))
    dbase = base.to(DEV)
    sd = dbase[1:].view(B, Hd, Tq, N)
    assert sd.data_ptr() % 16 == 4
    got = {}
    kinds = launched(lambda: got.update(r=sts.sts_select(sd, [0, 1, 2], k)))
    assert kinds == ({"select_clear", "select_agg", "select_hist", "select_write"} if select_path == 2 else FUSED)   # also with path 5
    o_idx, o_cnt, _ = oracle.select_indices(scores.numpy(), np.asarray([0, 1, 2], np.int32), k)
    np.testing.assert_array_equal(got["r"][0].cpu().numpy(), o_idx)
    np.testing.assert_array_equal(got["r"][1].cpu().numpy(), o_cnt)


@pytest.mark.parametrize("levels", [0, 3])
def test_pool_path_with_32768_token_chunks(levels, select_path):
    """Long rows with middle budgets: the pool stays small only with 32768-token chunks (1024
    threads per workgroup). Ragged lengths ending inside a chunk, on a chunk boundary and at 0."""
    B, Hd, Tq, N, k = 3, 11, 3, 100000, 2000         # 13 x 2000 is too much, 4 x 2000 fits; 33 rows x 4 chunks
    g = torch.Generator().manual_seed(40 + levels)
    if levels:
        scores = torch.randint(0, levels, (B, Hd, Tq, N), generator=g).float() / 4.0
    else:
        scores = softmax_scores(40, B, Hd, Tq, N)
    lens = torch.tensor([N, 65536, 0], dtype=torch.int32)
    hm, kh = [1, 0, 10, 5], [2000, 77] + [1500] * 9
    sd = scores.to(DEV)
    got = {}
    kinds = launched(lambda: got.update(r=sts.sts_select(sd, hm, k, seq_lens=lens.to(DEV), k_head=kh, want_agg=True)))
    assert kinds == ({"select_local", "select_pool"} if select_path == 2 else BAND if select_path == 5 else FUSED)
    idx, cnt, agg = got["r"]
    o_idx, o_cnt, o_agg = oracle.select_indices(scores.numpy(), np.asarray(hm, np.int32), k, seq_lens=lens.numpy(),
                                                k_head=kh)
    np.testing.assert_array_equal(agg.cpu().numpy().view(np.uint32), stored_agg(o_agg, lens).view(np.uint32))
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)


def test_hand_worked_cases_on_the_gpu():
    """The hand-worked fixture (tests/golden/select_handworked.json) straight through the library."""
    import json
    import os
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "select_handworked.json")) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        P = torch.tensor(case["probs"], dtype=torch.float32)[None].contiguous()      # [1,Hd,Tq,N]
        idx, cnt, agg = sts.sts_select(P.to(DEV), case["head_map"], case["k"], page_size=case.get("page", 1),
                                       k_head=case.get("k_head"), want_agg=True)
        np.testing.assert_array_equal(idx[0].cpu().numpy(), np.array(case["indices"], np.int32))
        np.testing.assert_array_equal(agg[0].cpu().numpy(), np.array(case["agg"], np.float32))
        if "counts" in case:
            np.testing.assert_array_equal(cnt[0].cpu().numpy(), np.array(case["counts"], np.int32))


@pytest.mark.parametrize("N,k,levels,off", [
    (40000, 9000, 0, 0),       # vector path
    (40000, 9000, 50, 0),      # heavy ties across chunks
    (70001, 20000, 0, 0),      # N % 4 != 0: scalar path
    (40004, 9000, 0, 1),       # misaligned base: scalar path on the caller's own tensor
])
def test_single_row_input_is_ranked_in_place(N, k, levels, off, select_path):
    """One fp32 probability row per head (Tq = 1; e.g. a ready-made aggregate) on the
    multi-workgroup pipeline: the rows are ranked where they lie (no copy into the workspace),
    the input stays untouched, and asking for the aggregate returns the input itself."""
    B, Hd, Hq = 2, 3, 6
    g = torch.Generator().manual_seed(5)
    if levels:
        s = torch.randint(0, levels, (B, Hd, 1, N), generator=g).float() / levels
    else:
        s = torch.softmax(torch.randn(B, Hd, 1, N, generator=g) * 2.0, dim=-1)
    head_map = [0, 0, 1, 1, 2, 2]
    lens = torch.tensor([N, N - 4097], dtype=torch.int32)
    flat = torch.zeros(s.numel() + 4, dtype=torch.float32, device=DEV)
    sd = flat[off:off + s.numel()].view(B, Hd, 1, N)
    sd.copy_(s)
    got = {}
    kinds = launched(lambda: got.update(r=sts.sts_select(sd, head_map, k, seq_lens=lens.to(DEV))))
    if not (select_path == 5 and off == 0):     # (an aligned tensor of the one-pass selection's shape goes there)
        assert kinds == ({"select_clear", "select_agg", "select_hist", "select_write"} if select_path == 2 else FUSED)
    idx, cnt, _ = got["r"]
    assert torch.equal(sd.cpu(), s)
    o_idx, o_cnt, o_agg = oracle.select_indices(s.numpy(), np.asarray(head_map, np.int32), k, seq_lens=lens.numpy())
    assert np.array_equal(idx.cpu().numpy(), o_idx) and np.array_equal(cnt.cpu().numpy(), o_cnt)
    idx2, cnt2, agg2 = sts.sts_select(sd, head_map, k, seq_lens=lens.to(DEV), want_agg=True)
    assert torch.equal(idx2, idx) and torch.equal(cnt2, cnt)
    for b, n in enumerate(lens.tolist()):
        assert np.array_equal(agg2[b, :, :n].cpu().numpy(), o_agg[b, :, :n])


@pytest.mark.parametrize("B,Hd,N,Hq,k,bf16,what", [
    (2, 4, 40000, 8, 700, False, "softmax"),        # fp32, three levels, rows of 40000 (not a multiple of a step)
    (2, 4, 40000, 8, 700, True, "softmax"),         # bf16: many ties among the widened values, two levels
    (1, 3, 16392, 3, 16392, False, "softmax"),      # k = N: everything kept
    (1, 2, 9000, 4, 100, True, "signed"),           # negative and positive scores, -0 and +0
    (1, 2, 9000, 4, 8000, True, "signed"),          # ... with the threshold among the negative ones
    (1, 2, 9000, 4, 8000, False, "signed"),
    (1, 2, 70000, 2, 5000, False, "quantised"),     # a handful of distinct values: the tie rule decides
    (1, 2, 70000, 2, 5000, True, "constant"),       # all equal: the first k tokens
    (72, 16, 8200, 16, 300, True, "softmax"),       # 1152 rows: the small workgroups the rule takes for many rows
    (72, 16, 8200, 16, 300, False, "softmax"),
    (2, 2, 70000, 2, 5000, True, "unsampled"),      # the sample puts the window of second-digit histograms in the wrong place
    (2, 2, 70000, 2, 5000, True, "clustered"),
    (2, 2, 70000, 2, 60000, True, "softmax"),       # the threshold far down the row
])
def test_one_workgroup_per_row_selection(B, Hd, N, Hq, k, bf16, what):
    """Single-score rows (Tq = 1) ranked by one workgroup per row in several passes over the row:
    index sets and counts bit for bit against the oracle, with ragged lengths (one ending inside a
    16-byte word, one empty), per-head budgets, a draft head read by several target heads and one
    read by none."""
    g = torch.Generator().manual_seed(N + k + bf16)
    if what == "softmax":
        scores = torch.softmax(torch.randn(B, Hd, 1, N, generator=g) * 2, dim=-1)
    elif what == "signed":
        scores = torch.randn(B, Hd, 1, N, generator=g)
        scores[..., ::7] = 0.0
        scores[..., 3::14] = -0.0
    elif what == "quantised":
        scores = torch.randint(0, 5, (B, Hd, 1, N), generator=g).float() / 8
    elif what == "constant":
        scores = torch.full((B, Hd, 1, N), 0.25)
    else:
        scores = band_scores(what, B, Hd, 1, N, N + k)
    if bf16:
        scores = scores.to(torch.bfloat16)
    hm = [min(t // 2, Hd - 1) for t in range(Hq)] if Hq > Hd else list(range(Hq))     # pairs share; the last heads may be unread
    kh = [max(1, k - 37 * j) for j in range(Hd)]
    lens = torch.full((B,), N, dtype=torch.int32)
    if B > 1:
        lens[1] = N - 13
    if B > 2:
        lens[2] = 0
        lens[3] = 5
    sd = scores.to(DEV)
    sts.set_knob("select_path", 4)
    try:
        got = {}
        kinds = launched(lambda: got.update(r=sts.sts_select(sd, hm, k, seq_lens=lens.to(DEV), k_head=kh)))
    finally:
        sts.set_knob("select_path", None)
    assert kinds == {"select_rowpass"}
    idx, cnt, _ = got["r"]
    o_idx, o_cnt, _ = oracle.select_indices(scores.float().numpy(), np.asarray(hm, np.int32), k, k_head=kh, seq_lens=lens.numpy())
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)


def test_calls_with_many_rows_take_one_workgroup_per_row():
    """The library's own rule for rows longer than one workgroup's LDS holds: from one row for
    every second compute unit on, one workgroup per row in one pass (any number of scores per
    token, the aggregate on request); one bf16 score per token and four rows per compute unit or
    more: one small workgroup per row in several passes; fewer rows, block granularity, or a
    budget whose band cannot fit keep the other paths."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    N = 32768 + 8
    hm = list(range(16))
    sts.set_knob("select_path", 0)
    try:
        s = torch.rand(cus // 32, 16, 2, N, device=DEV)                       # cus / 2 rows
        assert launched(lambda: sts.sts_select(s, hm, 100)) == {"select_band"}
        assert launched(lambda: sts.sts_select(s, hm, 100, want_agg=True)) == {"select_band"}
        assert launched(lambda: sts.sts_select(s.to(torch.bfloat16), hm, 3000)) == {"select_band"}
        assert "select_band" not in launched(lambda: sts.sts_select(s[:-1], hm, 100))
        assert "select_band" not in launched(lambda: sts.sts_select(s, hm, 100, page_size=8))
        assert "select_band" not in launched(lambda: sts.sts_select(s, hm, N - 100))        # nearly everything kept
        assert launched(lambda: sts.sts_select(s[:, :, :, :8192].contiguous(), hm, 100)) == {"select_small"}
        del s
        s1 = torch.rand(cus // 4, 16, 1, 8192 + 8, device=DEV)                # 4 rows per compute unit, one score per token
        assert launched(lambda: sts.sts_select(s1, hm, 100)) == {"select_small"}             # short rows, many of them
        s1 = torch.rand(cus // 4, 16, 1, N, device=DEV)
        assert launched(lambda: sts.sts_select(s1, hm, 100)) == {"select_band"}
        assert launched(lambda: sts.sts_select(s1.to(torch.bfloat16), hm, 100)) == {"select_rowpass"}
        assert launched(lambda: sts.sts_select(s1[:-1].to(torch.bfloat16), hm, 100)) == {"select_band"}
    finally:
        sts.set_knob("select_path", None)


def band_scores(what, B, Hd, Tq, N, seed):
    g = torch.Generator().manual_seed(seed)
    if what == "softmax":
        return torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1)
    if what == "signed":
        s = torch.randn(B, Hd, Tq, N, generator=g)
        s[..., ::7] = 0.0
        s[..., 3::14] = -0.0
        return s
    if what == "quantised":                        # a handful of distinct values: the band cannot hold the ties
        return torch.randint(0, 5, (B, Hd, Tq, N), generator=g).float() / 8
    if what == "constant":
        return torch.full((B, Hd, Tq, N), 0.25)
    if what == "clustered":                        # all heavy tokens in one stretch that the strided sample mostly misses
        s = torch.rand(B, Hd, Tq, N, generator=g) * 1e-3
        lo = N // 3
        s[..., lo:lo + N // 8] += 1.0
        return s
    if what == "unsampled":                        # heavy tokens only where neither kernel's strided sample looks
        s = torch.rand(B, Hd, Tq, N, generator=g) * 1e-3
        pos = torch.arange(N)
        s[..., (pos % 512) >= 64] += torch.rand(int(((pos % 512) >= 64).sum()), generator=g) + 0.5
        return s
    if what == "recent":                           # heavy tokens at the end of the context, plus scattered ones
        s = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1)
        s[..., -N // 20:] *= 50
        return s
    raise ValueError(what)


@pytest.mark.parametrize("B,Hd,Tq,N,Hq,k,dtype,what", [
    (2, 4, 5, 40000, 8, 4000, torch.float32, "softmax"),       # the usual shape: sample, one pass, band
    (2, 4, 1, 40000, 8, 4000, torch.bfloat16, "softmax"),      # bf16: ties at the threshold, the lower tokens win
    (2, 3, 3, 131072, 6, 13108, torch.float32, "softmax"),     # 128K rows, 10%
    (1, 2, 2, 262144 + 64, 2, 3000, torch.float32, "softmax"), # sample stride 64
    (2, 4, 5, 40000, 8, 100, torch.float32, "softmax"),        # small budget: no upper edge, the band is the top of the row
    (2, 4, 5, 40000, 8, 20000, torch.float32, "softmax"),      # half of the row
    (2, 4, 5, 40000, 8, 39000, torch.float32, "softmax"),      # nearly everything: ranked by plain passes
    (2, 2, 1, 9000, 4, 8000, torch.bfloat16, "signed"),        # negative keys, -0 and +0
    (2, 2, 2, 70000, 2, 5000, torch.float32, "quantised"),     # ties overflow the band: plain passes
    (2, 2, 1, 70000, 2, 5000, torch.bfloat16, "constant"),     # all equal: the first k tokens
    (2, 2, 2, 70000, 2, 5000, torch.float32, "clustered"),     # the sample misleads: the check sends the row to plain passes
    (2, 2, 4, 70000, 2, 3000, torch.float32, "recent"),
    (2, 2, 2, 70000, 2, 5000, torch.float32, "unsampled"),
    (2, 2, 1, 70000, 2, 5000, torch.bfloat16, "unsampled"),
    (2, 2, 1, 524288, 2, 3000, torch.float32, "softmax"),      # the longest row the bitmap holds, sample stride 32
    (2, 2, 2, 524288 - 64, 2, 40000, torch.bfloat16, "softmax"), # ... and a budget whose band cannot fit there: plain passes
    (2, 4, 5, 8000, 8, 777, torch.float32, "softmax"),         # rows that fit the band store whole: no sample
    (2, 4, 5, 8196, 8, 777, torch.float32, "softmax"),         # just above that
])
def test_one_workgroup_per_row_one_pass_selection(B, Hd, Tq, N, Hq, k, dtype, what):
    """select_band_kernel: index sets, counts and the aggregate bit for bit against the oracle,
    whichever way a row goes inside the kernel (band, or plain passes when the band does not fit or
    the sample misled), with ragged lengths, per-head budgets, shared and unread draft heads."""
    scores = band_scores(what, B, Hd, Tq, N, N + k + Tq).to(dtype)
    hm = [min(t // 2, Hd - 1) for t in range(Hq)] if Hq > Hd else list(range(Hq))
    kh = [max(1, k - 37 * j) for j in range(Hd)]
    lens = torch.full((B,), N, dtype=torch.int32)
    lens[-1] = N - 13
    sd = scores.to(DEV)
    sts.set_knob("select_path", 5)
    try:
        got = {}
        kinds = launched(lambda: got.update(r=sts.sts_select(sd, hm, k, seq_lens=lens.to(DEV), k_head=kh, want_agg=True)))
        idx2, cnt2, _ = sts.sts_select(sd, hm, k, seq_lens=lens.to(DEV), k_head=kh)
    finally:
        sts.set_knob("select_path", None)
    assert kinds == {"select_band"}
    idx, cnt, agg = got["r"]
    o_idx, o_cnt, o_agg = oracle.select_indices(scores.float().numpy(), np.asarray(hm, np.int32), k, k_head=kh, seq_lens=lens.numpy())
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    np.testing.assert_array_equal(agg.cpu().numpy().view(np.uint32), stored_agg(o_agg, lens).view(np.uint32))
    assert torch.equal(idx2, idx) and torch.equal(cnt2, cnt)


@pytest.mark.parametrize("kind,reduce", [(0, 1), (1, 0)])
def test_one_pass_selection_options(kind, reduce):
    """The same kernel with scaled-logit input and with the maximum reduction; lengths that end
    inside a quad, inside the first sampled run, and at zero."""
    B, Hd, Tq, N, k = 4, 4, 3, 40000, 700
    g = torch.Generator().manual_seed(23 + kind + 2 * reduce)
    logits = torch.randn(B, Hd, Tq, N, generator=g) * 2.0
    lse = torch.logsumexp(logits, dim=-1)
    scores = logits if kind == 1 else torch.softmax(logits, dim=-1)
    hm = [0, 0, 2, 3, 3, 2]
    kh = [700, 5, 1, 333]
    lens = torch.tensor([N, 9001, 7, 0], dtype=torch.int32)
    sts.set_knob("select_path", 5)
    try:
        idx, cnt, agg = sts.sts_select(scores.to(DEV), hm, k, lse=lse.to(DEV) if kind == 1 else None, seq_lens=lens.to(DEV),
                                       kind=kind, reduce=reduce, want_agg=True, k_head=kh)
    finally:
        sts.set_knob("select_path", None)
    agg = agg.cpu().numpy()
    o_agg = stored_agg(oracle.aggregate(scores.numpy(), lse.numpy() if kind == 1 else None, kind, reduce), lens)
    if kind == 0:
        np.testing.assert_array_equal(agg.view(np.uint32), o_agg.view(np.uint32))
    else:
        np.testing.assert_allclose(agg, o_agg, rtol=1e-5, atol=1e-12)
    sel, c = oracle.select_per_head(agg, k, kh, lens.numpy())       # stage-wise: rank the GPU's own aggregate
    o_idx, o_cnt = oracle.remap(sel, c, np.asarray(hm, np.int32))
    np.testing.assert_array_equal(cnt.cpu().numpy(), o_cnt)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
