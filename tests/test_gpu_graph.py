"""The whole path (select -> sparse attention, and dense) captured into a HIP graph and
replayed several times with new inputs, each replay checked against the eager result. The
library enqueues kernels only (no memset nodes, no allocation, no synchronisation), which is
what makes it capturable."""
from dataclasses import replace

import pytest
import torch

import paper_2605_15508_amd as sts
from workload import CONFIGS, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("N,budget", [
    (6000, 0.10),      # one workgroup per row; N is not a multiple of the chunk or tile sizes
    (40000, 0.02),     # chunk-local top-k + pool
    (40000, 0.25),     # histogram pipeline: clear kernel, published chunk counts
])
def test_graph_replays_match_eager(N, budget):
    cfg = replace(CONFIGS["c1"], N=N)
    ws = [make_workload(cfg, seed=s, budget=budget) for s in (1, 2, 3)]
    k = ws[0].k_budget
    hm = ws[0].head_map
    B, Hq, Tq, d = cfg.B, cfg.Hq, cfg.Tq, cfg.d
    # static buffers the graph reads and writes
    q = ws[0].q.to(DEV).clone()
    kk = ws[0].k.to(DEV).clone()
    vv = ws[0].v.to(DEV).clone()
    sc = ws[0].scores.to(DEV).clone()
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device=DEV)
    cnt = torch.empty(B, Hq, dtype=torch.int32, device=DEV)
    out = torch.empty(B, Tq, Hq, d, dtype=torch.float32, device=DEV)
    lse = torch.empty(B, Hq, Tq, dtype=torch.float32, device=DEV)
    dout = torch.empty_like(out)

    def path():
        sts.sts_select(sc, hm, k, out=(idx, cnt))
        sts.sts_sparse_attn(q, kk, vv, idx, ws[0].scale, counts=cnt, head_map=hm, out=out, lse_out=lse)
        sts.sts_dense_attn(q, kk, vv, ws[0].scale, out=dout, want_lse=False)

    path()                                        # warm-up: workspaces get allocated here
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    torch.cuda.synchronize()

    for w in ws + ws[:1]:
        q.copy_(w.q.to(DEV)); kk.copy_(w.k.to(DEV)); vv.copy_(w.v.to(DEV)); sc.copy_(w.scores.to(DEV))
        path()                                    # eager
        torch.cuda.synchronize()
        want = [t.clone() for t in (idx, cnt, out, lse, dout)]
        for t in (idx, cnt, out, lse, dout):
            t.fill_(0) if t.dtype == torch.int32 else t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((idx, cnt, out, lse, dout), want):
            assert torch.equal(got, ref)


def test_graph_replays_of_the_draft_chain_match_eager():
    """Draft attention with its summed weights -> in-place selection -> sparse attention, captured
    and replayed with new inputs (the second pass over K and the histogram-only first pass of the
    selection are ordinary kernel nodes as well)."""
    B, Tq, Hq, Hkv, d, N, Hd, dd, k = 2, 4, 8, 2, 128, 40000, 4, 64, 9000
    hm = [t * Hd // Hq for t in range(Hq)]
    g = torch.Generator().manual_seed(11)

    def fresh():
        return dict(q=torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16),
                    k=(torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16),
                    v=(torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16),
                    qd=torch.randn(B, Tq, Hd, dd, generator=g).to(torch.bfloat16),
                    kd=(torch.randn(B, Hkv, N, dd, generator=g) * 0.5).to(torch.bfloat16),
                    vd=(torch.randn(B, Hkv, N, dd, generator=g) * 0.5).to(torch.bfloat16))
    sets = [fresh() for _ in range(3)]
    buf = {n: t.to(DEV).clone() for n, t in sets[0].items()}
    A = torch.empty(B, Hd, N, dtype=torch.float32, device=DEV)
    dout = torch.empty(B, Tq, Hd, dd, dtype=torch.bfloat16, device=DEV)
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device=DEV)
    cnt = torch.empty(B, Hq, dtype=torch.int32, device=DEV)
    out = torch.empty(B, Tq, Hq, d, dtype=torch.float32, device=DEV)
    lse = torch.empty(B, Hq, Tq, dtype=torch.float32, device=DEV)

    def path():
        sts.sts_dense_attn(buf["qd"], buf["kd"], buf["vd"], 0.125, out=dout, want_lse=False, weights_sum_out=A)
        sts.sts_select(A.view(B, Hd, 1, N), hm, k, out=(idx, cnt))
        sts.sts_sparse_attn(buf["q"], buf["k"], buf["v"], idx, 0.09, counts=cnt, head_map=hm, out=out, lse_out=lse)

    path()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    torch.cuda.synchronize()
    for s in sets + sets[:1]:
        for n, t in s.items():
            buf[n].copy_(t.to(DEV))
        path()
        torch.cuda.synchronize()
        want = [t.clone() for t in (A, idx, cnt, out, lse)]
        for t in (A, out, lse):
            t.fill_(float("nan"))
        idx.fill_(0); cnt.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((A, idx, cnt, out, lse), want):
            assert torch.equal(got, ref)


def test_prepared_calls_repeat_the_call_on_fixed_buffers():
    """A PreparedCall holds the parameter block of a call: calling it again enqueues the same
    call; results equal those of the ordinary functions, also after the inputs changed in place."""
    from workload import CONFIGS, make_workload
    w = make_workload(CONFIGS["c1"], seed=5)
    q, k, v, scores = (t.to(DEV) for t in (w.q, w.k, w.v, w.scores))
    sel = sts.sts_select(scores, w.head_map, w.k_budget, prepare=True)
    idx, cnt, _ = sel()
    att = sts.sts_sparse_attn(q, k, v, idx, w.scale, counts=cnt, head_map=w.head_map, out_dtype=torch.float32, prepare=True)
    out, lse, _ = att()
    den = sts.sts_dense_attn(q, k, v, w.scale, out_dtype=torch.float32, prepare=True)
    dout, dlse, _ = den()
    torch.cuda.synchronize()
    r_idx, r_cnt, _ = sts.sts_select(scores, w.head_map, w.k_budget)
    r_out, r_lse = sts.sts_sparse_attn(q, k, v, r_idx, w.scale, counts=r_cnt, head_map=w.head_map, out_dtype=torch.float32)
    r_dout, r_dlse, _ = sts.sts_dense_attn(q, k, v, w.scale, out_dtype=torch.float32)
    assert torch.equal(idx, r_idx) and torch.equal(cnt, r_cnt) and torch.equal(out, r_out) and torch.equal(lse, r_lse)
    assert torch.equal(dout, r_dout) and torch.equal(dlse, r_dlse)
    # new scores in the same buffer: the prepared calls see them
    scores.copy_(torch.softmax(torch.randn_like(scores) * 2, dim=-1))
    sel(); att()
    torch.cuda.synchronize()
    r_idx, r_cnt, _ = sts.sts_select(scores, w.head_map, w.k_budget)
    r_out, _ = sts.sts_sparse_attn(q, k, v, r_idx, w.scale, counts=r_cnt, head_map=w.head_map, out_dtype=torch.float32)
    assert torch.equal(idx, r_idx) and torch.equal(out, r_out)
