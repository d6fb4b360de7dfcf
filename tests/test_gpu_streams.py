"""Drafting-speculation pipelining (Section 5: mask generation runs on its own stream beside
the forward pass, ordered by events). The library only enqueues on the caller's stream and
never synchronises, so mask building for the next round can overlap attention of the current
one. Results must equal the oracle's (and, bit for bit, the sequential run's)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts
from gpu_util import check_attn
from workload import CONFIGS, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_select_overlaps_attention_on_a_second_stream():
    cfg = replace(CONFIGS["c2"], N=16384)
    w0 = make_workload(cfg, seed=1)
    w1 = make_workload(cfg, seed=2)
    k = w0.k_budget
    hm = w0.head_map
    dev = lambda w: [t.to(DEV) for t in (w.q, w.k, w.v, w.scores)]
    (q0, k0, v0, s0), (q1, k1, v1, s1) = dev(w0), dev(w1)
    # sequential reference
    i0, c0, _ = sts.sts_select(s0, hm, k)
    o0, l0 = sts.sts_sparse_attn(q0, k0, v0, i0, w0.scale, counts=c0, head_map=hm, out_dtype=torch.float32)
    i1, c1, _ = sts.sts_select(s1, hm, k)
    o1, l1 = sts.sts_sparse_attn(q1, k1, v1, i1, w1.scale, counts=c1, head_map=hm, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (i0, c0, o0, l0, i1, c1, o1, l1)]

    main, side = torch.cuda.Stream(), torch.cuda.Stream()        # default priority on both
    idx = [torch.empty_like(i0), torch.empty_like(i0)]
    cnt = [torch.empty_like(c0), torch.empty_like(c0)]
    out = [torch.empty_like(o0), torch.empty_like(o0)]
    lse = [torch.empty_like(l0), torch.empty_like(l0)]
    mask_ready = [torch.cuda.Event(), torch.cuda.Event()]
    torch.cuda.synchronize()
    for rep in range(3):
        with torch.cuda.stream(side):
            sts.sts_select(s0, hm, k, out=(idx[0], cnt[0]))
            mask_ready[0].record(side)
        with torch.cuda.stream(main):
            main.wait_event(mask_ready[0])
            sts.sts_sparse_attn(q0, k0, v0, idx[0], w0.scale, counts=cnt[0], head_map=hm, out=out[0], lse_out=lse[0])
        with torch.cuda.stream(side):
            # the next round's mask is built while the attention above runs
            sts.sts_select(s1, hm, k, out=(idx[1], cnt[1]))
            mask_ready[1].record(side)
        with torch.cuda.stream(main):
            main.wait_event(mask_ready[1])
            sts.sts_sparse_attn(q1, k1, v1, idx[1], w1.scale, counts=cnt[1], head_map=hm, out=out[1], lse_out=lse[1])
        torch.cuda.synchronize()
        got = (idx[0], cnt[0], out[0], lse[0], idx[1], cnt[1], out[1], lse[1])
        for g, r in zip(got, ref):
            assert torch.equal(g, r)
    # what the two streams produced, against the oracle: index sets bit for bit, outputs in tolerance
    for w, i, c, o, l in ((w0, idx[0], cnt[0], out[0], lse[0]), (w1, idx[1], cnt[1], out[1], lse[1])):
        o_idx, o_cnt, _ = oracle.select_indices(w.scores.numpy(), np.asarray(hm, np.int32), k)
        np.testing.assert_array_equal(i.cpu().numpy(), o_idx)
        np.testing.assert_array_equal(c.cpu().numpy(), o_cnt)
        ref_attn = oracle.attn(oracle.bf16_bits(w.q), oracle.bf16_bits(w.k), oracle.bf16_bits(w.v), w.scale, o_idx, o_cnt)
        check_attn(o, l, ref_attn, what="two streams")
