"""GPU: sts_sparse_attn_static (the entry point that allocates nothing: its per-split partials go
to the library's static device array) against sts_sparse_attn on the same inputs, through the
C ABI. Two calls in a row share the array, the second with a smaller input; both must equal the
workspace call bit for bit (same kernels, same split count) and match the oracle."""
import ctypes
import math

import numpy as np
import pytest
import torch

import paper_2605_15508_amd as sts
from gpu_util import check_attn, oracle_attn
from paper_2605_15508_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(seed, B, Tq, Hq, Hkv, d, N, kk, shared):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16).to(DEV)
    k = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    v = (torch.randn(B, Hkv, N, d, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    head_map = [t // shared for t in range(Hq)]
    rng = np.random.default_rng(seed + 1)
    idx = np.empty((B, Hq, kk), np.int32)
    for b in range(B):
        rows = {}
        for t in range(Hq):
            if head_map[t] not in rows:
                rows[head_map[t]] = np.sort(rng.choice(N, kk, replace=False))
            idx[b, t] = rows[head_map[t]]
    cnt = torch.full((B, Hq), kk, dtype=torch.int32)
    cnt[:, ::3] = max(1, kk - 7)                      # some shorter lists (equal within a head set only if shared == 1)
    if shared > 1:
        cnt = cnt[:, [t - t % shared for t in range(Hq)]]
    return q, k, v, torch.from_numpy(idx).to(DEV), cnt.to(DEV), head_map


def _both(case):
    q, k, v, idx, cnt, head_map = case
    B, Tq, Hq, d = q.shape
    scale = 1.0 / math.sqrt(d)
    plan = sts.attn_plan(q, k, True, kmax=idx.shape[2], head_map=head_map)
    # preallocated outputs: neither the wrapper nor the C call allocates in the static call
    out_s = torch.full((B, Tq, Hq, d), float("nan"), dtype=torch.float32, device=DEV)
    lse_s = torch.full((B, Hq, Tq), float("nan"), dtype=torch.float32, device=DEV)
    out_w, lse_w = sts.sts_sparse_attn(q, k, v, idx, scale, counts=cnt, head_map=head_map, out_dtype=torch.float32)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sts.sts_sparse_attn_static(q, k, v, idx, scale, counts=cnt, head_map=head_map, out=out_s, lse_out=lse_s)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.equal(out_s, out_w), "static-scratch call differs from the workspace call"
    assert torch.equal(lse_s, lse_w)
    ref = oracle_attn(q, k, v, scale, idx, cnt)
    check_attn(out_s, lse_s, ref, what="static scratch")
    return plan


def test_two_calls_in_a_row_share_the_static_scratch():
    # first call: lists long enough to be split (partials + combine go through the array);
    # second call: a smaller input that reuses the array with the first call's contents in it
    big = _inputs(11, 2, 5, 8, 2, 128, 6000, 2400, 2)
    small = _inputs(12, 1, 5, 8, 2, 128, 3000, 1100, 2)
    plan_big = _both(big)
    plan_small = _both(small)
    assert plan_big["num_splits"] > 1 and plan_small["num_splits"] > 1, (plan_big, plan_small)
    # and once more the other way round, head size 64, single-split lists (no partials at all)
    _both(_inputs(13, 1, 3, 4, 2, 64, 500, 90, 1))
    _both(big)


def test_a_shape_beyond_the_array_is_refused():
    # 256 heads on their own, lists long enough for 2 splits: partials exceed 8 MiB
    B, Tq, Hq, Hkv, d, N, kk = 4, 16, 256, 16, 128, 4096, 2048
    q = torch.zeros(B, Tq, Hq, d, dtype=torch.bfloat16, device=DEV)
    k = torch.zeros(B, Hkv, N, d, dtype=torch.bfloat16, device=DEV)
    idx = torch.zeros(B, Hq, kk, dtype=torch.int32, device=DEV)
    out = torch.zeros(B, Tq, Hq, d, dtype=torch.bfloat16, device=DEV)
    p, _keep = binding._attn_params(q, k, k, 0.1, idx, None, None, None, out, None, None)
    lib = sts.load_library()
    need = lib.sts_attn_workspace_bytes(ctypes.byref(p), 1)
    assert need > sts.STS_STATIC_SCRATCH_BYTES
    rc = lib.sts_sparse_attn_static(ctypes.byref(p), binding._stream())
    assert rc == -3 and b"workspace" in lib.sts_strerror(rc)
    torch.cuda.synchronize()
