"""GPU parity for Algorithm 1 (head-mapping construction, Section 4.1): map and overlap
counts must equal the oracle's exactly (all-integer work)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2605_15508_amd as sts

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_both(a_d, a_t, k):
    mp, ov = sts.sts_head_map(torch.from_numpy(a_d).to(DEV), torch.from_numpy(a_t).to(DEV), k)
    torch.cuda.synchronize()
    o_mp, o_ov = oracle.head_mapping(a_d, a_t, k)
    np.testing.assert_array_equal(ov.cpu().numpy(), o_ov)
    np.testing.assert_array_equal(mp.cpu().numpy(), o_mp)
    return o_mp, o_ov


def test_headmap_handworked_fixture_on_gpu():
    with open(os.path.join(GOLDEN, "headmap_handworked.json")) as f:
        case = json.load(f)
    a_t = np.array(case["a_t"], np.float32)[None, :, None, :]
    a_d = np.array(case["a_d"], np.float32)[None, :, None, :]
    mp, ov = run_both(a_d, a_t, case["k"])
    np.testing.assert_array_equal(mp, case["map"])
    np.testing.assert_array_equal(ov, case["overlap"])


@pytest.mark.parametrize("S,Hd,Ht,R,N,k", [(3, 4, 6, 5, 40, 7), (2, 16, 32, 8, 1000, 100), (1, 2, 3, 1, 9, 20),
                                           (2, 3, 5, 4, 5000, 1)])
def test_headmap_random_traces(S, Hd, Ht, R, N, k):
    rng = np.random.default_rng(S * 100 + N)
    a_d = rng.random((S, Hd, R, N), dtype=np.float32)
    a_t = rng.random((S, Ht, R, N), dtype=np.float32)
    run_both(a_d, a_t, k)


@pytest.mark.parametrize("S,Hd,Ht,R,N,k", [
    (1, 8, 32, 16, 16384, 64),     # 128 draft rows go through the many-workgroup pipeline, 512 target rows one workgroup each
    (1, 4, 8, 4, 40000, 100),      # rows longer than one workgroup's LDS: pipeline for both traces
    (1, 2, 3, 6, 65536, 200),      # small budget on long rows: chunk-local top-k + pool
])
def test_headmap_rows_that_take_the_other_selection_paths(S, Hd, Ht, R, N, k):
    rng = np.random.default_rng(N + k)
    a_d = rng.random((S, Hd, R, N), dtype=np.float32)
    a_t = a_d[:, rng.integers(0, Hd, Ht)] * rng.random((S, Ht, R, N), dtype=np.float32)
    run_both(a_d, a_t, k)


def test_headmap_ties_and_planted_permutation():
    rng = np.random.default_rng(5)
    S, Hd, R, N, k = 2, 5, 4, 256, 16
    a_d = (rng.integers(0, 8, (S, Hd, R, N)) / 8.0).astype(np.float32)      # heavy ties
    src = np.array([3, 3, 0, 4, 1, 2, 2, 0])
    a_t = a_d[:, src].copy()
    mp, _ = run_both(a_d, a_t, k)
    # identical traces: every target head finds its source (or an earlier draft head that ties)
    for t, s_ in enumerate(src):
        assert mp[t] <= s_


def test_headmap_from_attention_traces_of_the_kernels():
    """End to end on self-generated traces: dense attention dumps the scaled logits of a
    'draft' and a 'target' whose heads are noisy copies of the draft's; softmax rows are the
    traces; the mapping recovers which draft head each target head was copied from."""
    g = torch.Generator().manual_seed(0)
    S, Hd, R, N, d = 2, 4, 8, 512, 64
    src = [2, 0, 3, 3, 1, 0, 2, 1]
    qd = torch.randn(S, R, Hd, d, generator=g)
    kd = torch.randn(S, Hd, N, d, generator=g)
    qt = qd[:, :, src] + 0.1 * torch.randn(S, R, len(src), d, generator=g)
    kt = kd[:, src] + 0.1 * torch.randn(S, len(src), N, d, generator=g)
    vz = torch.zeros(S, Hd, N, d)
    traces = []
    for q, k in ((qd, kd), (qt, kt)):
        H = q.shape[2]
        _, _, logits = sts.sts_dense_attn(q.to(torch.bfloat16).to(DEV), k.to(torch.bfloat16).to(DEV),
                                          torch.zeros(S, H, N, d, dtype=torch.bfloat16, device=DEV), 0.3,
                                          want_logits=True)
        traces.append(torch.softmax(logits, dim=-1).contiguous())          # [S,H,R,N]
    mp, ov = sts.sts_head_map(traces[0], traces[1], 32)
    torch.cuda.synchronize()
    o_mp, o_ov = oracle.head_mapping(traces[0].cpu().numpy(), traces[1].cpu().numpy(), 32)
    np.testing.assert_array_equal(mp.cpu().numpy(), o_mp)
    np.testing.assert_array_equal(ov.cpu().numpy(), o_ov)
    assert mp.cpu().tolist() == src
