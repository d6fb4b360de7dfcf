"""GPU parity: sts_sparse_attn / sts_dense_attn (through the C ABI) against the CPU oracle."""
import math

import numpy as np
import pytest
import torch

import paper_2605_15508_amd as sts
from gpu_util import check_attn, check_logits, oracle_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_qkv(seed, B, Tq, Hq, Hkv, d, N, kv_std=0.5):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Tq, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, N, d, generator=g) * kv_std).to(torch.bfloat16)
    v = (torch.randn(B, Hkv, N, d, generator=g) * kv_std).to(torch.bfloat16)
    return q.to(DEV), k.to(DEV), v.to(DEV)


def make_indices(seed, B, Hq, N, kk, head_map=None):
    rng = np.random.default_rng(seed)
    idx = np.empty((B, Hq, kk), np.int32)
    for b in range(B):
        rows = {}
        for t in range(Hq):
            key = t if head_map is None else int(head_map[t])
            if key not in rows:
                rows[key] = np.sort(rng.choice(N, kk, replace=False))
            idx[b, t] = rows[key]
    return torch.from_numpy(idx).to(DEV)


@pytest.mark.parametrize("B,Tq,Hq,Hkv,d,N", [
    (2, 5, 8, 2, 128, 1000),     # GQA 4, several tiles, ragged tail
    (1, 1, 4, 4, 128, 37),       # MHA, single query row, less than two tiles
    (1, 8, 16, 2, 128, 2500),    # GQA 8 x 8 rows = 64 query rows (4 query tiles)
    (2, 5, 8, 2, 64, 777),       # head dim 64
    (1, 16, 4, 2, 128, 300),     # 16 query rows per head
    (1, 3, 6, 2, 64, 31),        # GQA 3, less than one tile
])
def test_dense_matches_oracle(B, Tq, Hq, Hkv, d, N):
    q, k, v = make_qkv(1, B, Tq, Hq, Hkv, d, N)
    scale = 1.0 / math.sqrt(d)
    out, lse, _ = sts.sts_dense_attn(q, k, v, scale, out_dtype=torch.float32)
    ref = oracle_attn(q, k, v, scale)
    check_attn(out, lse, ref, what="dense f32")
    out16, lse16, _ = sts.sts_dense_attn(q, k, v, scale)
    assert out16.dtype == torch.bfloat16
    check_attn(out16, lse16, ref, what="dense bf16")


@pytest.mark.parametrize("B,Tq,Hq,Hkv,d,N,kk,shared", [
    (2, 5, 8, 2, 128, 1000, 100, 2),    # pairs of heads share a draft head
    (1, 5, 8, 2, 128, 1000, 333, 1),    # every head on its own
    (1, 5, 8, 2, 128, 1000, 45, 4),     # whole KV group shares (20 rows, 2 query tiles)
    (1, 8, 16, 2, 128, 3000, 700, 2),   # 16 rows per unit
    (2, 5, 8, 2, 64, 512, 64, 2),       # head dim 64
    (1, 1, 4, 2, 128, 64, 1, 1),        # a single key per head
    (1, 5, 8, 1, 128, 600, 77, 8),      # 8 heads x 5 rows = 40 rows (4 query tiles)
])
def test_sparse_matches_oracle(B, Tq, Hq, Hkv, d, N, kk, shared):
    q, k, v = make_qkv(2, B, Tq, Hq, Hkv, d, N)
    head_map = [t // shared for t in range(Hq)]
    idx = make_indices(3, B, Hq, N, kk, head_map)
    scale = 1.0 / math.sqrt(d)
    ref = oracle_attn(q, k, v, scale, idx)
    out, lse = sts.sts_sparse_attn(q, k, v, idx, scale, head_map=head_map, out_dtype=torch.float32)
    check_attn(out, lse, ref, what="sparse hinted")
    # without the hint every head is processed alone: same answer
    out2, lse2 = sts.sts_sparse_attn(q, k, v, idx, scale, out_dtype=torch.float32)
    check_attn(out2, lse2, ref, what="sparse unhinted")


def test_sparse_scattered_head_map_and_counts():
    B, Tq, Hq, Hkv, d, N, kk = 2, 5, 16, 2, 128, 2000, 150
    q, k, v = make_qkv(4, B, Tq, Hq, Hkv, d, N)
    rng = np.random.default_rng(0)
    head_map = rng.integers(0, 5, size=Hq).tolist()        # sets are not contiguous head ranges
    idx = make_indices(5, B, Hq, N, kk, head_map)
    by_key = {}
    counts = np.empty((B, Hq), np.int32)
    for b in range(B):
        for t in range(Hq):
            counts[b, t] = by_key.setdefault((b, head_map[t]), int(rng.integers(0, kk + 1)))
    counts[0, [t for t in range(Hq) if head_map[t] == head_map[0]]] = 0      # an empty row
    counts_d = torch.from_numpy(counts).to(DEV)
    # entries past the count are padding (-1) and must never be read as rows
    idx_pad = idx.clone()
    for b in range(B):
        for t in range(Hq):
            idx_pad[b, t, counts[b, t]:] = -1
    ref = oracle_attn(q, k, v, 0.09, idx, counts_d)
    out, lse = sts.sts_sparse_attn(q, k, v, idx_pad, 0.09, counts=counts_d, head_map=head_map,
                                   out_dtype=torch.float32)
    check_attn(out, lse, ref, what="scattered map + counts")
    empty = counts == 0
    assert (out.cpu().numpy().transpose(0, 2, 1, 3)[empty] == 0).all()


def test_full_budget_equals_dense_kernel():
    B, Tq, Hq, Hkv, d, N = 1, 5, 8, 2, 128, 500
    q, k, v = make_qkv(6, B, Tq, Hq, Hkv, d, N)
    idx = torch.arange(N, dtype=torch.int32, device=DEV).expand(B, Hq, N).contiguous()
    o_s, l_s = sts.sts_sparse_attn(q, k, v, idx, 0.1, head_map=[0] * Hq, out_dtype=torch.float32)
    o_d, l_d, _ = sts.sts_dense_attn(q, k, v, 0.1, out_dtype=torch.float32)
    ref = oracle_attn(q, k, v, 0.1)
    check_attn(o_s, l_s, ref, what="k = N sparse")
    check_attn(o_d, l_d, ref, what="dense")
    assert (o_s - o_d).abs().max().item() < 1e-5


def test_dense_seq_lens_strided_cache_and_logits():
    B, Tq, Hq, Hkv, d, N = 3, 5, 8, 2, 128, 640
    q, k, v = make_qkv(7, B, Tq, Hq, Hkv, d, N)
    kv = torch.stack([k, v], dim=3).contiguous()       # interleaved cache [B,Hkv,N,2,d]
    ks, vs = kv[:, :, :, 0], kv[:, :, :, 1]
    lens = torch.tensor([640, 129, 0], dtype=torch.int32, device=DEV)
    out, lse, logits = sts.sts_dense_attn(q, ks, vs, 0.09, seq_lens=lens, out_dtype=torch.float32,
                                          want_logits=True)
    ref = oracle_attn(q, k, v, 0.09, seq_lens=lens, want_logits=True)
    check_attn(out, lse, ref, what="dense seq_lens strided")
    lg, rl = logits.cpu().numpy(), ref["logits"]
    for b, n in enumerate(lens.tolist()):
        check_logits(lg[b, :, :, :n], rl[b, :, :, :n], what=f"batch {b}")
    assert (out[2] == 0).all() and torch.isneginf(lse[2]).all()


def test_logits_dump_head_dim_64_unaligned_n():
    B, Tq, Hq, Hkv, d, N = 1, 8, 8, 2, 64, 301       # N % 4 != 0: scalar store path
    q, k, v = make_qkv(8, B, Tq, Hq, Hkv, d, N)
    out, lse, logits = sts.sts_dense_attn(q, k, v, 0.125, out_dtype=torch.float32, want_logits=True)
    ref = oracle_attn(q, k, v, 0.125, want_logits=True)
    check_attn(out, lse, ref, what="dense d64 logits")
    check_logits(logits.cpu().numpy(), ref["logits"])


@pytest.mark.parametrize("d,N", [(128, 640), (64, 301), (128, 4099)])
def test_logits_dump_in_bf16(d, N):
    """The dump rounded to bf16 (Section 5 names no type for it): equal, bit for bit, to the fp32
    dump rounded to nearest even, and within one bf16 unit of the oracle's logits; sentinels
    planted beyond the valid length stay untouched."""
    B, Tq, Hq, Hkv = 2, 5, 8, 2
    q, k, v = make_qkv(31, B, Tq, Hq, Hkv, d, N)
    lens = torch.tensor([N, N // 3], dtype=torch.int32, device=DEV)
    out32, lse32, lg32 = sts.sts_dense_attn(q, k, v, 0.09, seq_lens=lens, out_dtype=torch.float32, want_logits=True)
    dump = torch.full((B, Hq, Tq, N), 7.0, dtype=torch.bfloat16, device=DEV)
    out16, lse16, lg16 = sts.sts_dense_attn(q, k, v, 0.09, seq_lens=lens, out_dtype=torch.float32, logits_out=dump)
    assert lg16 is dump and torch.equal(out16, out32) and torch.equal(lse16, lse32)
    ref = oracle_attn(q, k, v, 0.09, seq_lens=lens, want_logits=True)["logits"]
    for b, n in enumerate(lens.tolist()):
        assert torch.equal(lg16[b, :, :, :n], lg32[b, :, :, :n].to(torch.bfloat16))
        assert (lg16[b, :, :, n:] == 7.0).all()
        got = lg16[b, :, :, :n].float().cpu().numpy()
        assert (np.abs(got - ref[b, :, :, :n]) <= np.abs(ref[b, :, :, :n]) * 2.0 ** -7 + 1e-6).all()


@pytest.mark.parametrize("Tq,G,dump", [(8, 8, torch.float32), (5, 8, torch.bfloat16), (16, 4, torch.float32)])
def test_logits_dump_head_dim_128_group_of_more_than_32_rows(Tq, G, dump):
    """A KV group with more than 32 query rows at head size 128: the dump serves it with two units
    of at most two query tiles each (both read K and V); outputs, LSE and logits as for any shape.
    The attention without the dump takes the group as one unit of four query tiles."""
    B, Hkv, d, N = 2, 2, 128, 1500
    q, k, v = make_qkv(Tq * G, B, Tq, Hkv * G, Hkv, d, N)
    lens = torch.tensor([N, 700], dtype=torch.int32, device=DEV)
    out, lse, logits = sts.sts_dense_attn(q, k, v, 0.09, seq_lens=lens, out_dtype=torch.float32, want_logits=dump)
    ref = oracle_attn(q, k, v, 0.09, seq_lens=lens, want_logits=True)
    check_attn(out, lse, ref, what="dense d128, more than 32 rows per group, with the dump")
    lg, rl = logits.float().cpu().numpy(), ref["logits"]
    for b, n in enumerate(lens.tolist()):
        if dump == torch.float32:
            check_logits(lg[b, :, :, :n], rl[b, :, :, :n], what=f"batch {b}")
        else:
            assert (np.abs(lg[b, :, :, :n] - rl[b, :, :, :n]) <= np.abs(rl[b, :, :, :n]) * 2.0 ** -7 + 1e-6).all()
    out2, lse2, _ = sts.sts_dense_attn(q, k, v, 0.09, seq_lens=lens, out_dtype=torch.float32)
    check_attn(out2, lse2, ref, what="dense d128, four query tiles")
    # the gather with four query tiles: every head of the group shares one list
    idx = torch.arange(0, 1400, 2, dtype=torch.int32, device=DEV).expand(B, Hkv * G, 700).contiguous()
    o_s, l_s = sts.sts_sparse_attn(q, k, v, idx, 0.09, head_map=[0] * (Hkv * G), out_dtype=torch.float32)
    ref_s = oracle_attn(q, k, v, 0.09, indices=idx)
    check_attn(o_s, l_s, ref_s, what="gather d128, four query tiles")


def test_results_are_deterministic_run_to_run():
    B, Tq, Hq, Hkv, d, N, kk = 2, 5, 8, 2, 128, 4000, 400
    q, k, v = make_qkv(9, B, Tq, Hq, Hkv, d, N)
    hm = [t // 2 for t in range(Hq)]
    idx = make_indices(10, B, Hq, N, kk, hm)
    a, la = sts.sts_sparse_attn(q, k, v, idx, 0.09, head_map=hm, out_dtype=torch.float32)
    a, la = a.clone(), la.clone()
    b, lb = sts.sts_sparse_attn(q, k, v, idx, 0.09, head_map=hm, out_dtype=torch.float32)
    assert torch.equal(a, b) and torch.equal(la, lb)


def test_out_of_range_indices_are_clamped_not_faulting():
    B, Tq, Hq, Hkv, d, N, kk = 1, 5, 4, 2, 128, 100, 10
    q, k, v = make_qkv(11, B, Tq, Hq, Hkv, d, N)
    idx = make_indices(12, B, Hq, N, kk)
    bad = idx.clone()
    bad[0, 0, 0] = -5
    bad[0, 1, 3] = 10 ** 6
    out, _ = sts.sts_sparse_attn(q, k, v, bad, 0.09, out_dtype=torch.float32)
    torch.cuda.synchronize()
    fixed = idx.clone()
    fixed[0, 0, 0] = 0
    fixed[0, 1, 3] = N - 1
    ref = oracle_attn(q, k, v, 0.09, fixed)
    assert np.abs(out.cpu().numpy() - ref["out"]).max() < 1e-2


def test_empty_batch_and_workspace_errors():
    q, k, v = make_qkv(13, 1, 5, 8, 2, 128, 256)
    tiny = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(sts.StsError):
        sts.sts_dense_attn(q, k, v, 0.09, workspace=tiny)
    q0 = q[:0].contiguous()
    out, lse, _ = sts.sts_dense_attn(q0, k[:0].contiguous(), v[:0].contiguous(), 0.09)
    assert out.shape[0] == 0


def test_maximum_head_counts_and_group_size():
    """The largest shapes the tables carry: 256 query heads, 16 query heads per KV head,
    16 query rows; sets wider than 64 query rows are split into several units."""
    B, Tq, Hq, Hkv, d, N, kk = 1, 16, 256, 16, 64, 200, 24
    q, k, v = make_qkv(21, B, Tq, Hq, Hkv, d, N)
    hm = [t // 16 for t in range(Hq)]                 # the whole KV group shares one draft head: 256 rows per set
    idx = make_indices(22, B, Hq, N, kk, hm)
    ref = oracle_attn(q, k, v, 0.125, idx)
    out, lse = sts.sts_sparse_attn(q, k, v, idx, 0.125, head_map=hm, out_dtype=torch.float32)
    check_attn(out, lse, ref, what="Hq 256 / G 16 sparse")
    dref = oracle_attn(q, k, v, 0.125)
    dout, dlse, _ = sts.sts_dense_attn(q, k, v, 0.125, out_dtype=torch.float32)
    check_attn(dout, dlse, dref, what="Hq 256 / G 16 dense")
    plan = sts.attn_plan(q, k, True, kmax=kk, head_map=hm)
    assert plan["query_tiles"] == 4 and plan["units_per_batch"] == 16 * 4     # 16 heads x 16 rows -> 4 units of 64 rows
    # the same shape through the second pass over K (four sets of four heads per KV head)
    A = torch.empty(B, Hq, N, dtype=torch.float32, device=DEV)
    _, lse2, logits = sts.sts_dense_attn(q, k, v, 0.125, want_logits=True, weights_sum_out=A)
    _, _, agg = sts.sts_select(logits, list(range(Hq)), kk, lse=lse2, kind=sts.STS_SCORES_LOGITS_LSE, want_agg=True)
    assert torch.equal(A, agg)


def test_layers_read_their_slice_of_one_selection():
    """Several target layers whose heads map to the same draft heads: one sts_select over all
    their heads (the scores are aggregated and ranked once), then every layer's attention reads
    its own slice [:, l*Hq:(l+1)*Hq, :] of the index lists in place (batch stride wider than
    Hq*kmax), against the oracle on contiguous copies."""
    import oracle
    L, B, Tq, Hq, Hkv, Hd, d, N, k = 3, 2, 5, 8, 2, 4, 128, 3000, 300
    g = torch.Generator().manual_seed(77)
    scores = torch.softmax(torch.randn(B, Hd, Tq, N, generator=g) * 2, dim=-1)
    hm_all = [int(x) for x in torch.randint(0, Hd, (L * Hq,), generator=g)]
    kh = [300, 120, 300, 7]
    idx_all, cnt_all, _ = sts.sts_select(scores.to(DEV), hm_all, k, k_head=kh)
    o_idx, o_cnt, _ = oracle.select_indices(scores.numpy(), np.asarray(hm_all, np.int32), k, k_head=kh)
    np.testing.assert_array_equal(idx_all.cpu().numpy(), o_idx)
    for l in range(L):
        q, kc, vc = make_qkv(100 + l, B, Tq, Hq, Hkv, d, N)
        sl = slice(l * Hq, (l + 1) * Hq)
        idx_l, cnt_l = idx_all[:, sl], cnt_all[:, sl]
        assert not idx_l.is_contiguous()
        out, lse = sts.sts_sparse_attn(q, kc, vc, idx_l, 0.09, counts=cnt_l, head_map=hm_all[sl],
                                       out_dtype=torch.float32)
        ref = oracle_attn(q, kc, vc, 0.09, idx_l.contiguous(), cnt_l.contiguous())
        check_attn(out, lse, ref, what=f"layer {l} slice")


def test_closed_forms_on_the_gpu():
    """Values fixed by the mathematics alone, without the oracle: zero queries give the plain
    mean of the gathered value rows and LSE = ln(count); constant values come back unchanged."""
    B, Tq, Hq, Hkv, d, N, kk = 2, 5, 8, 2, 128, 5000, 777
    q, k, v = make_qkv(5, B, Tq, Hq, Hkv, d, N)
    hm = [t // 2 for t in range(Hq)]
    idx = make_indices(6, B, Hq, N, kk, head_map=hm)
    cnt = torch.full((B, Hq), kk, dtype=torch.int32, device=DEV)
    cnt[0, 2:4] = 100                                        # heads 2 and 3 share a row: same count
    out, lse = sts.sts_sparse_attn(torch.zeros_like(q), k, v, idx, 0.09, counts=cnt, head_map=hm,
                                   out_dtype=torch.float32)
    G = Hq // Hkv
    for b in range(B):
        for t in range(Hq):
            c = int(cnt[b, t])
            rows = v[b, t // G][idx[b, t, :c].long()].float()            # [c, d]
            want = rows.mean(dim=0)
            assert (out[b, :, t] - want[None]).abs().max().item() < 2e-3  # P is rounded to bf16 before P.V
            assert (lse[b, t] - math.log(c)).abs().max().item() < 1e-5
    vc = torch.full_like(v, 0.75)
    out, _ = sts.sts_sparse_attn(q, k, vc, idx, 0.09, counts=cnt, head_map=hm, out_dtype=torch.float32)
    assert (out - 0.75).abs().max().item() < 4e-3
    out, lse, _ = sts.sts_dense_attn(torch.zeros_like(q), k, v, 0.09, out_dtype=torch.float32)
    want = v.float().mean(dim=2)                                          # [B,Hkv,d]
    for t in range(Hq):
        assert (out[:, :, t] - want[:, t // G][:, None]).abs().max().item() < 2e-3
    assert (lse - math.log(N)).abs().max().item() < 1e-5


@pytest.mark.parametrize("B,Tq,Hq,Hkv,d,N", [
    (2, 5, 8, 2, 128, 1000),     # 20 rows per KV head: two query tiles, ragged last key tile
    (1, 8, 16, 2, 128, 2500),    # GQA 8 x 8 rows: four query tiles
    (2, 8, 8, 2, 64, 4100),      # head dim 64; several key-range pieces
    (1, 16, 16, 1, 64, 644),     # 16 heads x 16 rows: the heads of a KV group in four sets
    (1, 1, 4, 4, 128, 36),       # one query row: the sum is the row itself
    (1, 3, 6, 2, 64, 21),        # less than one key tile
    (2, 2, 12, 2, 64, 333),      # two rows per head: two heads per lane
    (1, 16, 6, 1, 128, 200),     # 6 heads x 16 rows: a full set of four heads and a set of two
    (1, 4, 20, 2, 128, 515),     # 10 heads x 4 rows per KV head: one head per lane
    (1, 7, 12, 1, 64, 1030),     # 12 heads x 7 rows (padded to 8): sets of 8 and 4 heads
])
def test_weights_summed_over_the_query_block(B, Tq, Hq, Hkv, d, N):
    """The second pass over K (Section 4.3: one mask per speculative batch; Section 5: the draft
    layer hands over its scores): equal, bit for bit, to what the selection aggregates the logits
    dump to, equal to the oracle's aggregate within the dump's tolerance, zero past the valid
    length, and the selection it feeds picks the same indices."""
    import oracle
    q, k, v = make_qkv(41, B, Tq, Hq, Hkv, d, N)
    lens = torch.tensor([N - 7, N // 3][:B], dtype=torch.int32, device=DEV)
    scale = 1.0 / math.sqrt(d)
    A = torch.full((B, Hq, N), 9.0, dtype=torch.float32, device=DEV)
    out, lse, logits = sts.sts_dense_attn(q, k, v, scale, seq_lens=lens, out_dtype=torch.float32,
                                          want_logits=True, weights_sum_out=A)
    out0, lse0, lg0 = sts.sts_dense_attn(q, k, v, scale, seq_lens=lens, out_dtype=torch.float32, want_logits=True)
    assert torch.equal(out, out0) and torch.equal(lse, lse0)      # the second pass leaves the first alone
    kk = max(1, N // 10)
    hm = list(range(Hq))
    idx_d, cnt_d, agg_d = sts.sts_select(logits, hm, kk, lse=lse, seq_lens=lens,
                                         kind=sts.STS_SCORES_LOGITS_LSE, want_agg=True)
    idx_a, cnt_a, _ = sts.sts_select(A.view(B, Hq, 1, N), hm, kk, seq_lens=lens)
    assert torch.equal(idx_a, idx_d) and torch.equal(cnt_a, cnt_d)
    ref = oracle_attn(q, k, v, scale, seq_lens=lens, want_logits=True)
    ref_A = oracle.aggregate(ref["logits"], ref["lse"], kind=oracle.LOGITS_LSE)
    got = A.cpu().numpy()
    for b, n in enumerate(lens.tolist()):
        assert torch.equal(A[b, :, :n], agg_d[b, :, :n])
        assert (A[b, :, n:] == 0).all()
        assert (np.abs(got[b, :, :n] - ref_A[b, :, :n]) <= 3e-5 * ref_A[b, :, :n] + 1e-10).all()
        # each row's weights sum to one, so the aggregate sums to Tq
        assert np.allclose(got[b, :, :n].sum(-1, dtype=np.float64), Tq, atol=2e-3)
    # without a caller's lse buffer the normalisers live in the workspace (no dump: the first
    # pass visits the tiles in another order, so its normalisers differ in the last bits)
    A2 = torch.empty_like(A)
    sts.sts_dense_attn(q, k, v, scale, seq_lens=lens, want_lse=False, weights_sum_out=A2)
    assert torch.allclose(A2, A, rtol=1e-4, atol=1e-9)


def test_weights_sum_unaligned_length_and_rejections():
    """A length that is no multiple of 4 (scalar tail of the dump, partial last line of the sum),
    and the cases the second pass does not cover: the speculative block's own keys, paged caches."""
    q, k, v = make_qkv(42, 1, 4, 4, 2, 128, 131)
    A = torch.empty(1, 4, 131, dtype=torch.float32, device=DEV)
    _, lse, logits = sts.sts_dense_attn(q, k, v, 0.1, want_logits=True, weights_sum_out=A)
    _, _, agg = sts.sts_select(logits, [0, 1, 2, 3], 13, lse=lse, kind=sts.STS_SCORES_LOGITS_LSE, want_agg=True)
    assert torch.equal(A, agg)
    kn = torch.zeros(1, 4, 2, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(RuntimeError):
        sts.sts_dense_attn(q, k, v, 0.1, k_new=kn, v_new=kn, weights_sum_out=A)
