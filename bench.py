#!/usr/bin/env python3
"""Benchmark of the STS hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input, all of it
resident in HBM before the timed region: sts_select (draft scores -> index sets),
sts_sparse_attn (verification attention over the gathered rows) and sts_dense_attn (the
same-family dense baseline on the same inputs). The headline value is the sparse
verification attention time per layer; selection and dense times, the speedup over dense and
the achieved HBM bandwidth on gathered KV bytes are reported beside it.

Prints ONE JSON line. `python bench.py` defaults to the 128K-context, batch-4, 10%-budget
configuration and finishes within a couple of minutes including the CPU-oracle baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "sparse verify-attn µs/layer + HBM GB/s at 90% sparsity, 128K ctx, vs dense"
HBM_PEAK_GBS = 8000.0
STS_PROF_BUDGET = 4096      # launches the library's event pool keeps per reset


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--budget", type=float, default=None, help="fraction of N kept per head")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="leave the dense baseline out of the step")
    ap.add_argument("--seed", type=int, default=20251127)
    ap.add_argument("--page-size", type=int, default=1,
                    help="selection / attention granularity in tokens (1 = token-wise, 8 = the paper's p_s=8)")
    ap.add_argument("--paged", action="store_true",
                    help="keep K/V in a pool of pages behind a random page table (needs --page-size)")
    ap.add_argument("--warm", action="store_true",
                    help="reuse one KV buffer even when it fits the 256 MB Infinity Cache (default: rotate over "
                         "enough distinct layers to exceed 2 GiB so that every pass starts cache-cold)")
    ap.add_argument("--gain", type=float, default=None,
                    help="strength of the planted keys (default: the configuration's, 3.0)")
    ap.add_argument("--head-map", default="default", choices=["default", "random"],
                    help="target head -> draft head: t*Hd//Hq, or a seeded random map (robustness point)")
    ap.add_argument("--positions", default="scattered", choices=["scattered", "recent"],
                    help="heavy tokens scattered over the context (worst case for the gather) or clustered at its end")
    ap.add_argument("--scores", default="fp32", choices=["fp32", "bf16"],
                    help="type of the draft scores read by sts_select (and of the logits dump of the draft layer)")
    ap.add_argument("--draft-heads", type=int, default=None,
                    help="number of draft heads Hd (default: the configuration's); fewer draft heads make more "
                         "target heads of a KV group share one index row")
    ap.add_argument("--draft-scores", default="dump", choices=["dump", "sum"],
                    help="draft-layer configuration: the draft attention dumps its logits and sts_select aggregates "
                         "them (dump), or it sums the attention weights over the query block itself in a second "
                         "pass over K and sts_select ranks that aggregate (sum)")
    ap.add_argument("--fused-tail", action="store_true",
                    help="also pass the speculative block's own keys/values (k_new, v_new) to the attention calls, "
                         "which then append them causally in their final merge")
    ap.add_argument("--prefill-blocks", type=int, default=0,
                    help="other mode: chunked sparse prefill, this many 16-row query blocks over ONE shared cache "
                         "of the configuration's context (batch 1), each block with its own mask; prints its own JSON line")
    ap.add_argument("--prefill-masks", default="block", choices=["block", "rows"],
                    help="with --prefill-blocks: one mask per 16-row block (from the rows' summed scores), or one per "
                         "query row, gathered once per block as the union of the rows' sets (row bits)")
    ap.add_argument("--headmap", action="store_true",
                    help="other mode: offline head-mapping construction (Algorithm 1) on synthetic traces; prints its own JSON line")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the budget sweep, the paper's budgets, the 32K point and the graph-replayed figures")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (scales rocprofv3 --pmc byte counters)")
    return ap.parse_args()


def read_traffic(kernel: str, workload: str, version: int):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    (profiles/traffic_<kernel>_<workload>.txt: `hbm_bytes_per_launch: <int>`, taken with the library
    whose `library_version: <int>` the file states). None when the file belongs to another version of
    the library: a counter reading says nothing about kernels that have changed since."""
    path = os.path.join(ROOT, "profiles", f"traffic_{kernel}_{workload}.txt")
    vals = {}
    try:
        with open(path) as f:
            for line in f:
                for key in ("hbm_bytes_per_launch", "library_version", "kernel_avg_us"):
                    if line.startswith(key + ":"):
                        vals[key] = float(line.split(":", 1)[1])
    except OSError:
        return None
    if "hbm_bytes_per_launch" not in vals or int(vals.get("library_version", -1)) != version:
        return None
    return int(vals["hbm_bytes_per_launch"])


def cpu_baseline(w, idx, cnt, out_s, page=1, budget_s=25.0, scores=None, lse=None):
    """Time the CPU oracle (as it stands, untuned) on this machine's host cores on a bounded sample
    of the same workload, and compare what it computes with what the GPU computed (outside any
    timed region). Returns (cpu_baseline object, parity object)."""
    import numpy as np

    import oracle

    cfg = w.cfg
    threads = oracle.num_threads()
    qb = oracle.bf16_bits(w.q.cpu())
    # sample: as many whole batch elements as fit the time budget, estimated from one head
    kb = oracle.bf16_bits(w.k[:1].cpu())
    vb = oracle.bf16_bits(w.v[:1].cpu())
    def tokens(i, c):
        # the oracle attends over token ids: expand block ids when the selection is block-wise
        i, c = i.cpu().numpy(), c.cpu().numpy()
        return oracle.expand_blocks(i, c, page, cfg.N) if page > 1 else (i, c)

    idx0, cnt0 = tokens(idx[:1], cnt[:1])
    t0 = time.perf_counter()
    oracle.attn(qb[:1], kb, vb, w.scale, idx0, cnt0, heads=range(0, min(threads, cfg.Hq)))
    probe = time.perf_counter() - t0
    per_batch = probe * cfg.Hq / min(threads, cfg.Hq)
    nb = int(max(1, min(cfg.B, budget_s // max(per_batch, 1e-3))))
    kb = oracle.bf16_bits(w.k[:nb].cpu())
    vb = oracle.bf16_bits(w.v[:nb].cpu())
    idxn, cntn = tokens(idx[:nb], cnt[:nb])
    best = float("inf")
    ref = None
    for _ in range(2):
        t0 = time.perf_counter()
        ref = oracle.attn(qb[:nb], kb, vb, w.scale, idxn, cntn)
        best = min(best, time.perf_counter() - t0)
    sparse_us_layer = best / nb * cfg.B * 1e6
    # selection on one batch element
    # (the draft-layer configuration selects from the scaled logits + LSE the GPU just dumped)
    src = w.scores if scores is None else scores
    sc = src[:1].float().cpu().numpy()       # bf16 scores are widened exactly, as the library does
    ls = None if lse is None else lse[:1].cpu().numpy()
    t0 = time.perf_counter()
    o_idx, o_cnt, _ = oracle.select_indices(sc, w.head_map.numpy(), idx.shape[2], page=page, lse=ls,
                                            kind=oracle.PROBS if ls is None else oracle.LOGITS_LSE)
    sel_us_layer = (time.perf_counter() - t0) * cfg.B * 1e6
    # dense on one KV group of batch 0 (extrapolated linearly)
    G = cfg.Hq // cfg.Hkv
    t0 = time.perf_counter()
    oracle.attn(qb[:1], kb[:1], vb[:1], w.scale, heads=range(0, G))
    dense_us_layer = (time.perf_counter() - t0) * cfg.Hkv * cfg.B * 1e6
    # parity of this very run: the GPU's index sets against the oracle's on the batch element the
    # oracle ranked, the GPU's sparse outputs against the oracle's on every batch element it computed
    # (the oracle attended over the GPU's index lists, so the two comparisons are independent)
    err = np.abs(out_s[:nb].float().cpu().numpy() - ref["out"])
    rms = float(np.sqrt(np.mean(ref["out"].astype(np.float64) ** 2)))
    exact_select = ls is None       # with scaled-logit input the device exponential differs from libm in the last bits
    same_idx = bool(np.array_equal(idx[:1].cpu().numpy(), o_idx) and np.array_equal(cnt[:1].cpu().numpy(), o_cnt))
    parity = {
        "index_sets_equal": same_idx if exact_select else None,
        "index_sets_checked": (f"batch element 0, all {cfg.Hq} heads, k={idx.shape[2]}" if exact_select else
                               "not compared here: logits input (checked stage-wise in the GPU tests)"),
        "out_max_abs_err": float(err.max()), "out_mean_abs_err": float(err.mean()), "out_rms": rms,
        "out_checked": f"sts_sparse_attn, {nb} of {cfg.B} batch elements, all heads and query rows",
        "tolerance": {"max_abs": 1e-2, "mean_abs": 1e-3},
        "ok": bool((same_idx or not exact_select) and err.max() <= 1e-2 and err.mean() <= 1e-3),
    }
    base = {
        "value": round(sparse_us_layer, 1), "unit": "us/layer", "cores": threads, "kind": "oracle",
        "sample": (f"sts_sparse_attn oracle on {nb} of {cfg.B} batch elements (all {cfg.Hq} heads, "
                   f"k={idx.shape[2]}{' blocks of %d' % page if page > 1 else ''}), best of 2, scaled to the batch; select timed on 1 batch element, "
                   f"dense on 1 KV group of 1 batch element, both scaled linearly"),
        "select_us_layer": round(sel_us_layer, 1),
        "dense_us_layer_extrapolated": round(dense_us_layer, 1),
    }
    return base, parity


def _timed(fn, steps, warmup, torch):
    """Median / mean of `steps` event-timed calls of fn() on the current stream, microseconds."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    xs = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    return {"median": round(statistics.median(xs), 2), "mean": round(statistics.fmean(xs), 2),
            "min": round(xs[0], 2), "p90": round(xs[min(len(xs) - 1, int(0.9 * len(xs)))], 2)}


def run_prefill(args, torch, sts):
    """Chunked sparse prefill (2-D masks: one mask per block of 16 query rows and head). NB query
    blocks are one batch over a single shared cache (kv_stride_b = 0); block i sees the first
    N - 16*(NB-1-i) cached tokens and adds its own 16 tokens causally. Draft scores are bf16."""
    from dataclasses import replace

    from workload import CONFIGS, budget_tokens, make_workload
    dev = torch.device("cuda:0")
    cfg = replace(CONFIGS[args.config], B=1, Tq=16)
    NB, T = args.prefill_blocks, 16
    w = make_workload(cfg, seed=args.seed, device=dev, budget=args.budget, with_scores=False)
    N, Hq, Hkv, d, Hd = cfg.N, cfg.Hq, cfg.Hkv, cfg.d, cfg.Hd
    k = budget_tokens(cfg, args.budget)
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed + 17)
    q = torch.randn(NB, T, Hq, d, generator=gen, device=dev).to(torch.bfloat16)
    kn = (torch.randn(NB, T, Hkv, d, generator=gen, device=dev) * 0.5).to(torch.bfloat16)
    vn = (torch.randn(NB, T, Hkv, d, generator=gen, device=dev) * 0.5).to(torch.bfloat16)
    lens = (N - T * (NB - 1 - torch.arange(NB, device=dev))).to(torch.int32)
    scores = torch.empty(NB, Hd, T, N, dtype=torch.bfloat16, device=dev)
    for b in range(NB):      # softmax over the visible prefix, block by block: the rows of a block share the
        # block's logits up to noise (neighbouring query tokens attend to much the same keys; same
        # noise level as the draft scores of the configuration)
        lg = (torch.randn(Hd, 1, N, generator=gen, device=dev) * 2
              + torch.randn(Hd, T, N, generator=gen, device=dev) * cfg.noise)
        lg[:, :, int(lens[b]):] = float("-inf")
        scores[b] = torch.softmax(lg, dim=-1).to(torch.bfloat16)
        del lg
    kx, vx = w.k.expand(NB, Hkv, N, d), w.v.expand(NB, Hkv, N, d)
    out = torch.empty(NB, T, Hq, d, dtype=torch.bfloat16, device=dev)
    rows = args.prefill_masks == "rows"
    if rows:
        # a mask per query row (Section 4.2): per-row selection, union of a block's 16 row sets with
        # row bits, one gather of the union per block
        pitch = min(4 * k, T * k, N)    # the caller sizes the union's buffers; checked below that nothing was cut
        ridx = torch.empty(NB, Hd, T, k, dtype=torch.int32, device=dev)
        rcnt = torch.empty(NB, Hd, T, dtype=torch.int32, device=dev)
        idx = torch.empty(NB, Hq, pitch, dtype=torch.int32, device=dev)
        msk = torch.empty(NB, Hq, pitch, dtype=torch.int16, device=dev)
        cnt = torch.empty(NB, Hq, dtype=torch.int32, device=dev)
        def sel():
            sts.sts_select_rows(scores, k, seq_lens=lens, out=(ridx, rcnt))
            sts.sts_union_rows(ridx, rcnt, w.head_map, N, pitch=pitch, out=(idx, msk, cnt))
        att = lambda: sts.sts_sparse_attn(q, kx, vx, idx, w.scale, counts=cnt, head_map=w.head_map, out=out,
                                          want_lse=False, k_new=kn, v_new=vn, causal=True, row_mask=msk)
    else:
        idx = torch.empty(NB, Hq, k, dtype=torch.int32, device=dev)
        cnt = torch.empty(NB, Hq, dtype=torch.int32, device=dev)
        sel = lambda: sts.sts_select(scores, w.head_map, k, seq_lens=lens, out=(idx, cnt))
        att = lambda: sts.sts_sparse_attn(q, kx, vx, idx, w.scale, counts=cnt, head_map=w.head_map, out=out,
                                          want_lse=False, k_new=kn, v_new=vn, causal=True)
    t_sel = _timed(sel, args.steps, args.warmup, torch)
    if rows and int(cnt.max().item()) >= pitch:
        raise SystemExit("bench.py: the union of a block's row masks does not fit the pitch chosen for it")
    t_att = _timed(att, args.steps, args.warmup, torch)
    parts = {}
    if rows:      # the two steps of mask building on their own
        parts["select_rows_us"] = _timed(lambda: sts.sts_select_rows(scores, k, seq_lens=lens, out=(ridx, rcnt)),
                                         args.steps, args.warmup, torch)["median"]
        parts["union_rows_us"] = _timed(lambda: sts.sts_union_rows(ridx, rcnt, w.head_map, N, pitch=pitch, out=(idx, msk, cnt)),
                                        args.steps, args.warmup, torch)["median"]
    sts.prof_enable(True)
    sts.prof_reset()
    for _ in range(max(1, min(args.steps, 20))):
        att()
    torch.cuda.synchronize()
    prof = sts.prof_read()
    sts.prof_enable(False)
    split_us = prof["attn_sparse"][1] * 1e3 / max(prof["attn_sparse"][0], 1)
    plan = sts.attn_plan(q, torch.empty(NB, Hkv, N, d, device="meta"), True, kmax=idx.shape[2], head_map=w.head_map)
    row_bytes = 2 * d * 2
    units = plan["units_per_batch"]
    # the heads of a KV group that share a draft head form one unit and share one gathered list
    G, hm = Hq // Hkv, [int(x) for x in w.head_map]
    leaders, seen = [], set()
    for t in range(Hq):
        if (t // G, hm[t]) not in seen:
            seen.add((t // G, hm[t]))
            leaders.append(t)
    assert len(leaders) == units
    entries = int(cnt[:, leaders].sum().item()) if rows else NB * units * k       # gathered once per unit
    b_set = entries * row_bytes
    extra = dict(parts)
    if rows:
        # what one gather per query row (the single-row formulation) would move for the same masks
        per_row_entries = int(rcnt[:, [hm[t] for t in leaders]].sum().item())
        extra.update({"union_entries_per_block_and_unit": round(entries / (NB * units), 1),
                      "gathered_kv_bytes_one_gather_per_row": per_row_entries * row_bytes,
                      "union_saves": round(per_row_entries / max(entries, 1), 2)})
    print(json.dumps({
        "metric": "chunked sparse prefill: attention us per 16-token query block over a shared cache", "unit": "us/block",
        "value": round(t_att["median"] / NB, 2), "higher_is_better": False, "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
        "steps": args.steps, "warmup": args.warmup,
        "config": {"workload": f"{cfg.name} shape, one cache of N{N} Hq{Hq}/Hkv{Hkv} d{d}, {NB} blocks of {T} rows, "
                               f"budget {k} tokens per head and " + ("query row (a mask per row, gathered as the block's union)" if rows else "block")
                               + f", draft scores bf16 [{NB},{Hd},{T},{N}]", "masks": args.prefill_masks},
        "sparse_attn_us": t_att, "select_us": t_sel, "gathered_kv_bytes_b_set": b_set,
        "gathered_kv_gbs_b_set": round(b_set / (t_att["median"] * 1e-6) / 1e9, 1),
        "roofline": {"bound": "hbm", "kernel": "attn_split_kernel<sparse" + (", row bits>" if rows else ">"),
                     "achieved": round(b_set / (split_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(b_set / (split_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "avg_launch_us": round(split_us, 2),
                     "algorithmic_bytes_per_launch": b_set,
                     "note": "blocks gather overlapping rows of one cache, so part of the traffic is served by the caches"},
        "launch": plan, "library_version": sts.sts_version(), **extra}))


def run_headmap(args, torch, sts):
    """Algorithm 1 on synthetic attention-weight traces of both models (offline step)."""
    dev = torch.device("cuda:0")
    S, R, Hd, Ht, N, k = 2, 128, 16, 32, 32768, 512
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    a_d = torch.softmax(torch.randn(S, Hd, R, N, generator=gen, device=dev) * 2, dim=-1)
    # target heads follow a planted draft head plus noise, so the map has something to find
    planted = torch.randint(0, Hd, (Ht,), generator=gen, device=dev)
    a_t = torch.softmax(torch.log(a_d[:, planted]) + torch.randn(S, Ht, R, N, generator=gen, device=dev), dim=-1)
    res = {}
    fn = lambda: res.update(r=sts.sts_head_map(a_d, a_t, k))
    t = _timed(fn, max(3, min(args.steps, 10)), 2, torch)
    mp = res["r"][0].cpu()
    print(json.dumps({
        "metric": "offline head-mapping construction (Algorithm 1), ms per call", "unit": "ms", "value": round(t["median"] / 1e3, 3),
        "higher_is_better": False, "n_gpus": 1, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"traces a_d [{S},{Hd},{R},{N}] and a_t [{S},{Ht},{R},{N}] fp32, top-{k} per row"},
        "call_us": t, "planted_map_recovered": bool((mp == planted.cpu().to(mp.dtype)).all()),
        "trace_bytes": int(a_d.numel() * 4 + a_t.numel() * 4)}))


def _median(xs):
    return round(statistics.median(xs), 2)


class Point:
    """select -> sparse attention -> dense attention on one resident workload at one budget, with
    index and output buffers of its own; the dense pass between two sparse passes (and the
    rotation over layers) keeps every sparse pass cache-cold."""

    def __init__(self, torch, sts, w, layers, kb, page=1, extra=None):
        cfg = w.cfg
        dev = w.q.device
        self.torch, self.sts, self.w, self.layers, self.kb, self.page = torch, sts, w, layers, kb, page
        self.extra = dict(extra or {})
        self.idx = torch.empty(cfg.B, cfg.Hq, kb, dtype=torch.int32, device=dev)
        self.cnt = torch.empty(cfg.B, cfg.Hq, dtype=torch.int32, device=dev)
        self.out_s = torch.empty(cfg.B, cfg.Tq, cfg.Hq, cfg.d, dtype=torch.bfloat16, device=dev)
        self.out_d = torch.empty_like(self.out_s)
        self._calls = {}

    # the parameter block of every call is built once (PreparedCall): a launch then costs the host
    # one ctypes call, as in a serving loop that repeats the step on fixed buffers
    def _prepared(self, kind, layer=0):
        key = (kind, layer, self.torch.cuda.current_stream().cuda_stream)
        call = self._calls.get(key)
        if call is None:
            sts, w = self.sts, self.w
            if kind == "select":
                call = sts.sts_select(w.scores, w.head_map, self.kb, out=(self.idx, self.cnt), page_size=self.page, prepare=True)
            else:
                lk, lv = self.layers[layer]
                if kind == "sparse":
                    call = sts.sts_sparse_attn(w.q, lk, lv, self.idx, w.scale, counts=self.cnt, head_map=w.head_map,
                                               out=self.out_s, want_lse=False, prepare=True, **self.extra)
                else:
                    call = sts.sts_dense_attn(w.q, lk, lv, w.scale, out=self.out_d, want_lse=False, prepare=True, **self.extra)
            self._calls[key] = call
        return call

    def select(self):
        self._prepared("select")()

    def sparse(self, layer=0):
        self._prepared("sparse", layer)()

    def dense(self, layer=0):
        self._prepared("dense", layer)()

    def bytes_set(self):
        plan = self.sts.attn_plan(self.w.q, self.torch.empty(self.w.cfg.B, self.w.cfg.Hkv, self.w.cfg.N, self.w.cfg.d, device="meta"),
                                  True, kmax=self.kb, head_map=self.w.head_map, page_size=self.page)
        return self.w.cfg.B * plan["units_per_batch"] * self.kb * self.page * 2 * self.w.cfg.d * 2, plan

    def eager(self, steps, warmup=2):
        """Per-call medians (us) over `steps` event-timed steps, then the split kernel's own time
        from the library's dispatch-stamped events."""
        torch, sts = self.torch, self.sts
        L = len(self.layers)
        for _ in range(warmup):
            for l in range(L):
                self.select(); self.sparse(l); self.dense(l)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps * L)]
        torch.cuda.synchronize()
        for i in range(steps):
            for l in range(L):
                ev = evs[i * L + l]
                ev[0].record(); self.select(); ev[1].record(); self.sparse(l); ev[2].record(); self.dense(l); ev[3].record()
        torch.cuda.synchronize()
        t = [_median([ev[i].elapsed_time(ev[i + 1]) * 1e3 for ev in evs]) for i in range(3)]
        sts.prof_enable(True)
        sts.prof_reset()
        for i in range(max(1, min(steps, STS_PROF_BUDGET // (8 * L)))):
            for l in range(L):
                self.select(); self.sparse(l); self.dense(l)
        torch.cuda.synchronize()
        prof = sts.prof_read()
        sts.prof_enable(False)
        kus = {k: round(ms * 1e3 / n, 2) for k, (n, ms) in prof.items() if n}
        b_set, plan = self.bytes_set()
        split = kus.get("attn_sparse", 0.0)
        return {"budget_tokens": self.kb * self.page, "select_us": t[0], "sparse_attn_us": t[1], "dense_attn_us": t[2],
                "speedup_vs_dense": round(t[2] / t[1], 3) if t[1] > 0 else None,
                # (the combine kernel's figure averages the sparse and the dense call's launches)
                "kernel_us": {k: v for k, v in kus.items() if k.startswith("attn_sparse") or k.startswith("select")
                              or (k == "attn_combine" and plan["num_splits"] > 1)},
                "gathered_kv_bytes_b_set": b_set, "num_splits": plan["num_splits"],
                "split_kernel_frac": round(b_set / (split * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if split > 0 else None,
                "call_frac": round(b_set / (t[1] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if t[1] > 0 else None}

    def stacked(self, stack, reps=20):
        """sts_sparse_attn on a stack of layers back to back (each layer its own K/V buffers, the
        same index sets), one event pair around the whole stack: what a layer costs inside a
        forward pass, where no event packets stand between the calls. Eager launches, no graph."""
        torch = self.torch
        saved = self.layers
        self.layers = stack
        try:
            for l in range(len(stack)):
                self.sparse(l)
            torch.cuda.synchronize()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
            evs[0].record()
            for i in range(reps):
                for l in range(len(stack)):
                    self.sparse(l)
                evs[i + 1].record()
            torch.cuda.synchronize()
            us = statistics.median(evs[i].elapsed_time(evs[i + 1]) for i in range(reps)) * 1e3 / len(stack)
        finally:
            self.layers = saved
            self._calls = {k: v for k, v in self._calls.items() if k[0] != "sparse"}
        return {"layers": len(stack), "sparse_attn_us_per_layer": round(us, 2)}

    def graph(self, reps=30):
        """The same calls captured in HIP graphs and replayed (no host launch cost between the
        kernels). A call's time is the difference between a graph that holds it after a dense pass
        (which leaves the caches cold for it) and a graph that holds the dense pass alone."""
        torch = self.torch
        L = len(self.layers)

        def capture(body):
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                body()                               # workspaces of this stream exist before the capture
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=s):
                    body()
            torch.cuda.synchronize()
            return g

        def run(g):
            g.replay()
            torch.cuda.synchronize()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
            evs[0].record()
            for i in range(reps):
                g.replay()
                evs[i + 1].record()
            torch.cuda.synchronize()
            # median over the replays: one disturbed replay must not decide a difference of a few us
            return statistics.median(evs[i].elapsed_time(evs[i + 1]) for i in range(reps)) * 1e3 / L

        def every_layer(fn):
            def body():
                for l in range(L):
                    fn(l)
            return body

        t_dense = run(capture(every_layer(lambda l: self.dense(l))))
        t_ds = run(capture(every_layer(lambda l: (self.dense(l), self.sparse(l)))))
        t_dsel = run(capture(every_layer(lambda l: (self.dense(l), self.select()))))
        t_step = run(capture(every_layer(lambda l: (self.select(), self.sparse(l), self.dense(l)))))
        return {"sparse_attn_us": round(t_ds - t_dense, 2), "select_us": round(t_dsel - t_dense, 2),
                "dense_attn_us": round(t_dense, 2), "step_us": round(t_step, 2)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2605_15508_amd as sts
    from dataclasses import replace

    from workload import CONFIGS, budget_tokens, make_draft_layer, make_workload

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sts.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.prefill_blocks > 0:
        return run_prefill(args, torch, sts)
    if args.headmap:
        return run_headmap(args, torch, sts)
    cfg = CONFIGS[args.config]
    if args.gain is not None:
        cfg = replace(cfg, gain=args.gain)
    if args.draft_heads is not None:
        assert not cfg.draft_d, "the draft-layer configuration fixes its head count"
        cfg = replace(cfg, Hd=args.draft_heads)
    if args.positions == "recent":
        cfg = replace(cfg, clustered=True)
    head_map = None
    if args.head_map == "random":
        hg = torch.Generator().manual_seed(args.seed + 4242)
        head_map = torch.randint(0, cfg.Hd, (cfg.Hq,), generator=hg, dtype=torch.int32)
    w = make_workload(cfg, seed=args.seed, device=dev, budget=args.budget, with_scores=not cfg.draft_d,
                      head_map=head_map)
    page = max(1, args.page_size)
    kb = -(-w.k_budget // page)          # same token budget, counted in blocks of `page` tokens
    B, N, Hq, Hkv, d, Tq, Hd = cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.d, cfg.Tq, cfg.Hd
    draft = make_draft_layer(w) if cfg.draft_d else None
    # distinct resident layers (1M-context configuration: 32 x 4 GiB of KV); the draft scores
    # are shared by the layers, the KV caches are not
    layers = [(w.k, w.v)]
    kv_bytes = 2 * B * Hkv * N * d * 2
    n_layers = cfg.layers
    if not args.warm:
        n_layers = max(n_layers, min(128, -(-(2 << 30) // kv_bytes)))     # cold-cache rotation
    for l in range(1, n_layers):
        wl = make_workload(cfg, seed=args.seed + l, device=dev, budget=args.budget, with_scores=False)
        layers.append((wl.k, wl.v))
        del wl
    table = None
    if args.paged:
        # scatter every layer's cache into a pool [pages, Hkv, page, d] behind one random table
        assert N % page == 0, "--paged needs N divisible by the page size"
        nblk = N // page
        gen = torch.Generator(device=dev)
        gen.manual_seed(args.seed + 999)
        table = torch.randperm(B * nblk, generator=gen, device=dev).to(torch.int32).view(B, nblk)
        inv = table.view(-1).long()
        pooled = []
        for (lk, lv) in layers:
            pk = torch.empty(B * nblk, Hkv, page, d, dtype=torch.bfloat16, device=dev)
            pv = torch.empty_like(pk)
            pk[inv] = lk.view(B, Hkv, nblk, page, d).permute(0, 2, 1, 3, 4).reshape(B * nblk, Hkv, page, d)
            pv[inv] = lv.view(B, Hkv, nblk, page, d).permute(0, 2, 1, 3, 4).reshape(B * nblk, Hkv, page, d)
            pooled.append((pk, pv))
        layers = pooled      # w.k / w.v keep the logical layer-0 cache for the CPU baseline
    pg = dict(page_size=page, block_table=table, N=N) if table is not None else dict(page_size=page)
    torch.cuda.synchronize()

    # persistent outputs so the timed region allocates nothing
    idx = torch.empty(B, Hq, kb, dtype=torch.int32, device=dev)
    cnt = torch.empty(B, Hq, dtype=torch.int32, device=dev)
    out_s = torch.empty(B, Tq, Hq, d, dtype=torch.bfloat16, device=dev)
    out_d = torch.empty_like(out_s)
    d_out = d_lse = d_logits = d_sum = None
    if draft is not None:
        d_out = torch.empty(B, Tq, Hd, cfg.draft_d, dtype=torch.bfloat16, device=dev)
        d_lse = torch.empty(B, Hd, Tq, dtype=torch.float32, device=dev)
        if args.draft_scores == "sum":
            d_sum = torch.empty(B, Hd, N, dtype=torch.float32, device=dev)
        else:
            d_logits = torch.empty(B, Hd, Tq, N, dtype=torch.bfloat16 if args.scores == "bf16" else torch.float32, device=dev)
    elif args.scores == "bf16":
        w.scores = w.scores.to(torch.bfloat16)

    if args.fused_tail:
        tg = torch.Generator(device=dev)
        tg.manual_seed(args.seed + 5)
        pg["k_new"] = (torch.randn(B, Tq, Hkv, d, generator=tg, device=dev) * 0.5).to(torch.bfloat16)
        pg["v_new"] = (torch.randn(B, Tq, Hkv, d, generator=tg, device=dev) * 0.5).to(torch.bfloat16)
        pg["causal"] = True

    def step(ev=None, layer=0):
        lk, lv = layers[layer]
        if ev: ev[0].record()
        if draft is not None and d_sum is not None:
            sts.sts_dense_attn(draft["q"], draft["k"], draft["v"], draft["scale"], out=d_out,
                               lse_out=d_lse, weights_sum_out=d_sum)
            if ev: ev[1].record()
            sts.sts_select(d_sum.view(B, Hd, 1, N), w.head_map, kb, out=(idx, cnt), page_size=page)
        elif draft is not None:
            sts.sts_dense_attn(draft["q"], draft["k"], draft["v"], draft["scale"], out=d_out,
                               lse_out=d_lse, logits_out=d_logits)
            if ev: ev[1].record()
            sts.sts_select(d_logits, w.head_map, kb, lse=d_lse, kind=sts.STS_SCORES_LOGITS_LSE, out=(idx, cnt),
                           page_size=page)
        else:
            if ev: ev[1].record()
            sts.sts_select(w.scores, w.head_map, kb, out=(idx, cnt), page_size=page)
        if ev: ev[2].record()
        sts.sts_sparse_attn(w.q, lk, lv, idx, w.scale, counts=cnt, head_map=w.head_map, out=out_s,
                            want_lse=False, **pg)
        if ev: ev[3].record()
        if not args.no_dense:
            sts.sts_dense_attn(w.q, lk, lv, w.scale, out=out_d, want_lse=False, **pg)
        if ev: ev[4].record()

    L = len(layers)
    for _ in range(args.warmup):
        for l in range(L):
            step(layer=l)
    torch.cuda.synchronize()

    # timed region: exactly K steps, sync on both sides; per-call times from events recorded on
    # the stream the library launches on (torch's current stream)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps * L)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        for l in range(L):
            step(events[i * L + l], layer=l)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # second pass of K steps with the library's per-kernel HIP events switched on: every dispatch
    # stamps its own begin and end into a pair of events (kept out of the region that gives
    # `value`, which is timed without them)
    sts.prof_enable(True)
    sts.prof_reset()
    prof_steps = min(args.steps, max(1, STS_PROF_BUDGET // (8 * L))) * L
    for i in range(prof_steps // L):
        for l in range(L):
            step(layer=l)
    torch.cuda.synchronize()
    prof = sts.prof_read()
    sts.prof_enable(False)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # one kernel reading 1 GiB and writing 1 GiB
        torch.cuda.synchronize()
        del src, dst

    def stage(i):
        xs = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for ev in events)      # microseconds
        pick = lambda f: xs[min(len(xs) - 1, int(f * len(xs)))]
        return statistics.fmean(xs), statistics.median(xs), min(xs), pick(0.10), pick(0.90)

    draft_us, select_us, sparse_us, dense_us = stage(0), stage(1), stage(2), stage(3)
    K = args.steps
    split_n, split_ms = prof["attn_sparse"]
    split_us = split_ms * 1e3 / max(split_n, 1)
    dsplit_n, dsplit_ms = prof["attn_dense"]
    plan = sts.attn_plan(w.q, layers[0][0] if table is None else torch.empty(B, Hkv, N, d, device="meta"), True,
                         kmax=kb, head_map=w.head_map, page_size=page)
    units = plan["units_per_batch"]
    row_bytes = 2 * d * 2                                   # one K row + one V row, bf16
    b_set = B * units * kb * page * row_bytes               # gathered once per distinct index row
    b_req = B * Hq * kb * page * row_bytes                  # gathered per query head
    b_dense = B * Hkv * N * row_bytes
    # union of the rows requested per (batch, KV head): what perfect reuse between the sets of a
    # KV group would have to move (reported beside B_set so cache reuse cannot hide in it)
    G = Hq // Hkv
    seen = torch.zeros(B, Hkv, -(-N // page), dtype=torch.bool, device=dev)
    ii = idx.view(B, Hkv, G * kb).long().clamp_(0, seen.shape[2] - 1)
    seen.scatter_(2, ii, True)
    b_uniq = int(seen.sum().item()) * page * row_bytes
    del seen, ii
    achieved = b_set / (split_us * 1e-6) / 1e9 if split_us > 0 else 0.0
    workload = (f"{cfg.name}: B{B} N{N} Hq{Hq}/Hkv{Hkv} d{d} Tq{Tq} Hd{Hd} budget "
                f"{kb * page} tokens ({kb * page / N:.1%})"
                + (f" as {kb} blocks of {page}" if page > 1 else "") + (" paged KV" if args.paged else ""))
    result = {
        "metric": METRIC,
        "value": round(sparse_us[1], 2),
        "value_stat": "median of the per-call times of the timed steps (mean, min, p10, p90 below)",
        "unit": "us/layer",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": round(wall / K * 1e3, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": workload, "context": N, "batch": B, "budget_tokens": kb * page, "page_size": page, "paged_kv": bool(args.paged),
                   "layers": L, "cache": "cold: every pass reads KV that has left the caches" if (L > 1 or kv_bytes > (256 << 20)) else "warm", "head_map": "t*Hd//Hq" if args.head_map == "default" else "seeded random", "gain": cfg.gain, "heavy_positions": args.positions, "scores": args.scores, "fused_tail": bool(args.fused_tail), "step": ("%d layers x (" % L if L > 1 else "(") + "select + sparse_attn" + ("" if args.no_dense else " + dense_attn")
                   + ((" + draft dense attn with logits dump" if d_sum is None else " + draft dense attn with summed weights") if draft is not None else "") + ")"},
        "sparse_attn_us": {"mean": round(sparse_us[0], 2), "median": round(sparse_us[1], 2), "min": round(sparse_us[2], 2), "p10": round(sparse_us[3], 2), "p90": round(sparse_us[4], 2)},
        "dense_attn_us": None if args.no_dense else {"mean": round(dense_us[0], 2), "median": round(dense_us[1], 2), "min": round(dense_us[2], 2), "p10": round(dense_us[3], 2), "p90": round(dense_us[4], 2)},
        "select_us": {"mean": round(select_us[0], 2), "median": round(select_us[1], 2), "min": round(select_us[2], 2), "p10": round(select_us[3], 2), "p90": round(select_us[4], 2)},
        "speedup_vs_dense": round(dense_us[1] / sparse_us[1], 3) if not args.no_dense and sparse_us[1] > 0 else None,
        "gathered_kv_gbs": {"b_set": round(b_set / (sparse_us[1] * 1e-6) / 1e9, 1),
                            "b_req": round(b_req / (sparse_us[1] * 1e-6) / 1e9, 1),
                            "b_uniq": round(b_uniq / (sparse_us[1] * 1e-6) / 1e9, 1)},
        "gathered_kv_bytes": {"b_set": b_set, "b_req": b_req, "b_uniq": b_uniq, "dense": b_dense},
        "dense_kv_gbs": round(b_dense / (dense_us[1] * 1e-6) / 1e9, 1) if not args.no_dense else None,
        "kernel_us": {k: round(ms * 1e3 / n, 2) for k, (n, ms) in prof.items() if n},
        "launch": plan,
        "roofline": {
            "bound": "hbm", "kernel": "attn_split_kernel<sparse>", "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
            "algorithmic_bytes_per_launch": b_set, "avg_launch_us": round(split_us, 2), "launches": split_n,
            "traffic": None,       # filled in below from the committed counter summary, if it belongs to this library version
        },
        "paper_context": "2.67x end-to-end speedup at ~90% sparsity on NVIDIA H20 (other hardware, whole serving stack)",
    }
    agg_n, agg_ms = prof["select_agg"]
    if agg_n:
        # the one HBM-bound kernel of the selection: reads Tq rows of scores, writes one row of A
        tq_in = 1 if d_sum is not None else Tq
        src_rows = B * Hd * (tq_in * N * (2 if args.scores == "bf16" else 4) + N * 4)
        agg_us = agg_ms * 1e3 / agg_n
        result["roofline_select_agg"] = {"bound": "hbm", "achieved": round(src_rows / (agg_us * 1e-6) / 1e9, 1),
                                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": round(src_rows / (agg_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                         "algorithmic_bytes_per_launch": src_rows, "avg_launch_us": round(agg_us, 2)}
    if draft is not None:
        result["draft_attn_us"] = {"mean": round(draft_us[0], 2), "median": round(draft_us[1], 2)}
    if dsplit_n:
        result["roofline_dense"] = {"achieved": round(b_dense / (dsplit_ms * 1e-3 / dsplit_n) / 1e9, 1),
                                    "frac": round(b_dense / (dsplit_ms * 1e-3 / dsplit_n) / 1e9 / HBM_PEAK_GBS, 4)}
    version = sts.sts_version()
    result["library_version"] = version
    result["roofline"]["traffic"] = (read_traffic("attn_sparse_split", cfg.name, version)
                                     if (args.budget is None and page == 1) else None)
    result["roofline"]["scope"] = ("the split kernel alone (the dominant kernel of sts_sparse_attn); the whole call, "
                                   "with the combine kernel and the gaps between launches, is roofline_call")
    # the same algorithmic bytes over the time of the whole sts_sparse_attn call (`value`)
    result["roofline_call"] = {"bound": "hbm", "bytes": b_set, "us": round(sparse_us[1], 2), "unit": "GB/s",
                               "achieved": round(b_set / (sparse_us[1] * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS,
                               "frac": round(b_set / (sparse_us[1] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    # the selection against the same roofline: the score tensor it ranks is read once (its lists are
    # small next to it); kernels = the sum of its kernels' own times, call = the event-timed call
    sel_src = d_sum if (draft is not None and d_sum is not None) else (d_logits if draft is not None else w.scores)
    sel_bytes = sel_src.numel() * sel_src.element_size()
    sel_kernels = sum(ms * 1e3 for k_, (n, ms) in prof.items() if n and k_.startswith("select")) / prof_steps
    result["roofline_select"] = {"bound": "hbm", "bytes": sel_bytes, "unit": "GB/s", "peak": HBM_PEAK_GBS,
                                 "kernels_us": round(sel_kernels, 2), "call_us": round(select_us[1], 2),
                                 "frac_kernels": round(sel_bytes / (sel_kernels * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if sel_kernels > 0 else None,
                                 "frac_call": round(sel_bytes / (select_us[1] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    plain = draft is None and not args.paged and page == 1 and not args.fused_tail and args.scores == "fp32"
    if plain and not args.no_extras:
        here = Point(torch, sts, w, layers, kb)
        here.select()
        result["graph_replay"] = here.graph()
        result["graph_replay"]["call_frac"] = round(b_set / (result["graph_replay"]["sparse_attn_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        # the budget sweep of the 128K configuration (5% and 20% beside the 10% above), same resident inputs
        if cfg.name == "c3" and args.budget is None:
            # eight layers' caches (16 GiB) attended back to back: the gathered rows of a pass (3.4 GB)
            # exceed every cache, so each call still reads its rows from HBM
            stack = [layers[0]] + [(layers[0][0].clone(), layers[0][1].clone()) for _ in range(7)]
            result["stacked_layers"] = here.stacked(stack)
            result["stacked_layers"]["call_frac"] = round(
                b_set / (result["stacked_layers"]["sparse_attn_us_per_layer"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
            del stack
            result["sweep"] = {}
            for frac in (0.05, 0.20):
                pt = Point(torch, sts, w, layers, budget_tokens(cfg, frac))
                result["sweep"]["%g%%" % (frac * 100)] = pt.eager(min(K, 10))
                del pt
            # the paper's own operating points (Sections 6.2, 6.3: budgets of 256, 512 and 4096 tokens)
            result["paper_budgets"] = {}
            for kk in (256, 512, 4096):
                pt = Point(torch, sts, w, layers, kk)
                r = pt.eager(min(K, 10))
                r["graph_replay"] = pt.graph()
                result["paper_budgets"]["%s@%d" % (cfg.name, kk)] = r
                del pt
            # and the 32K configuration at its 10% budget (16 rotating layers: cold caches)
            c2 = CONFIGS["c2"]
            w2 = make_workload(c2, seed=args.seed, device=dev)
            layers2 = [(w2.k, w2.v)]
            for l in range(1, 16):
                wl = make_workload(c2, seed=args.seed + l, device=dev, with_scores=False)
                layers2.append((wl.k, wl.v))
                del wl
            pt = Point(torch, sts, w2, layers2, w2.k_budget)
            r = pt.eager(min(K, 10))
            r["graph_replay"] = pt.graph(reps=5)
            result["paper_budgets"]["c2@%d" % w2.k_budget] = r
            del pt, w2, layers2
    if not args.no_cpu_baseline:
        step(layer=0)                     # the outputs of layer 0, whose cache the oracle reads below
        torch.cuda.synchronize()
        if d_sum is not None:
            result["cpu_baseline"], result["parity"] = cpu_baseline(w, idx, cnt, out_s, page=page, scores=d_sum.view(B, Hd, 1, N), lse=None)
        else:
            result["cpu_baseline"], result["parity"] = cpu_baseline(w, idx, cnt, out_s, page=page, scores=d_logits, lse=d_lse)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
