"""CPU oracle for the STS hot path -- TEST INFRASTRUCTURE ONLY.

ctypes wrapper around ``sts_oracle.c`` (plain C, fp64 accumulation). Only tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; the product path
never does. It shares no code with the HIP library.

Arrays are numpy (host). bf16 tensors are passed as ``uint16`` bit patterns; use
:func:`bf16_bits` to get them from a torch bf16 tensor.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sts_oracle.c")
_LIB = os.path.join(_HERE, "libsts_oracle.so")

PROBS, LOGITS_LSE = 0, 1
SUM, MAX = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp, no fast-math). Returns the library path."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)
            and os.path.getmtime(_LIB) >= os.path.getmtime(os.path.join(_HERE, "sts_oracle.h"))):
        return _LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # STS_ORACLE_LIB: a library built elsewhere from (a variant of) sts_oracle.c; the
        # mutation test uses it to show that the pins reject planted mistakes
        _lib = ctypes.CDLL(os.environ.get("STS_ORACLE_LIB") or build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def bf16_bits(t) -> np.ndarray:
    """uint16 bit patterns of a (CPU, contiguous or strided) torch bf16 tensor, same shape/strides."""
    import torch

    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.view(torch.int16).numpy().view(np.uint16)


def _p(a: Optional[np.ndarray], ty):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what} failed with oracle status {rc}")


def aggregate(scores: np.ndarray, lse: Optional[np.ndarray] = None, kind: int = PROBS,
              reduce: int = SUM) -> np.ndarray:
    """scores [B,Hd,Tq,N] fp32 (+ lse [B,Hd,Tq]) -> A [B,Hd,N] fp32. See oracle_aggregate."""
    scores = _c(scores, np.float32)
    B, Hd, Tq, N = scores.shape
    if lse is not None:
        lse = _c(lse, np.float32)
        assert lse.shape == (B, Hd, Tq)
    A = np.empty((B, Hd, N), np.float32)
    rc = _load().oracle_aggregate(_p(scores, ctypes.c_float), _p(lse, ctypes.c_float), B, Hd, Tq, N,
                                  kind, reduce, _p(A, ctypes.c_float))
    _check(rc, "oracle_aggregate")
    return A


def select(A: np.ndarray, k: int, seq_lens: Optional[np.ndarray] = None):
    """A [B,Hd,N] fp32 -> (sel [B,Hd,k] int32 ascending, -1 padded ; cnt [B,Hd]). See oracle_select."""
    A = _c(A, np.float32)
    B, Hd, N = A.shape
    if seq_lens is not None:
        seq_lens = _c(seq_lens, np.int32)
        assert seq_lens.shape == (B,)
    sel = np.empty((B, Hd, k), np.int32)
    cnt = np.empty((B, Hd), np.int32)
    rc = _load().oracle_select(_p(A, ctypes.c_float), B, Hd, N, _p(seq_lens, ctypes.c_int32), int(k),
                               _p(sel, ctypes.c_int32), _p(cnt, ctypes.c_int32))
    _check(rc, "oracle_select")
    return sel, cnt


def block_scores(A: np.ndarray, page: int, seq_lens: Optional[np.ndarray] = None) -> np.ndarray:
    """A [B,Hd,N] -> per-block sums [B,Hd,ceil(N/page)]. See oracle_block_scores."""
    A = _c(A, np.float32)
    B, Hd, N = A.shape
    if seq_lens is not None:
        seq_lens = _c(seq_lens, np.int32)
    NB = (N + page - 1) // page
    blk = np.empty((B, Hd, NB), np.float32)
    rc = _load().oracle_block_scores(_p(A, ctypes.c_float), B, Hd, N, _p(seq_lens, ctypes.c_int32),
                                     int(page), _p(blk, ctypes.c_float))
    _check(rc, "oracle_block_scores")
    return blk


def expand_blocks(indices: np.ndarray, counts: Optional[np.ndarray], page: int, N: int):
    """Block ids [B,Hq,kb] (+counts in blocks) -> token ids [B,Hq,kb*page] and token counts:
    block m stands for tokens m*page .. min((m+1)*page, N)-1, in order. Rows are left-packed."""
    indices = _c(indices, np.int32)
    B, Hq, kb = indices.shape
    tok = np.full((B, Hq, kb * page), -1, np.int32)
    cnt = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for t in range(Hq):
            c = kb if counts is None else int(counts[b, t])
            row = []
            for m in indices[b, t, :c]:
                row.extend(range(int(m) * page, min((int(m) + 1) * page, N)))
            tok[b, t, :len(row)] = row
            cnt[b, t] = len(row)
    return tok, cnt


def select_per_head(A: np.ndarray, k: int, k_head, seq_lens: Optional[np.ndarray] = None):
    """Per-head budgets (Section 6.4: layers, and heads, differ in how much they can drop):
    head j keeps min(k_head[j], N_b) entries, rows stay k wide and are padded with -1."""
    A = _c(A, np.float32)
    B, Hd, N = A.shape
    assert len(k_head) == Hd and all(1 <= int(x) <= k for x in k_head)
    sel = np.full((B, Hd, k), -1, np.int32)
    cnt = np.zeros((B, Hd), np.int32)
    for j in range(Hd):
        kj = int(k_head[j])
        s, c = select(A[:, j:j + 1], kj, seq_lens)
        sel[:, j, :kj] = s[:, 0]
        cnt[:, j] = c[:, 0]
    return sel, cnt


def select_indices(scores, head_map, k, lse=None, kind=PROBS, reduce=SUM, seq_lens=None, page=1,
                   k_head=None):
    """The whole selection half: aggregate -> [block scores] -> select -> remap. With page > 1
    the result holds block ids (k counts blocks). Returns (indices, counts, A)."""
    A = aggregate(scores, lse, kind, reduce)
    pick = select if k_head is None else (lambda a, kk, ln: select_per_head(a, kk, k_head, ln))
    if page > 1:
        src = block_scores(A, page, seq_lens)
        lens = None if seq_lens is None else (np.asarray(seq_lens, np.int64) + page - 1) // page
        sel, cnt = pick(src, k, None if lens is None else lens.astype(np.int32))
    else:
        sel, cnt = pick(A, k, seq_lens)
    indices, counts = remap(sel, cnt, head_map)
    return indices, counts, A


def remap(sel: np.ndarray, cnt: np.ndarray, head_map: np.ndarray):
    """sel [B,Hd,k], cnt [B,Hd], head_map [Hq] -> (indices [B,Hq,k], counts [B,Hq]). See oracle_remap."""
    sel = _c(sel, np.int32)
    cnt = _c(cnt, np.int32)
    head_map = _c(head_map, np.int32)
    B, Hd, k = sel.shape
    Hq = head_map.shape[0]
    indices = np.empty((B, Hq, k), np.int32)
    counts = np.empty((B, Hq), np.int32)
    rc = _load().oracle_remap(_p(sel, ctypes.c_int32), _p(cnt, ctypes.c_int32), B, Hd, Hq, k,
                              _p(head_map, ctypes.c_int32), _p(indices, ctypes.c_int32),
                              _p(counts, ctypes.c_int32))
    _check(rc, "oracle_remap")
    return indices, counts


def attn(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
         indices: Optional[np.ndarray] = None, counts: Optional[np.ndarray] = None,
         seq_lens: Optional[np.ndarray] = None, want_logits: bool = False,
         batches: Optional[range] = None, heads: Optional[range] = None,
         k_new: Optional[np.ndarray] = None, v_new: Optional[np.ndarray] = None, causal: bool = True):
    """Sparse (indices given) or dense (indices None) softmax attention. See oracle_attn.

    q [B,Tq,Hq,d] uint16 (bf16 bits); k, v [B,Hkv,N,d] uint16, any strides with unit stride on d.
    Returns dict(out [B,Tq,Hq,d] fp32, lse [B,Hq,Tq] fp32, logits [B,Hq,Tq,N] or None).
    ``batches``/``heads`` (contiguous ranges) restrict which outputs are computed; the others
    stay zero (lse NaN). ``k_new``/``v_new`` [B,Tq,Hkv,d] uint16 are the speculative block's own
    keys/values, appended after the cached keys (row i sees new tokens 0..i when ``causal``).
    """
    assert q.dtype == np.uint16 and k.dtype == np.uint16 and v.dtype == np.uint16
    q = np.ascontiguousarray(q)
    B, Tq, Hq, d = q.shape
    Bk, Hkv, N, dk = k.shape
    assert (Bk, dk) == (B, d) and v.shape == k.shape and v.strides == k.strides
    assert k.strides[3] == 2
    sb, sh, sn = (s // 2 for s in k.strides[:3])
    kmax = 0
    if indices is not None:
        indices = _c(indices, np.int32)
        assert indices.shape[:2] == (B, Hq)
        kmax = indices.shape[2]
        if counts is not None:
            counts = _c(counts, np.int32)
            assert counts.shape == (B, Hq)
    if seq_lens is not None:
        seq_lens = _c(seq_lens, np.int32)
    if k_new is not None:
        k_new, v_new = np.ascontiguousarray(k_new), np.ascontiguousarray(v_new)
        assert k_new.dtype == np.uint16 and k_new.shape == (B, Tq, Hkv, d) and v_new.shape == k_new.shape
    out = np.zeros((B, Tq, Hq, d), np.float32)
    lse = np.full((B, Hq, Tq), np.nan, np.float32)
    logits = np.zeros((B, Hq, Tq, N), np.float32) if want_logits else None
    bb, be = (batches.start, batches.stop) if batches is not None else (0, B)
    hb, he = (heads.start, heads.stop) if heads is not None else (0, Hq)
    lib = _load()
    rc = lib.oracle_attn(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                         B, Tq, Hq, Hkv, d, N, ctypes.c_int64(sb), ctypes.c_int64(sh),
                         ctypes.c_int64(sn), _p(indices, ctypes.c_int32), _p(counts, ctypes.c_int32),
                         kmax, _p(seq_lens, ctypes.c_int32), ctypes.c_float(scale),
                         _p(out, ctypes.c_float), _p(lse, ctypes.c_float), _p(logits, ctypes.c_float),
                         bb, be, hb, he, _p(k_new, ctypes.c_uint16), _p(v_new, ctypes.c_uint16),
                         1 if causal else 0)
    _check(rc, "oracle_attn")
    return {"out": out, "lse": lse, "logits": logits}


def select_rows(scores, k, lse=None, kind=PROBS, seq_lens=None):
    """Per-row selection for prefill (Section 4.2: during prefill every query token has a mask
    of its own, a two-dimensional pattern per head): every one of the Tq score rows of a draft
    head is ranked by itself. scores [B,Hd,Tq,N] -> (sel [B,Hd,Tq,k] ascending, -1 padded;
    cnt [B,Hd,Tq]). It is the single-row case of the selection, row by row."""
    scores = _c(scores, np.float32)
    B, Hd, Tq, N = scores.shape
    sel = np.empty((B, Hd, Tq, k), np.int32)
    cnt = np.empty((B, Hd, Tq), np.int32)
    for i in range(Tq):
        A = aggregate(scores[:, :, i:i + 1], None if lse is None else np.ascontiguousarray(lse[:, :, i:i + 1]), kind, SUM)
        sel[:, :, i], cnt[:, :, i] = select(A, k, seq_lens)
    return sel, cnt


def union_rows(row_sel: np.ndarray, row_cnt: Optional[np.ndarray], head_map, pitch: Optional[int] = None):
    """The tokens any query row of a block keeps, per target head, and which rows keep each of
    them. row_sel [B,Hd,Tq,k] (the valid entries of a row come first, row_cnt [B,Hd,Tq] or None = k
    of them), head_map [Hq] target head -> draft head. Returns (union [B,Hq,pitch] int32 ascending,
    -1 padded; mask [B,Hq,pitch] uint16, bit i set iff row i keeps the token; cnt [B,Hq]).
    Written out as the definition: a set union per target head (Section 4.2: the target attends to
    the key-value pairs the indices name, here one index set per query row)."""
    row_sel = np.asarray(row_sel)
    B, Hd, Tq, k = row_sel.shape
    assert Tq <= 16
    head_map = np.asarray(head_map)
    Hq = head_map.shape[0]
    rows = [[None] * Hq for _ in range(B)]
    longest = 0
    for b in range(B):
        for t in range(Hq):
            j = int(head_map[t])
            keep = {}
            for i in range(Tq):
                c = k if row_cnt is None else int(row_cnt[b, j, i])
                for n in row_sel[b, j, i, :c]:
                    keep[int(n)] = keep.get(int(n), 0) | (1 << i)
            rows[b][t] = sorted(keep.items())
            longest = max(longest, len(keep))
    pitch = longest if pitch is None else pitch
    assert pitch >= longest
    union = np.full((B, Hq, pitch), -1, np.int32)
    mask = np.zeros((B, Hq, pitch), np.uint16)
    cnt = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for t in range(Hq):
            cnt[b, t] = len(rows[b][t])
            for p, (n, bits) in enumerate(rows[b][t]):
                union[b, t, p] = n
                mask[b, t, p] = bits
    return union, mask, cnt


def attn_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float, row_idx: np.ndarray,
              row_cnt: Optional[np.ndarray] = None):
    """Attention with an index set per query row: row i of head t attends to row_idx[b,t,i,:c]
    (row_cnt [B,Hq,Tq] valid entries, or all). The definition, query row by query row: each row is
    the one-row case of `attn`. Returns dict(out [B,Tq,Hq,d], lse [B,Hq,Tq])."""
    B, Tq, Hq, d = q.shape
    out = np.zeros((B, Tq, Hq, d), np.float32)
    lse = np.zeros((B, Hq, Tq), np.float32)
    for i in range(Tq):
        r = attn(np.ascontiguousarray(q[:, i:i + 1]), k, v, scale, np.ascontiguousarray(row_idx[:, :, i]),
                 None if row_cnt is None else np.ascontiguousarray(row_cnt[:, :, i]))
        out[:, i] = r["out"][:, 0]
        lse[:, :, i] = r["lse"][:, :, 0]
    return {"out": out, "lse": lse}


def rows_of_union(union: np.ndarray, mask: np.ndarray, cnt: np.ndarray, Tq: int, pitch: int):
    """Back from (union, mask) to one index list per query row: [B,Hq,Tq,pitch] (-1 padded) and
    counts [B,Hq,Tq]."""
    B, Hq, _ = union.shape
    rows = np.full((B, Hq, Tq, pitch), -1, np.int32)
    rc = np.zeros((B, Hq, Tq), np.int32)
    for b in range(B):
        for t in range(Hq):
            c = int(cnt[b, t])
            for i in range(Tq):
                mine = union[b, t, :c][(mask[b, t, :c] >> i) & 1 == 1]
                rows[b, t, i, :len(mine)] = mine
                rc[b, t, i] = len(mine)
    return rows, rc


def head_mapping(a_d: np.ndarray, a_t: np.ndarray, k: int):
    """Algorithm 1. a_d [S,Hd,R,N], a_t [S,Ht,R,N] fp32 -> (map [Ht] int32, overlap [Ht,Hd] int64)."""
    a_d = _c(a_d, np.float32)
    a_t = _c(a_t, np.float32)
    S, Hd, R, N = a_d.shape
    St, Ht, Rt, Nt = a_t.shape
    assert (St, Rt, Nt) == (S, R, N)
    mp = np.empty((Ht,), np.int32)
    ov = np.empty((Ht, Hd), np.int64)
    rc = _load().oracle_head_mapping(_p(a_d, ctypes.c_float), _p(a_t, ctypes.c_float), S, Hd, Ht, R,
                                     N, int(k), _p(mp, ctypes.c_int32), _p(ov, ctypes.c_int64))
    _check(rc, "oracle_head_mapping")
    return mp, ov
