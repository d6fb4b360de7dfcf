"""ctypes binding of include/sts.h. Argument marshalling only.

torch is used for device memory (outputs, workspace) and for the current HIP stream.

Workspaces: without a `workspace=` argument a call uses a cached scratch buffer per kind of
call (selection, attention, head mapping), device and stream, so calls that may overlap on
different streams never share scratch (the C interface leaves that to the caller).
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsts.so")

STS_SCORES_PROBS, STS_SCORES_LOGITS_LSE = 0, 1
STS_REDUCE_SUM, STS_REDUCE_MAX = 0, 1
STS_BF16, STS_F32 = 0, 1
KERNEL_KINDS = {"select_clear": 0, "select_agg": 1, "select_hist": 2, "select_rowpass": 3,
                "select_write": 4, "attn_sparse": 5, "attn_dense": 6, "attn_combine": 7, "select_block": 8,
                "headmap": 9, "select_small": 10, "select_local": 11, "select_pool": 12,
                "attn_probsum": 13, "select_fused": 14, "union_rows": 15, "select_band": 16}
KNOBS = {"attn_wgs_per_cu": 0, "select_spin_limit": 1, "probsum_wgs_per_cu": 2, "select_path": 3, "select_row_threads": 4}

# every symbol include/sts.h declares
EXPORTS = ["sts_select_workspace_bytes", "sts_attn_workspace_bytes", "sts_select", "sts_sparse_attn",
           "sts_dense_attn", "sts_strerror", "sts_version", "sts_prof_enable", "sts_prof_reset",
           "sts_prof_read", "sts_attn_plan", "sts_head_map", "sts_headmap_workspace_bytes",
           "sts_sparse_attn_static", "sts_set_knob", "sts_get_knob", "sts_union_rows"]
STS_STATIC_SCRATCH_BYTES = 8 << 20


class StsError(RuntimeError):
    pass


class SelectParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hd", ctypes.c_int32), ("Tq", ctypes.c_int32),
                ("N", ctypes.c_int32), ("Hq", ctypes.c_int32), ("k", ctypes.c_int32),
                ("scores", ctypes.c_void_p), ("lse", ctypes.c_void_p), ("head_map", ctypes.c_void_p),
                ("seq_lens", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("counts", ctypes.c_void_p),
                ("agg_out", ctypes.c_void_p), ("kind", ctypes.c_int32), ("reduce", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("k_head", ctypes.c_void_p), ("scores_bf16", ctypes.c_int32),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class AttnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Tq", ctypes.c_int32), ("Hq", ctypes.c_int32),
                ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32), ("N", ctypes.c_int32),
                ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64),
                ("kv_stride_n", ctypes.c_int64), ("indices", ctypes.c_void_p),
                ("counts", ctypes.c_void_p), ("kmax", ctypes.c_int32), ("head_map", ctypes.c_void_p),
                ("seq_lens", ctypes.c_void_p), ("scale", ctypes.c_float), ("out", ctypes.c_void_p),
                ("out_dtype", ctypes.c_int32), ("lse_out", ctypes.c_void_p),
                ("logits_out", ctypes.c_void_p), ("page_size", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("table_stride", ctypes.c_int32),
                ("num_pages", ctypes.c_int32), ("kv_stride_page", ctypes.c_int64),
                ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p), ("causal", ctypes.c_int32),
                ("logits_bf16", ctypes.c_int32), ("idx_stride_b", ctypes.c_int64), ("cnt_stride_b", ctypes.c_int64),
                ("weights_sum_out", ctypes.c_void_p), ("row_mask", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class UnionParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hd", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Tq", ctypes.c_int32),
                ("N", ctypes.c_int32), ("k", ctypes.c_int32), ("row_indices", ctypes.c_void_p),
                ("row_counts", ctypes.c_void_p), ("head_map", ctypes.c_void_p), ("pitch", ctypes.c_int32),
                ("indices", ctypes.c_void_p), ("row_mask", ctypes.c_void_p), ("counts", ctypes.c_void_p)]


class HeadmapParams(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int32), ("R", ctypes.c_int32), ("Hd", ctypes.c_int32), ("Ht", ctypes.c_int32),
                ("N", ctypes.c_int32), ("k", ctypes.c_int32), ("a_d", ctypes.c_void_p), ("a_t", ctypes.c_void_p),
                ("map", ctypes.c_void_p), ("overlap", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsts.so built in-tree. Fails loudly if it is missing (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise StsError(f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.sts_select_workspace_bytes.restype = ctypes.c_size_t
    lib.sts_select_workspace_bytes.argtypes = [ctypes.POINTER(SelectParams)]
    lib.sts_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.sts_attn_workspace_bytes.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_int]
    lib.sts_select.restype = ctypes.c_int
    lib.sts_select.argtypes = [ctypes.POINTER(SelectParams), ctypes.c_void_p]
    for f in (lib.sts_sparse_attn, lib.sts_dense_attn, lib.sts_sparse_attn_static):
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_void_p]
    lib.sts_strerror.restype = ctypes.c_char_p
    lib.sts_strerror.argtypes = [ctypes.c_int]
    lib.sts_version.restype = ctypes.c_int
    lib.sts_prof_enable.argtypes = [ctypes.c_int]
    lib.sts_prof_enable.restype = None
    lib.sts_prof_reset.restype = None
    lib.sts_prof_read.restype = ctypes.c_int
    lib.sts_prof_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
    lib.sts_headmap_workspace_bytes.restype = ctypes.c_size_t
    lib.sts_headmap_workspace_bytes.argtypes = [ctypes.POINTER(HeadmapParams)]
    lib.sts_head_map.restype = ctypes.c_int
    lib.sts_head_map.argtypes = [ctypes.POINTER(HeadmapParams), ctypes.c_void_p]
    lib.sts_attn_plan.restype = ctypes.c_int
    lib.sts_attn_plan.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_int] + [ctypes.POINTER(ctypes.c_int32)] * 3
    lib.sts_union_rows.restype = ctypes.c_int
    lib.sts_union_rows.argtypes = [ctypes.POINTER(UnionParams), ctypes.c_void_p]
    lib.sts_set_knob.restype = None
    lib.sts_set_knob.argtypes = [ctypes.c_int, ctypes.c_double]
    lib.sts_get_knob.restype = ctypes.c_double
    lib.sts_get_knob.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def exported_symbols() -> Dict[str, bool]:
    lib = load_library()
    return {name: hasattr(lib, name) for name in EXPORTS}


def sts_version() -> int:
    return int(load_library().sts_version())


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().sts_strerror(rc).decode()
        raise StsError(f"{what}: {msg} ({rc})")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    """Raw handle of torch's current stream on the current device (the cheap accessor: the
    Stream object behind torch.cuda.current_stream() costs several microseconds per call)."""
    import torch

    return torch._C._cuda_getCurrentRawStream(torch.cuda.current_device())


class PreparedCall:
    """A library call with its parameter block built once: calling the object enqueues the call
    again on torch's current stream with the same pointers (the tensors it was built from are kept
    alive here; the workspace is the one that was current when it was built, so use it on the
    stream it was prepared on). For serving loops that repeat a call on fixed buffers: the
    per-call cost on the host is one ctypes call."""

    def __init__(self, fn, params, what, result, keep):
        self._fn, self._p, self._what, self.result, self._keep = fn, params, what, result, keep
        self._ref = ctypes.byref(params)

    def __call__(self):
        rc = self._fn(self._ref, _stream())
        if rc != 0:
            _check(rc, self._what)
        return self.result


_ws_cache: Dict[Tuple[str, int, int], "object"] = {}


def _workspace(tag: str, nbytes: int, device):
    """A cached device scratch buffer (256-byte aligned by the torch allocator)."""
    import torch

    # one buffer per kind of call, device and stream: calls that may overlap (different streams)
    # never share scratch, calls on one stream are ordered anyway
    key = (tag, device.index if device.index is not None else torch.cuda.current_device(), _stream())
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < nbytes:
        buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


_i32_cache: Dict[tuple, ctypes.Array] = {}


def _host_i32(seq) -> ctypes.Array:
    """Host int32 array for a short list of ints (head maps, budgets); arrays are cached by value."""
    vals = tuple(seq.tolist() if hasattr(seq, "tolist") else seq)
    arr = _i32_cache.get(vals)
    if arr is None:
        if len(_i32_cache) > 256:
            _i32_cache.clear()
        arr = (ctypes.c_int32 * len(vals))(*[int(x) for x in vals])
        _i32_cache[vals] = arr
    return arr


def sts_select(scores, head_map, k: int, lse=None, seq_lens=None, kind: int = STS_SCORES_PROBS,
               reduce: int = STS_REDUCE_SUM, want_agg: bool = False, out=None, workspace=None,
               page_size: int = 1, k_head=None, prepare: bool = False):
    """scores [B,Hd,Tq,N] fp32 or bf16 (device), head_map [Hq] (host ints) -> (indices [B,Hq,k] int32,
    counts [B,Hq] int32, agg [B,Hd,N] fp32 or None). With page_size > 1, k counts blocks and the
    indices are block ids. k_head [Hd] (host ints, each <= k) gives every draft head its own
    budget. See sts_select in include/sts.h."""
    import torch

    lib = load_library()
    assert scores.is_cuda and scores.dtype in (torch.float32, torch.bfloat16) and scores.is_contiguous()
    B, Hd, Tq, N = scores.shape
    hm = _host_i32(head_map)
    Hq = len(hm)
    kh = None
    if k_head is not None:
        kh = _host_i32(k_head)
        assert len(kh) == Hd
    dev = scores.device
    if out is None:
        indices = torch.empty(B, Hq, k, dtype=torch.int32, device=dev)
        counts = torch.empty(B, Hq, dtype=torch.int32, device=dev)
    else:
        indices, counts = out
    agg = torch.empty(B, Hd, N, dtype=torch.float32, device=dev) if want_agg else None
    if lse is not None:
        assert lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous() and lse.shape == (B, Hd, Tq)
    if seq_lens is not None:
        assert seq_lens.is_cuda and seq_lens.dtype == torch.int32 and seq_lens.shape == (B,)
    p = SelectParams(B=B, Hd=Hd, Tq=Tq, N=N, Hq=Hq, k=int(k), scores=_ptr(scores), lse=_ptr(lse),
                     head_map=ctypes.cast(hm, ctypes.c_void_p), seq_lens=_ptr(seq_lens),
                     indices=_ptr(indices), counts=_ptr(counts), agg_out=_ptr(agg), kind=kind,
                     reduce=reduce, page_size=int(page_size),
                     k_head=ctypes.cast(kh, ctypes.c_void_p) if kh is not None else None,
                     scores_bf16=1 if scores.dtype == torch.bfloat16 else 0,
                     workspace=None, workspace_bytes=0)
    need = lib.sts_select_workspace_bytes(ctypes.byref(p))
    ws = workspace if workspace is not None else _workspace("select", need, dev)
    p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    if prepare:       # build once, launch many times (see PreparedCall)
        return PreparedCall(lib.sts_select, p, "sts_select", (indices, counts, agg),
                            (scores, lse, seq_lens, hm, kh, ws))
    _check(lib.sts_select(ctypes.byref(p), _stream()), "sts_select")
    return indices, counts, agg


def _attn_params(q, k, v, scale, indices, counts, head_map, seq_lens, out, lse_out, logits_out,
                 page_size=1, block_table=None, N=None, k_new=None, v_new=None, causal=True, row_mask=None):
    import torch

    assert q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous()
    assert k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16 and k.is_cuda and v.is_cuda
    B, Tq, Hq, d = q.shape
    assert v.shape == k.shape and v.stride() == k.stride() and k.stride(3) == 1 and k.shape[3] == d
    if block_table is None:
        # contiguous-per-sequence cache [B,Hkv,N,d] (any strides on the first three dims)
        Bk, Hkv, Nk, _ = k.shape
        assert Bk == B
        N = Nk if N is None else N
        sb, sh, sn, sp, npages, tstride = k.stride(0), k.stride(1), k.stride(2), 0, 0, 0
    else:
        # pool of pages [num_pages,Hkv,page,d] + table [B,T] of physical page ids
        npages, Hkv, pg, _ = k.shape
        assert pg == page_size and N is not None
        assert block_table.is_cuda and block_table.dtype == torch.int32 and block_table.is_contiguous()
        assert block_table.shape[0] == B
        sb, sh, sn, sp, tstride = 0, k.stride(1), k.stride(2), k.stride(0), block_table.shape[1]
    kmax = 0
    isb = csb = 0
    if indices is not None:
        # [B,Hq,kmax], rows contiguous; the batch stride may be wider (a slice of heads of a wider list)
        assert indices.is_cuda and indices.dtype == torch.int32 and indices.shape[:2] == (B, Hq)
        kmax = indices.shape[2]
        assert kmax == 0 or (indices.stride(2) == 1 and (Hq == 1 or indices.stride(1) == kmax))
        isb = indices.stride(0) if B > 1 else 0
    if counts is not None:
        assert counts.is_cuda and counts.dtype == torch.int32 and counts.shape == (B, Hq)
        assert Hq == 1 or counts.stride(1) == 1
        csb = counts.stride(0) if B > 1 else 0
    if seq_lens is not None:
        assert seq_lens.is_cuda and seq_lens.dtype == torch.int32 and seq_lens.shape == (B,)
    hm = _host_i32(head_map) if head_map is not None else None
    out_dtype = STS_BF16 if out.dtype == torch.bfloat16 else STS_F32
    if k_new is not None:
        for t in (k_new, v_new):
            assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and tuple(t.shape) == (B, Tq, Hkv, d)
    p = AttnParams(B=B, Tq=Tq, Hq=Hq, Hkv=Hkv, d=d, N=N, q=_ptr(q), k=_ptr(k), v=_ptr(v),
                   kv_stride_b=sb, kv_stride_h=sh, kv_stride_n=sn,
                   indices=_ptr(indices), counts=_ptr(counts), kmax=kmax,
                   head_map=ctypes.cast(hm, ctypes.c_void_p) if hm is not None else None,
                   seq_lens=_ptr(seq_lens), scale=float(scale), out=_ptr(out), out_dtype=out_dtype,
                   lse_out=_ptr(lse_out), logits_out=_ptr(logits_out), page_size=int(page_size),
                   block_table=_ptr(block_table), table_stride=tstride, num_pages=npages,
                   kv_stride_page=sp, k_new=_ptr(k_new), v_new=_ptr(v_new), causal=1 if causal else 0,
                   idx_stride_b=isb, cnt_stride_b=csb, workspace=None, workspace_bytes=0)
    if row_mask is not None:
        # uint16 words (torch.int16 storage is accepted: same bits), laid out like the indices
        assert indices is not None and row_mask.is_cuda and row_mask.element_size() == 2
        assert tuple(row_mask.shape) == tuple(indices.shape) and row_mask.stride() == indices.stride()
        p.row_mask = row_mask.data_ptr()
    return p, hm


def _run_attn(sparse: bool, q, k, v, scale, indices=None, counts=None, head_map=None, seq_lens=None,
              out=None, out_dtype=None, want_lse=True, want_logits=False, workspace=None,
              lse_out=None, logits_out=None, page_size=1, block_table=None, N=None,
              k_new=None, v_new=None, causal=True, weights_sum_out=None, static=False, row_mask=None,
              prepare=False):
    import torch

    lib = load_library()
    B, Tq, Hq, d = q.shape
    if N is None:
        assert block_table is None, "a paged cache needs the logical length bound N"
        N = k.shape[2]
    dev = q.device
    if out is None:
        out = torch.empty(B, Tq, Hq, d, dtype=out_dtype or torch.bfloat16, device=dev)
    lse = lse_out
    if lse is None and want_lse:
        lse = torch.empty(B, Hq, Tq, dtype=torch.float32, device=dev)
    logits = logits_out
    if logits is None and want_logits:
        # want_logits=True: fp32; a torch dtype (float32 or bfloat16) chooses the type of the dump
        ldt = want_logits if isinstance(want_logits, torch.dtype) else torch.float32
        logits = torch.empty(B, Hq, Tq, N, dtype=ldt, device=dev)
    assert lse is None or (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous()
                           and tuple(lse.shape) == (B, Hq, Tq))
    assert logits is None or (logits.is_cuda and logits.dtype in (torch.float32, torch.bfloat16)
                              and logits.is_contiguous() and tuple(logits.shape) == (B, Hq, Tq, N))
    p, _keep = _attn_params(q, k, v, scale, indices, counts, head_map, seq_lens, out, lse, logits,
                            page_size=page_size, block_table=block_table, N=N,
                            k_new=k_new, v_new=v_new, causal=causal, row_mask=row_mask)
    if static:      # the library's own scratch array: no workspace, nothing allocated by the call
        assert sparse and workspace is None
        _check(lib.sts_sparse_attn_static(ctypes.byref(p), _stream()), "sts_sparse_attn_static")
        return out, lse, logits
    need = lib.sts_attn_workspace_bytes(ctypes.byref(p), 1 if sparse else 0)
    ws = workspace if workspace is not None else _workspace("attn", need, dev)
    p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    p.logits_bf16 = 1 if (logits is not None and logits.dtype == torch.bfloat16) else 0
    if weights_sum_out is not None:
        w = weights_sum_out
        assert not sparse and w.is_cuda and w.dtype == torch.float32 and w.is_contiguous()
        assert tuple(w.shape) == (B, Hq, N)
        p.weights_sum_out = w.data_ptr()
        need = lib.sts_attn_workspace_bytes(ctypes.byref(p), 0)
        if workspace is None:
            ws = _workspace("attn", need, dev)
            p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    fn = lib.sts_sparse_attn if sparse else lib.sts_dense_attn
    if prepare:       # build once, launch many times (see PreparedCall)
        return PreparedCall(fn, p, "sts_sparse_attn" if sparse else "sts_dense_attn", (out, lse, logits),
                            (q, k, v, indices, counts, seq_lens, block_table, k_new, v_new, row_mask, weights_sum_out, _keep, ws))
    _check(fn(ctypes.byref(p), _stream()), "sts_sparse_attn" if sparse else "sts_dense_attn")
    return out, lse, logits


def sts_sparse_attn(q, k, v, indices, scale, counts=None, head_map=None, out=None, out_dtype=None,
                    want_lse=True, workspace=None, lse_out=None, page_size=1, block_table=None, N=None,
                    k_new=None, v_new=None, causal=True, row_mask=None, prepare=False):
    """Attention over the gathered rows indices[b,t,:counts[b,t]] of the full cache.
    q [B,Tq,Hq,d] bf16, k/v [B,Hkv,N,d] bf16 (strided ok) -> (out [B,Tq,Hq,d], lse [B,Hq,Tq]).
    row_mask (16-bit words shaped like indices): query row i attends only to entries with bit i.
    prepare=True returns a PreparedCall instead of launching."""
    r = _run_attn(True, q, k, v, scale, indices=indices, counts=counts, head_map=head_map,
                  out=out, out_dtype=out_dtype, want_lse=want_lse, workspace=workspace,
                  lse_out=lse_out, page_size=page_size, block_table=block_table, N=N,
                  k_new=k_new, v_new=v_new, causal=causal, row_mask=row_mask, prepare=prepare)
    if prepare:
        return r
    return r[0], r[1]


def sts_select_rows(scores, k: int, lse=None, seq_lens=None, kind: int = STS_SCORES_PROBS, out=None, workspace=None):
    """Per-row selection for prefill: every one of the Tq score rows of a draft head is ranked by
    itself. scores [B,Hd,Tq,N] -> (row_indices [B,Hd,Tq,k], row_counts [B,Hd,Tq]). Marshalling only:
    it is sts_select on the same memory viewed as [B, Hd*Tq, 1, N] with the identity head map
    (Hd*Tq <= 256)."""
    B, Hd, Tq, N = scores.shape
    assert Hd * Tq <= 256, "sts_select takes up to 256 heads: split the draft heads over several calls"
    idx, cnt, _ = sts_select(scores.view(B, Hd * Tq, 1, N), list(range(Hd * Tq)), k,
                             lse=None if lse is None else lse.view(B, Hd * Tq, 1), seq_lens=seq_lens, kind=kind,
                             out=None if out is None else (out[0].view(B, Hd * Tq, k), out[1].view(B, Hd * Tq)),
                             workspace=workspace)
    return idx.view(B, Hd, Tq, k), cnt.view(B, Hd, Tq)


def sts_union_rows(row_indices, row_counts, head_map, N: int, pitch: Optional[int] = None, out=None):
    """Per-row lists [B,Hd,Tq,k] (+ counts [B,Hd,Tq] or None) -> (indices [B,Hq,pitch] ascending union,
    row_mask [B,Hq,pitch] int16 storage of the 16-bit words, counts [B,Hq]). See sts_union_rows in
    include/sts.h."""
    import torch

    lib = load_library()
    assert row_indices.is_cuda and row_indices.dtype == torch.int32 and row_indices.is_contiguous()
    B, Hd, Tq, k = row_indices.shape
    if row_counts is not None:
        assert row_counts.is_cuda and row_counts.dtype == torch.int32 and row_counts.is_contiguous()
        assert tuple(row_counts.shape) == (B, Hd, Tq)
    hm = _host_i32(head_map)
    Hq = len(hm)
    pitch = min(Tq * k, N) if pitch is None else int(pitch)
    dev = row_indices.device
    if out is None:
        indices = torch.empty(B, Hq, pitch, dtype=torch.int32, device=dev)
        mask = torch.empty(B, Hq, pitch, dtype=torch.int16, device=dev)
        counts = torch.empty(B, Hq, dtype=torch.int32, device=dev)
    else:
        indices, mask, counts = out
    p = UnionParams(B=B, Hd=Hd, Hq=Hq, Tq=Tq, N=int(N), k=k, row_indices=_ptr(row_indices), row_counts=_ptr(row_counts),
                    head_map=ctypes.cast(hm, ctypes.c_void_p), pitch=pitch, indices=_ptr(indices), row_mask=_ptr(mask),
                    counts=_ptr(counts))
    _check(lib.sts_union_rows(ctypes.byref(p), _stream()), "sts_union_rows")
    return indices, mask, counts


def sts_sparse_attn_static(q, k, v, indices, scale, counts=None, head_map=None, out=None, out_dtype=None,
                           want_lse=True, lse_out=None, page_size=1, block_table=None, N=None,
                           k_new=None, v_new=None, causal=True):
    """sts_sparse_attn on the library's static scratch array (no workspace; the C call allocates
    nothing; pass `out` and `lse_out` so that this wrapper allocates nothing either). Shapes whose
    partial results exceed STS_STATIC_SCRATCH_BYTES raise StsError (workspace)."""
    out, lse, _ = _run_attn(True, q, k, v, scale, indices=indices, counts=counts, head_map=head_map,
                            out=out, out_dtype=out_dtype, want_lse=want_lse, lse_out=lse_out,
                            page_size=page_size, block_table=block_table, N=N,
                            k_new=k_new, v_new=v_new, causal=causal, static=True)
    return out, lse


def sts_dense_attn(q, k, v, scale, seq_lens=None, out=None, out_dtype=None, want_lse=True,
                   want_logits=False, workspace=None, lse_out=None, logits_out=None, page_size=1,
                   block_table=None, N=None, k_new=None, v_new=None, causal=True, weights_sum_out=None,
                   prepare=False):
    """Dense attention of the same kernel family -> (out, lse, logits [B,Hq,Tq,N] or None).
    want_logits: True (fp32 dump) or a torch dtype (float32 / bfloat16); logits_out: a buffer of
    either type. weights_sum_out: an fp32 [B,Hq,N] buffer that receives the attention weights
    summed over the Tq query rows (what sts_select aggregates the dump to; feed it to sts_select
    as probabilities with Tq = 1)."""
    return _run_attn(False, q, k, v, scale, seq_lens=seq_lens, out=out, out_dtype=out_dtype,
                     want_lse=want_lse, want_logits=want_logits, workspace=workspace,
                     lse_out=lse_out, logits_out=logits_out, page_size=page_size,
                     block_table=block_table, N=N, k_new=k_new, v_new=v_new, causal=causal,
                     weights_sum_out=weights_sum_out, prepare=prepare)


def sts_head_map(a_d, a_t, k: int, workspace=None):
    """Algorithm 1 on the GPU. a_d [S,Hd,R,N], a_t [S,Ht,R,N] fp32 attention-weight traces
    (device) -> (map [Ht] int32, overlap [Ht,Hd] int64). See sts_head_map in include/sts.h."""
    import torch

    lib = load_library()
    for t in (a_d, a_t):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.dim() == 4
    S, Hd, R, N = a_d.shape
    St, Ht, Rt, Nt = a_t.shape
    assert (St, Rt, Nt) == (S, R, N)
    dev = a_d.device
    mp = torch.empty(Ht, dtype=torch.int32, device=dev)
    ov = torch.empty(Ht, Hd, dtype=torch.int64, device=dev)
    p = HeadmapParams(S=S, R=R, Hd=Hd, Ht=Ht, N=N, k=int(k), a_d=_ptr(a_d), a_t=_ptr(a_t), map=_ptr(mp),
                      overlap=_ptr(ov), workspace=None, workspace_bytes=0)
    need = lib.sts_headmap_workspace_bytes(ctypes.byref(p))
    ws = workspace if workspace is not None else _workspace("headmap", need, dev)
    p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    _check(lib.sts_head_map(ctypes.byref(p), _stream()), "sts_head_map")
    return mp, ov


def attn_plan(q, k, sparse: bool, kmax: int = 0, head_map=None, page_size: int = 1) -> Dict[str, int]:
    """Launch geometry the library picks for a shape (reports only)."""
    lib = load_library()
    B, Tq, Hq, d = q.shape
    _, Hkv, N, _ = k.shape
    hm = _host_i32(head_map) if head_map is not None else None
    p = AttnParams(B=B, Tq=Tq, Hq=Hq, Hkv=Hkv, d=d, N=N, kv_stride_b=k.stride(0), kv_stride_h=k.stride(1),
                   kv_stride_n=k.stride(2), kmax=kmax, scale=1.0, page_size=int(page_size),
                   head_map=ctypes.cast(hm, ctypes.c_void_p) if hm is not None else None)
    s, u, nq = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib.sts_attn_plan(ctypes.byref(p), 1 if sparse else 0, ctypes.byref(s), ctypes.byref(u),
                             ctypes.byref(nq)), "sts_attn_plan")
    return {"num_splits": s.value, "units_per_batch": u.value, "query_tiles": nq.value}


def set_knob(name: str, value=None):
    """Set a tuning / test knob of the library (see sts_set_knob in include/sts.h); None restores
    the library's own rule."""
    load_library().sts_set_knob(KNOBS[name], float("nan") if value is None else float(value))


def get_knob(name: str) -> float:
    return float(load_library().sts_get_knob(KNOBS[name]))


def prof_enable(on: bool = True):
    load_library().sts_prof_enable(1 if on else 0)


def prof_reset():
    load_library().sts_prof_reset()


def prof_read() -> Dict[str, Tuple[int, float]]:
    """Per kernel kind: (launches, total milliseconds) since the last reset (synchronises)."""
    lib = load_library()
    res = {}
    for name, kind in KERNEL_KINDS.items():
        n, ms = ctypes.c_int32(), ctypes.c_double()
        _check(lib.sts_prof_read(kind, ctypes.byref(n), ctypes.byref(ms)), "sts_prof_read")
        res[name] = (n.value, ms.value)
    return res
