"""Helpers shared by the GPU parity tests: tolerances and oracle calls on device tensors."""
import numpy as np
import torch

import oracle

# bf16 inputs, fp32 accumulation, against the fp64 oracle (the bar the benchmark spec fixes)
MAX_ABS = 1e-2
MEAN_ABS = 1e-3
LSE_ABS = 1e-3
# what the arithmetic leaves: the dumped logits are fp32 sums of exact bf16 products (observed
# 2-5e-7 at |s| ~ 2), the log-sum-exp goes through the hardware exp2/log2 (observed <= 2e-6)
LOGIT_TOL = 4e-6      # times (1 + |s|)
LSE_TIGHT = 5e-5
# and relative to the rms of the compared outputs (see check_attn)
REL_MAX = 4e-2
REL_MEAN = 5e-3


def bits(t: torch.Tensor) -> np.ndarray:
    return oracle.bf16_bits(t.detach().cpu())


def oracle_attn(q, k, v, scale, indices=None, counts=None, seq_lens=None, want_logits=False,
                batches=None, heads=None):
    return oracle.attn(bits(q), bits(k), bits(v), scale,
                       None if indices is None else indices.cpu().numpy(),
                       None if counts is None else counts.cpu().numpy(),
                       None if seq_lens is None else seq_lens.cpu().numpy(),
                       want_logits=want_logits, batches=batches, heads=heads)


def check_attn(out, lse, ref, sel=None, what=""):
    """Compare a GPU result with the oracle's within the stated tolerances. `sel` optionally
    restricts to (batch slice, head slice)."""
    o = out.float().cpu().numpy()
    l = lse.cpu().numpy()
    ro, rl = ref["out"], ref["lse"]
    if sel is not None:
        bs, hs = sel
        o, ro = o[bs][:, :, hs], ro[bs][:, :, hs]
        l, rl = l[bs][:, hs], rl[bs][:, hs]
    err = np.abs(o - ro)
    assert np.isfinite(o).all(), what
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"
    # The absolute bar says little when the outputs themselves are small (an average over
    # thousands of N(0, 0.5^2) value rows is of order 1e-2 or less), so the error is also held
    # against the scale of the compared outputs: the attention weights enter the PV product
    # rounded to bf16 (relative 2^-9 each) and everything else is fp32, which leaves errors of
    # about 1% of the outputs' rms at worst (measured over this suite: 1.2% max, 0.13% mean);
    # a bf16 output adds its own rounding, up to 2^-9 of the largest element.
    if ro.size:
        rms = float(np.sqrt(np.mean(ro.astype(np.float64) ** 2)))
        rounding = 2.0 ** -8 * float(np.abs(ro).max()) if out.dtype == torch.bfloat16 else 0.0
        assert err.max() <= REL_MAX * rms + rounding + 1e-6, f"{what}: max-abs {err.max():.3e} at output rms {rms:.3e}"
        assert err.mean() <= REL_MEAN * rms + rounding / 8 + 1e-7, f"{what}: mean-abs {err.mean():.3e} at output rms {rms:.3e}"
    fin = np.isfinite(rl)
    assert (np.isneginf(l) == np.isneginf(rl)).all(), what
    assert np.abs(l[fin] - rl[fin]).max(initial=0.0) <= LSE_ABS, f"{what}: lse {np.abs(l[fin] - rl[fin]).max():.3e}"
    assert (np.abs(l[fin] - rl[fin]) <= LSE_TIGHT * (1.0 + np.abs(rl[fin]))).all(), f"{what}: lse {np.abs(l[fin] - rl[fin]).max():.3e}"
    return float(err.max()), float(err.mean())


def check_logits(got, ref, what=""):
    """Dumped scaled logits against the oracle's: fp32 accumulation of exact products."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    bad = np.abs(got - ref) > LOGIT_TOL * (1.0 + np.abs(ref))
    assert not bad.any(), f"{what}: logits differ by up to {np.abs(got - ref).max():.3e}"


def stored_agg(o_agg, seq_lens):
    """What sts_select stores in agg_out for the oracle's aggregate: the same values up to each
    batch element's valid length, 0 past it (the interface's rule; the oracle aggregates all N)."""
    if seq_lens is None:
        return o_agg
    a = np.array(o_agg, copy=True)
    lens = np.asarray(seq_lens.cpu().numpy() if hasattr(seq_lens, "cpu") else seq_lens)
    for b in range(a.shape[0]):
        a[b, :, int(lens[b]):] = 0.0
    return a
