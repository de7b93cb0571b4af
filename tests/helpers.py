"""Helpers shared by the GPU parity tests (tests may use both the oracle and the library)."""
import numpy as np
import torch

from oracle import moe_oracle as orc
from paper_2303_06182_amd import workloads as wl

# Tolerances of the layer output against the fp64 oracle, as normalised max error
#   max_i |y_gpu - y_ref| / max_i |y_ref|
# (per-element relative error is meaningless near zero crossings of y).
TOL = {"bf16": 2e-2, "f32": 1e-5}
# A second gate beside it, on the whole compared block: RMS(y_gpu - y_ref) / RMS(y_ref).  The max-normalised
# error leaves room for a local defect (a K tile left out of one GEMM tile moves those outputs by a few per cent
# of max|y|, near the bar, not over it); the RMS of the bf16 rounding chain (H, Yp and y rounded once each)
# sits at 2-3e-3, so 6e-3 fails as soon as a visible share of the rows is off by more than rounding.
RMS_TOL = {"bf16": 6e-3, "f32": 3e-6}
# gate logits: fp32 accumulation of exact products vs. the fp64 sum rounded to fp32
LOGIT_RTOL, LOGIT_ATOL = 2e-6, 1e-7
# gate weights: fp32 expf / division vs. fp64
W_TOL = 2e-6
# smallest top-k decision margin the workloads are allowed to contain (>> accumulation noise)
MARGIN = 2.0 ** -20


def norm_max_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (denom if denom > 0 else 1.0))


def rms_rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = np.sqrt(np.mean(ref * ref))
    return float(np.sqrt(np.mean((got - ref) ** 2)) / (denom if denom > 0 else 1.0))


def worst_row_rms_rel_err(got, ref) -> float:
    """The same ratio per output row, largest over the rows (rows whose reference is all zero are skipped): a
    single token row computed from the wrong expert, tile or K range shows here even in a 65 536-row block."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.sqrt(np.mean((got - ref) ** 2, axis=1))
    den = np.sqrt(np.mean(ref * ref, axis=1))
    ok = den > 0
    return float((num[ok] / den[ok]).max()) if ok.any() else 0.0


def p999_rel_err(got, ref) -> float:
    """99.9th percentile of the per-element relative error over the elements that are not near a zero
    crossing (|y_ref| > 1e-3 max|y_ref|): reported beside the normalised max error, never the gate."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    big = np.abs(ref) > 1e-3 * np.abs(ref).max()
    if not big.any():
        return 0.0
    return float(np.percentile(np.abs(got[big] - ref[big]) / np.abs(ref[big]), 99.9))


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.numpy()


def margins(logits: np.ndarray, k: int) -> np.ndarray:
    """Per token: the smallest gap that decides the ordered top-k: between consecutive
    selected logits and between the k-th and the (k+1)-th."""
    s = -np.sort(-logits.astype(np.float64), axis=1)
    upto = min(k + 1, s.shape[1])
    if upto < 2:
        return np.full(s.shape[0], np.inf)
    return (s[:, :upto - 1] - s[:, 1:upto]).min(axis=1)


def guarded_inputs(w: wl.Workload, device="cpu", with_ffn_bias=False):
    """make_inputs + the margin guard: tokens whose top-k decision sits within MARGIN of a
    tie (by the oracle's logits) are redrawn.  Returns (inputs, number of redraws)."""
    inp = wl.make_inputs(w, device=device, with_ffn_bias=with_ffn_bias)
    wg_h = inp["wg"].cpu()
    gb_h = None if inp["gate_bias"] is None else inp["gate_bias"].cpu()

    def margin_fn(xrows):
        return margins(orc.gate_logits(xrows.cpu(), wg_h, gb_h), w.k)

    redraws = wl.clear_margins(w, inp["x"], margin_fn, delta=MARGIN)
    return inp, redraws
