"""Seeded synthetic inputs for the dynamically gated MoE layer.

This module only *draws numbers*: it holds no part of the layer's arithmetic
(no gate product, no routing, no FFN), so both the CPU oracle's tests and the
GPU path's tests can take their inputs from it without sharing any method code.

The paper evaluates trained LM and MT MoE checkpoints on text corpora (its
experimental-setup table gives token dim 1024 / hidden 4096 / 512 experts for
the LM and 2048 / 8192 / 128 for the MT model, top-2 gating).  None of that data
is used here: the five workloads below take from the paper only the layer shapes
and the load structure (skewed but mostly dense expert use for the LM and the MT
encoder, mostly idle experts for a decoder step).

Generator: counter based.  Element i of stream s of seed z is

    h  = splitmix64_finalizer(i + GOLDEN * (z * 64 + s + 1))
    u1 = (high 32 bits of h + 0.5) / 2**32,  u2 = (low 32 bits of h + 0.5) / 2**32
    n  = sqrt(-2 ln u1) * cos(2 pi u2)                      (Box-Muller, fp64)

so any slice of any tensor can be drawn on its own, on the host or on the GPU.
The integer part is exact on every device; the fp64 transcendental part may
differ in the last bit between devices, so a test draws its inputs ONCE and
copies them to wherever they are needed.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import torch

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# streams (one per tensor of the layer)
STREAM_X, STREAM_WG, STREAM_W1, STREAM_W2, STREAM_PI, STREAM_B1, STREAM_B2 = range(7)

# Standard deviation of an unbiased gate logit for x ~ N(0, 0.02), wg ~ N(0, 1/sqrt(D)):
# 0.02 * D**-0.5 * sqrt(D) = 0.02, whatever D is.  The Zipf offsets are scaled by it.
LOGIT_STD = 0.02


def _s64(v: int) -> int:
    """Python int (mod 2**64) -> the same bits as a signed 64-bit value."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(z: torch.Tensor, n: int) -> torch.Tensor:
    """Logical shift right of int64 lanes (torch's >> is arithmetic)."""
    return (z >> n) & ((1 << (64 - n)) - 1)


def _hash64(counter: torch.Tensor, key: int) -> torch.Tensor:
    z = counter + _s64(_GOLDEN * (key + 1))
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def _key(seed: int, stream: int, attempt: int = 0) -> int:
    return (seed * 64 + stream) * 4096 + attempt


def uniform_bits(seed: int, stream: int, start: int, n: int, device, attempt: int = 0) -> torch.Tensor:
    """n int64 hashes for counters start..start+n-1."""
    c = torch.arange(start, start + n, dtype=torch.int64, device=device)
    return _hash64(c, _key(seed, stream, attempt))


def _normal_from_hash(h: torch.Tensor) -> torch.Tensor:
    hi = _lsr(h, 32).to(torch.float64)
    lo = (h & 0xFFFFFFFF).to(torch.float64)
    u1 = (hi + 0.5) * (1.0 / 4294967296.0)
    u2 = (lo + 0.5) * (1.0 / 4294967296.0)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def normal(seed: int, stream: int, shape, std: float, dtype: torch.dtype, device="cpu",
           start: int = 0, attempt: int = 0, chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of the given shape with N(0, std) entries, drawn from counters
    start .. start+numel-1 of (seed, stream), rounded once (RNE) to dtype."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    for a in range(0, n, chunk):
        m = min(chunk, n - a)
        h = uniform_bits(seed, stream, start + a, m, device, attempt)
        out[a:a + m] = (_normal_from_hash(h) * std).to(dtype)
    return out.view(*shape)


def permutation(seed: int, stream: int, n: int) -> torch.Tensor:
    """Seeded permutation of 0..n-1 (always drawn on the host)."""
    h = uniform_bits(seed, stream, 0, n, "cpu")
    return torch.argsort(h, stable=True)


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # "f32" | "bf16": storage type of x, weights and y
    T: int
    D: int
    F: int
    E: int
    k: int = 2
    zipf_s: float = 0.0     # exponent of the per-expert popularity offset (0 = none)
    zipf_c: float = 0.0     # offset scale in units of LOGIT_STD
    gate_scale: float = 1.0  # multiplies wg ("sharp gate" test variant: 100)
    seed: int = 0

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five workloads (shapes and load structure from the benchmark definition).
CONFIGS: Dict[str, Workload] = {
    "tiny_f32": Workload("tiny_f32", "f32", T=512, D=512, F=2048, E=8, seed=1000),
    "lm": Workload("lm", "bf16", T=8192, D=1024, F=4096, E=64, zipf_s=0.8, zipf_c=0.25, seed=2000),
    "mt_encoder": Workload("mt_encoder", "bf16", T=16384, D=2048, F=8192, E=16, seed=3000),
    "mt_decoder": Workload("mt_decoder", "bf16", T=64, D=2048, F=8192, E=128, seed=4000),
    "skewed_large": Workload("skewed_large", "bf16", T=65536, D=2048, F=8192, E=128,
                             zipf_s=1.2, zipf_c=0.5, seed=5000),
}
CONFIG_ORDER = ["tiny_f32", "lm", "mt_encoder", "mt_decoder", "skewed_large"]


def zipf_bias(w: Workload) -> Optional[torch.Tensor]:
    """Per-expert gate offset  bias[pi(r)] = -s * c * LOGIT_STD * ln(r),  r = 1..E the
    popularity rank and pi a seeded permutation, so the hot experts are scattered
    over the expert ids.  None when the workload has no skew."""
    if w.zipf_s == 0.0:
        return None
    pi = permutation(w.seed, STREAM_PI, w.E)
    r = torch.arange(1, w.E + 1, dtype=torch.float64)
    b = torch.empty(w.E, dtype=torch.float64)
    b[pi] = -w.zipf_s * w.zipf_c * LOGIT_STD * torch.log(r)
    return b.to(torch.float32)


def make_inputs(w: Workload, device="cpu", with_ffn_bias: bool = False) -> Dict[str, Optional[torch.Tensor]]:
    """Draw x [T,D], wg [E,D], gate_bias [E] (fp32) or None, w1 [E,F,D], w2 [E,D,F]
    (and b1 [E,F], b2 [E,D] when asked) on `device` in the workload's storage type."""
    dt = w.torch_dtype
    out: Dict[str, Optional[torch.Tensor]] = {}
    out["x"] = normal(w.seed, STREAM_X, (w.T, w.D), 0.02, dt, device)
    out["wg"] = normal(w.seed, STREAM_WG, (w.E, w.D), w.gate_scale / math.sqrt(w.D), dt, device)
    gb = zipf_bias(w)
    out["gate_bias"] = None if gb is None else gb.to(device)
    out["w1"] = normal(w.seed, STREAM_W1, (w.E, w.F, w.D), 0.02, dt, device)
    out["w2"] = normal(w.seed, STREAM_W2, (w.E, w.D, w.F), 0.02, dt, device)
    if with_ffn_bias:
        out["b1"] = normal(w.seed, STREAM_B1, (w.E, w.F), 0.02, dt, device)
        out["b2"] = normal(w.seed, STREAM_B2, (w.E, w.D), 0.02, dt, device)
    else:
        out["b1"] = None
        out["b2"] = None
    return out


def decode_steps(w: Workload, n_steps: int, rho: float = 0.9, device="cpu") -> List[torch.Tensor]:
    """A synthetic sequence of decode steps for the expert-buffering workload: n_steps token
    batches x_s [T,D] whose rows drift slowly (per element an AR(1) process of correlation rho
    and the same marginal N(0, 0.02^2) as make_inputs' x), so that consecutive steps activate
    overlapping sets of experts -- the temporal locality the paper's decoder traces show
    (Sec. 6, "Cache Management").  Step 0 is make_inputs' x.  The recursion runs in fp32 and
    every step is rounded once to the storage type."""
    dt = w.torch_dtype
    cur = normal(w.seed, STREAM_X, (w.T, w.D), 0.02, torch.float32, device)
    out = [cur.to(dt)]
    for s in range(1, n_steps):
        noise = normal(w.seed, STREAM_X, (w.T, w.D), 0.02, torch.float32, device, attempt=1000 + s)
        cur = rho * cur + math.sqrt(1.0 - rho * rho) * noise
        out.append(cur.to(dt))
    return out


def redraw_rows(w: Workload, x: torch.Tensor, rows: torch.Tensor, attempt: int) -> None:
    """Replace the given token rows of x in place by fresh draws (sub-stream `attempt` >= 1,
    same counters).  Used by tests to move tokens whose top-k decision would sit within
    accumulation-order noise of a tie."""
    for t in rows.tolist():
        x[t] = normal(w.seed, STREAM_X, (w.D,), 0.02, x.dtype, x.device,
                      start=t * w.D, attempt=attempt)


def clear_margins(w: Workload, x: torch.Tensor, margin_fn, delta: float = 2.0 ** -20,
                  max_attempts: int = 16) -> int:
    """Redraw token rows until every token's decision margin is at least delta.
    margin_fn(rows_of_x) -> one margin per given row; it is supplied by the caller (how a
    margin is computed is the caller's business, this module only redraws).  Returns how
    many token draws were replaced."""
    rows = torch.arange(x.shape[0])
    total = 0
    for attempt in range(1, max_attempts + 1):
        m = torch.as_tensor(margin_fn(x[rows.to(x.device)]))
        rows = rows[(m < delta).cpu()]
        if rows.numel() == 0:
            return total
        total += int(rows.numel())
        redraw_rows(w, x, rows, attempt)
    raise RuntimeError("margin guard did not converge")
