"""CPU oracle of the dynamically gated MoE layer -- TEST INFRASTRUCTURE ONLY.

Python face of ``moe_oracle.c`` (the slow loops, built with gcc) plus the few steps
whose definition is a single indexing expression.  Only tests, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this; the product path never does,
and this module never imports the GPU package.

Paper passages followed: gate = linear layer (Sec. 2.4); top-1/top-2 gating
(Sec. 2.3); dynamic gating = sort index + per-expert counts + reorder + split,
no drops, no placeholders, order restored by indexing (Sec. 5.1); static gating =
fixed capacity, first-empty-row dispatch mask, drops and zero padding (Sec. 3.2,
Sec. 5.1).

Every function takes host arrays (numpy, or torch CPU tensors in fp32 / bf16) and
returns numpy arrays; floating point results are fp64 except the gate logits
(fp32: the top-k decision is specified on fp32 logits).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (OpenMP, AVX2 so the binary runs on any recent host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.moe_oracle_route.restype = ctypes.c_int
        _lib.moe_oracle_static_slots.restype = ctypes.c_int
    return _lib


def _host(a):
    """-> (numpy array, dt) with dt = 0 for fp32 storage, 1 for bf16 bit patterns."""
    if a is None:
        return None, None
    try:
        import torch
        if isinstance(a, torch.Tensor):
            a = a.detach().cpu().contiguous()
            if a.dtype == torch.bfloat16:
                return a.view(torch.int16).numpy().view(np.uint16), 1
            return a.to(torch.float32).numpy(), 0
    except ImportError:  # pragma: no cover
        pass
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return a, 1
    return np.ascontiguousarray(a, dtype=np.float32), 0


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _same_dt(*dts):
    s = {d for d in dts if d is not None}
    if len(s) != 1:
        raise ValueError("oracle inputs must share one storage type")
    return s.pop()


def n_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS if set, else the host's cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return int(v.split(",")[0])
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


def gate_logits(x, wg, gate_bias=None) -> np.ndarray:
    """logits[t,e] = sum_d x[t,d] wg[e,d] + bias[e]; fp64 sum, rounded once to fp32."""
    xh, d0 = _host(x)
    wh, d1 = _host(wg)
    dt = _same_dt(d0, d1)
    T, D = xh.shape
    E = wh.shape[0]
    b = None if gate_bias is None else np.ascontiguousarray(_host(gate_bias)[0], dtype=np.float32)
    out = np.empty((T, E), dtype=np.float32)
    _load().moe_oracle_gate_logits(_p(xh), _p(wh), _p(b), T, D, E, dt, _p(out))
    return out


def topk(logits: np.ndarray, k: int, renormalize: bool = True):
    """-> (idx [T,k] int32, w [T,k] fp64); ties to the lowest expert index."""
    l = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = l.shape
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float64)
    _load().moe_oracle_topk(_p(l), T, E, k, int(bool(renormalize)), _p(idx), _p(w))
    return idx, w


def route(idx: np.ndarray, E: int):
    """-> counts [E], offsets [E+1], dst_row [T,k], src_tok [k*T]  (all int32)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    dst_row = np.empty((T, k), dtype=np.int32)
    src_tok = np.empty(T * k, dtype=np.int32)
    rc = _load().moe_oracle_route(_p(idx), T, E, k, _p(counts), _p(offsets), _p(dst_row), _p(src_tok))
    if rc != 0:
        raise ValueError("expert index out of range")
    return counts, offsets, dst_row, src_tok


def dispatch(x, src_tok: np.ndarray) -> np.ndarray:
    """xp[r,:] = x[src_tok[r],:]  -- a pure copy, returned as fp64."""
    xh, dt = _host(x)
    if dt == 1:
        xh = (xh.astype(np.uint32) << 16).view(np.float32)
    return xh[np.asarray(src_tok, dtype=np.int64)].astype(np.float64)


def expert_ffn(xp, offsets, w1, w2, b1=None, b2=None, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """yp[r,:] = FFN_e(xp[r,:]) for the expert e whose range [offsets[e], offsets[e+1]) holds r."""
    xh, d0 = _host(xp)
    w1h, d1 = _host(w1)
    w2h, d2 = _host(w2)
    b1h, d3 = _host(b1)
    b2h, d4 = _host(b2)
    dt = _same_dt(d0, d1, d2, d3, d4)
    N, D = xh.shape
    E, F, _ = w1h.shape
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    if rows is None:
        r, n = None, N
    else:
        r = np.ascontiguousarray(rows, dtype=np.int32)
        n = int(r.size)
    out = np.empty((n, D), dtype=np.float64)
    _load().moe_oracle_expert_ffn_rows(_p(xh), _p(off), E, _p(w1h), _p(w2h), _p(b1h), _p(b2h),
                                       _p(r), n, D, F, dt, _p(out))
    return out


def combine(yp: np.ndarray, dst_row: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y[t,:] = sum_j (in order j = 0..k-1) w[t,j] * yp[dst_row[t,j],:]   (fp64)."""
    yp = np.asarray(yp, dtype=np.float64)
    T, k = dst_row.shape
    y = np.zeros((T, yp.shape[1]), dtype=np.float64)
    for j in range(k):
        y += np.asarray(w, dtype=np.float64)[:, j:j + 1] * yp[np.asarray(dst_row)[:, j].astype(np.int64)]
    return y


def layer_tokens(x, w1, w2, idx, w, tokens=None, b1=None, b2=None, keep=None) -> np.ndarray:
    """y rows for the listed tokens (all when None) given the routing (idx, w)."""
    xh, d0 = _host(x)
    w1h, d1 = _host(w1)
    w2h, d2 = _host(w2)
    b1h, d3 = _host(b1)
    b2h, d4 = _host(b2)
    dt = _same_dt(d0, d1, d2, d3, d4)
    T, D = xh.shape
    F = w1h.shape[1]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    k = idx.shape[1]
    w = np.ascontiguousarray(w, dtype=np.float64)
    kp = None if keep is None else np.ascontiguousarray(keep, dtype=np.uint8)
    if tokens is None:
        tk, n = None, T
    else:
        tk = np.ascontiguousarray(tokens, dtype=np.int32)
        n = int(tk.size)
    y = np.empty((n, D), dtype=np.float64)
    _load().moe_oracle_layer_tokens(_p(xh), _p(w1h), _p(w2h), _p(b1h), _p(b2h), _p(idx), _p(w), _p(kp),
                                    _p(tk), n, D, F, k, dt, _p(y))
    return y


def layer(x, wg, w1, w2, k: int, gate_bias=None, b1=None, b2=None, renormalize: bool = True,
          tokens=None) -> dict:
    """The whole dynamically gated layer.  Returns logits, idx, w, counts, offsets,
    dst_row, src_tok and y (rows of `tokens`, or all)."""
    logits = gate_logits(x, wg, gate_bias)
    idx, w = topk(logits, k, renormalize)
    counts, offsets, dst_row, src_tok = route(idx, logits.shape[1])
    y = layer_tokens(x, w1, w2, idx, w, tokens=tokens, b1=b1, b2=b2)
    return dict(logits=logits, idx=idx, w=w, counts=counts, offsets=offsets,
                dst_row=dst_row, src_tok=src_tok, y=y)


def static_slots(idx: np.ndarray, E: int, capacity: int):
    """-> (slot [T,k] int32 (-1 = dropped), keep [T,k] uint8, dropped count)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    slot = np.empty((T, k), dtype=np.int32)
    keep = np.empty((T, k), dtype=np.uint8)
    dropped = _load().moe_oracle_static_slots(_p(idx), T, E, k, int(capacity), _p(slot), _p(keep))
    return slot, keep, int(dropped)


def static_layer(x, wg, w1, w2, k: int, capacity: int, gate_bias=None, b1=None, b2=None,
                 renormalize: bool = True, tokens=None) -> dict:
    """Static-capacity layer: same gate and weights, assignments beyond an expert's
    capacity contribute nothing (weights are NOT renormalised after a drop)."""
    logits = gate_logits(x, wg, gate_bias)
    idx, w = topk(logits, k, renormalize)
    slot, keep, dropped = static_slots(idx, logits.shape[1], capacity)
    y = layer_tokens(x, w1, w2, idx, w, tokens=tokens, b1=b1, b2=b2, keep=keep)
    return dict(logits=logits, idx=idx, w=w, slot=slot, keep=keep, dropped=dropped, y=y)


def static_masks(idx: np.ndarray, w: np.ndarray, E: int, capacity: int):
    """The paper's dispatch-mask form of static gating (Sec. 5.1): E masks of shape
    (S, capacity); token i assigned to expert e marks column i of the first empty row of
    mask e, i.e. mask[e, i, row] = 1.  Returns (dispatch_mask [E,S,cap] of 0/1,
    combine_weights [E,S,cap] = mask * gate weight).  Dense -- tiny inputs only."""
    slot, keep, _ = static_slots(idx, E, capacity)
    T, k = idx.shape
    m = np.zeros((E, T, capacity), dtype=np.float64)
    cw = np.zeros((E, T, capacity), dtype=np.float64)
    for t in range(T):
        for j in range(k):
            if keep[t, j]:
                m[idx[t, j], t, slot[t, j]] = 1.0
                cw[idx[t, j], t, slot[t, j]] = w[t, j]
    return m, cw


def capacity_paper(C: float, S: int) -> int:
    """Rows per expert in the paper's convention: capacity factor times the number of
    tokens S (Sec. 3, Sec. 5.1: S = 6, C = 0.5 gives 3)."""
    return int(np.ceil(C * S - 1e-9))


def capacity_share(cf: float, T: int, E: int, k: int) -> int:
    """Rows per expert in the per-expert-share convention: cf * k*T / E, rounded up."""
    return int(np.ceil(cf * k * T / E - 1e-9))
