"""Thin Python binding of libmoe355 (include/moe.h): argument marshalling only.

Every step of the layer runs in the library's HIP kernels; torch is used for device
memory (tensors own the buffers) and for the current stream.  If the library has not been
built the import of this module's functions raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe355.so")

MOE_OK = 0
MOE_ERR_INVALID_ARG = -1
MOE_ERR_UNSUPPORTED = -2
MOE_ERR_WORKSPACE = -3
MOE_ERR_HIP = -4
MOE_DTYPE_F32 = 0
MOE_DTYPE_BF16 = 1
MOE_STATIC_EINSUM = 0
MOE_STATIC_INDEXED = 1
MOE_CAPACITY_PAPER = 0
MOE_CAPACITY_SHARE = 1

EXPORTS = [
    "moe_create", "moe_destroy", "moe_last_error", "moe_workspace_bytes", "moe_static_workspace_bytes",
    "moe_capacity", "moe_gate_topk", "moe_route_counts", "moe_dispatch", "moe_expert_ffn", "moe_combine",
    "moe_layer_forward", "moe_layer_forward_static", "moe_profile_begin", "moe_profile_end", "moe_profile_name",
    "moe_cache_policy_create", "moe_cache_policy_destroy", "moe_cache_policy_reset", "moe_cache_policy_step",
    "moe_cache_policy_stats", "moe_expert_cache_bytes", "moe_expert_cache_create", "moe_expert_cache_destroy",
    "moe_expert_cache_reset", "moe_expert_cache_stats", "moe_layer_forward_buffered",
    "moe_placement_greedy", "moe_placement_anticorrelation", "moe_placement_loads",
    "moe_quantize_e4m3", "moe_expert_ffn_w8", "moe_layer_forward_w8",
    "moe_mxfp4_scale_bytes", "moe_quantize_mxfp4", "moe_expert_ffn_w4", "moe_layer_forward_w4",
    "moe_expert_cache_bytes_q", "moe_expert_cache_create_q", "moe_layer_forward_noalloc",
]
MOE_NOALLOC_SCRATCH_BYTES = 8 * 1024 * 1024


class MoeConfig(ctypes.Structure):
    _fields_ = [("T_max", ctypes.c_int32), ("D", ctypes.c_int32), ("F", ctypes.c_int32), ("E", ctypes.c_int32),
                ("k", ctypes.c_int32), ("dtype", ctypes.c_int32), ("renormalize", ctypes.c_int32)]


class MoeRouting(ctypes.Structure):
    _fields_ = [("logits", ctypes.c_void_p), ("topk_idx", ctypes.c_void_p), ("topk_w", ctypes.c_void_p),
                ("counts", ctypes.c_void_p), ("offsets", ctypes.c_void_p), ("dst_row", ctypes.c_void_p),
                ("src_tok", ctypes.c_void_p)]


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libmoe355 error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libmoe355.so (built by paper_2303_06182_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libmoe355.so is not built (run `python -m paper_2303_06182_amd.build`); "
                           "there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.moe_create.argtypes = [ctypes.POINTER(MoeConfig), ctypes.POINTER(vp)]
    lib.moe_create.restype = ctypes.c_int
    lib.moe_destroy.argtypes = [vp]
    lib.moe_destroy.restype = ctypes.c_int
    lib.moe_last_error.argtypes = []
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_workspace_bytes.argtypes = [vp]
    lib.moe_workspace_bytes.restype = i64
    lib.moe_static_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.moe_static_workspace_bytes.restype = i64
    lib.moe_capacity.argtypes = [i32, i32, i32, ctypes.c_double, i32]
    lib.moe_capacity.restype = i32
    lib.moe_gate_topk.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, i64, vp]
    lib.moe_gate_topk.restype = ctypes.c_int
    lib.moe_route_counts.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, i64, vp]
    lib.moe_route_counts.restype = ctypes.c_int
    lib.moe_dispatch.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.moe_dispatch.restype = ctypes.c_int
    lib.moe_expert_ffn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i64, vp]
    lib.moe_expert_ffn.restype = ctypes.c_int
    lib.moe_combine.argtypes = [vp, vp, vp, vp, i32, vp, vp]
    lib.moe_combine.restype = ctypes.c_int
    lib.moe_layer_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.POINTER(MoeRouting), vp, i64, vp]
    lib.moe_layer_forward.restype = ctypes.c_int
    lib.moe_layer_forward_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.POINTER(MoeRouting), vp]
    lib.moe_layer_forward_noalloc.restype = ctypes.c_int
    lib.moe_layer_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp,
                                             ctypes.POINTER(MoeRouting), vp, i64, vp]
    lib.moe_layer_forward_static.restype = ctypes.c_int
    lib.moe_profile_begin.argtypes = [vp]
    lib.moe_profile_begin.restype = ctypes.c_int
    lib.moe_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32)]
    lib.moe_profile_end.restype = ctypes.c_int
    lib.moe_profile_name.argtypes = [vp, i32]
    lib.moe_profile_name.restype = ctypes.c_char_p
    pi32, pi64 = ctypes.POINTER(i32), ctypes.POINTER(i64)
    lib.moe_cache_policy_create.argtypes = [i32, i32, ctypes.POINTER(vp)]
    lib.moe_cache_policy_create.restype = ctypes.c_int
    lib.moe_cache_policy_destroy.argtypes = [vp]
    lib.moe_cache_policy_destroy.restype = ctypes.c_int
    lib.moe_cache_policy_reset.argtypes = [vp]
    lib.moe_cache_policy_reset.restype = ctypes.c_int
    lib.moe_cache_policy_step.argtypes = [vp, pi32, pi32, pi32, pi32, i32, pi32, pi32]
    lib.moe_cache_policy_step.restype = ctypes.c_int
    lib.moe_cache_policy_stats.argtypes = [vp, pi64, pi64, pi32]
    lib.moe_cache_policy_stats.restype = ctypes.c_int
    lib.moe_expert_cache_bytes.argtypes = [vp, i32]
    lib.moe_expert_cache_bytes.restype = i64
    lib.moe_expert_cache_create.argtypes = [vp, i32, vp, vp, vp, i64, ctypes.POINTER(vp)]
    lib.moe_expert_cache_create.restype = ctypes.c_int
    lib.moe_expert_cache_destroy.argtypes = [vp]
    lib.moe_expert_cache_destroy.restype = ctypes.c_int
    lib.moe_expert_cache_reset.argtypes = [vp]
    lib.moe_expert_cache_reset.restype = ctypes.c_int
    lib.moe_expert_cache_stats.argtypes = [vp, pi64, pi64, pi64, pi64]
    lib.moe_expert_cache_stats.restype = ctypes.c_int
    lib.moe_layer_forward_buffered.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.POINTER(MoeRouting), vp,
                                               i64, vp]
    lib.moe_layer_forward_buffered.restype = ctypes.c_int
    pf, pd = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    lib.moe_placement_greedy.argtypes = [pf, i32, i32, i32, pi32]
    lib.moe_placement_greedy.restype = ctypes.c_int
    lib.moe_placement_anticorrelation.argtypes = [pf, i32, i32, i32, ctypes.c_double, pi32]
    lib.moe_placement_anticorrelation.restype = ctypes.c_int
    lib.moe_placement_loads.argtypes = [pf, i32, i32, pi32, i32, pd, pd]
    lib.moe_placement_loads.restype = ctypes.c_int
    lib.moe_quantize_e4m3.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.moe_quantize_e4m3.restype = ctypes.c_int
    lib.moe_expert_ffn_w8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i64, vp]
    lib.moe_expert_ffn_w8.restype = ctypes.c_int
    lib.moe_layer_forward_w8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.POINTER(MoeRouting),
                                         vp, i64, vp]
    lib.moe_layer_forward_w8.restype = ctypes.c_int
    lib.moe_mxfp4_scale_bytes.argtypes = [i32, i32]
    lib.moe_mxfp4_scale_bytes.restype = i64
    lib.moe_quantize_mxfp4.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.moe_quantize_mxfp4.restype = ctypes.c_int
    lib.moe_expert_ffn_w4.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i64, vp]
    lib.moe_expert_ffn_w4.restype = ctypes.c_int
    lib.moe_layer_forward_w4.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.POINTER(MoeRouting),
                                         vp, i64, vp]
    lib.moe_layer_forward_w4.restype = ctypes.c_int
    lib.moe_expert_cache_bytes_q.argtypes = [vp, i32, i32]
    lib.moe_expert_cache_bytes_q.restype = i64
    lib.moe_expert_cache_create_q.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i64, ctypes.POINTER(vp)]
    lib.moe_expert_cache_create_q.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != MOE_OK:
        raise MoeError(rc, load_library().moe_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def moe_capacity(T: int, E: int, k: int, cf: float, convention: int = MOE_CAPACITY_SHARE) -> int:
    c = load_library().moe_capacity(T, E, k, cf, convention)
    if c < 0:
        _check(c)
    return c


class MoeLayer:
    """A handle (moe_create) plus a workspace tensor.  Methods mirror the C entry points and
    only marshal arguments; outputs are allocated by the caller or, for convenience, here
    (torch.empty) before the call."""

    def __init__(self, T_max: int, D: int, F: int, E: int, k: int = 2, dtype: str = "bf16",
                 renormalize: bool = True, device: str = "cuda:0", alloc_workspace: bool = True):
        self.lib = load_library()
        self.cfg = MoeConfig(T_max, D, F, E, k, MOE_DTYPE_BF16 if dtype == "bf16" else MOE_DTYPE_F32,
                             int(renormalize))
        self.T_max, self.D, self.F, self.E, self.k = T_max, D, F, E, k
        self.dtype = dtype
        self.torch_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.device = torch.device(device)
        h = ctypes.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.lib.moe_create(ctypes.byref(self.cfg), ctypes.byref(h)))
        self.h = h
        self.workspace_bytes = int(self.lib.moe_workspace_bytes(self.h))
        self.workspace = None
        if alloc_workspace:
            self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.device)

    def __del__(self):
        try:
            if getattr(self, "h", None):
                self.lib.moe_destroy(self.h)
                self.h = None
        except Exception:
            pass

    # -- helpers ---------------------------------------------------------------------------
    def _ws(self):
        if self.workspace is None:
            return None, 0
        return _ptr(self.workspace), self.workspace.numel()

    def _new(self, shape, dtype):
        return torch.empty(shape, dtype=dtype, device=self.device)

    def empty_routing(self, T: int) -> dict:
        return dict(logits=self._new((T, self.E), torch.float32), topk_idx=self._new((T, self.k), torch.int32),
                    topk_w=self._new((T, self.k), torch.float32), counts=self._new((self.E,), torch.int32),
                    offsets=self._new((self.E + 1,), torch.int32), dst_row=self._new((T, self.k), torch.int32),
                    src_tok=self._new((T * self.k,), torch.int32))

    @staticmethod
    def _routing_struct(r: Optional[dict]):
        if r is None:
            return None
        s = MoeRouting()
        for name in ("logits", "topk_idx", "topk_w", "counts", "offsets", "dst_row", "src_tok"):
            t = r.get(name)
            setattr(s, name, None if t is None else t.data_ptr())
        return ctypes.byref(s)

    # -- the entry points ------------------------------------------------------------------
    def moe_gate_topk(self, x, wg, gate_bias=None, logits_out=None, topk_idx=None, topk_w=None):
        T = x.shape[0]
        if logits_out is None:
            logits_out = self._new((T, self.E), torch.float32)
        if topk_idx is None:
            topk_idx = self._new((T, self.k), torch.int32)
        if topk_w is None:
            topk_w = self._new((T, self.k), torch.float32)
        ws, wsb = self._ws()
        _check(self.lib.moe_gate_topk(self.h, _ptr(x), _ptr(wg), _ptr(gate_bias), T, _ptr(logits_out),
                                      _ptr(topk_idx), _ptr(topk_w), ws, wsb, _stream()))
        return logits_out, topk_idx, topk_w

    def moe_route_counts(self, topk_idx):
        T = topk_idx.shape[0]
        counts = self._new((self.E,), torch.int32)
        offsets = self._new((self.E + 1,), torch.int32)
        dst_row = self._new((T, self.k), torch.int32)
        src_tok = self._new((T * self.k,), torch.int32)
        ws, wsb = self._ws()
        _check(self.lib.moe_route_counts(self.h, _ptr(topk_idx), T, _ptr(counts), _ptr(offsets), _ptr(dst_row),
                                         _ptr(src_tok), ws, wsb, _stream()))
        return counts, offsets, dst_row, src_tok

    def moe_dispatch(self, x, dst_row):
        T = x.shape[0]
        xp = self._new((T * self.k, self.D), self.torch_dtype)
        _check(self.lib.moe_dispatch(self.h, _ptr(x), _ptr(dst_row), T, _ptr(xp), _stream()))
        return xp

    def moe_expert_ffn(self, xp, offsets, w1, w2, b1=None, b2=None):
        n_rows = xp.shape[0]
        yp = self._new((n_rows, self.D), self.torch_dtype)
        ws, wsb = self._ws()
        _check(self.lib.moe_expert_ffn(self.h, _ptr(xp), _ptr(offsets), _ptr(w1), _ptr(w2), _ptr(b1), _ptr(b2),
                                       n_rows, _ptr(yp), ws, wsb, _stream()))
        return yp

    def moe_combine(self, yp, dst_row, topk_w):
        T = dst_row.shape[0]
        y = self._new((T, self.D), self.torch_dtype)
        _check(self.lib.moe_combine(self.h, _ptr(yp), _ptr(dst_row), _ptr(topk_w), T, _ptr(y), _stream()))
        return y

    def moe_layer_forward(self, x, wg, w1, w2, gate_bias=None, b1=None, b2=None, y=None, routing_out=None):
        T = x.shape[0]
        if y is None:
            y = self._new((T, self.D), self.torch_dtype)
        ws, wsb = self._ws()
        _check(self.lib.moe_layer_forward(self.h, _ptr(x), _ptr(wg), _ptr(gate_bias), _ptr(w1), _ptr(w2), _ptr(b1),
                                          _ptr(b2), T, _ptr(y), self._routing_struct(routing_out), ws, wsb,
                                          _stream()))
        return y

    def moe_layer_forward_noalloc(self, x, wg, w1, w2, y, gate_bias=None, b1=None, b2=None, routing_out=None):
        """moe_layer_forward on the library's own scratch array: no workspace, and nothing is allocated
        here either (the caller brings y and the routing arrays)."""
        _check(self.lib.moe_layer_forward_noalloc(self.h, _ptr(x), _ptr(wg), _ptr(gate_bias), _ptr(w1), _ptr(w2),
                                                  _ptr(b1), _ptr(b2), x.shape[0], _ptr(y),
                                                  self._routing_struct(routing_out), _stream()))
        return y

    def moe_quantize_e4m3(self, w):
        """w [E, rows, cols] -> (q uint8 [E, rows * cols] in the library's blocked layout, scale [E] fp32)."""
        E, rows, cols = w.shape
        q = self._new((E, rows * cols), torch.uint8)
        scale = self._new((E,), torch.float32)
        _check(self.lib.moe_quantize_e4m3(self.h, _ptr(w), E, rows, cols, _ptr(q), _ptr(scale), _stream()))
        return q, scale

    def moe_expert_ffn_w8(self, xp, offsets, w1_q, w2_q, w1_scale, w2_scale, b1=None, b2=None):
        n_rows = xp.shape[0]
        yp = self._new((n_rows, self.D), self.torch_dtype)
        ws, wsb = self._ws()
        _check(self.lib.moe_expert_ffn_w8(self.h, _ptr(xp), _ptr(offsets), _ptr(w1_q), _ptr(w2_q), _ptr(w1_scale),
                                          _ptr(w2_scale), _ptr(b1), _ptr(b2), n_rows, _ptr(yp), ws, wsb, _stream()))
        return yp

    def moe_layer_forward_w8(self, x, wg, w1_q, w2_q, w1_scale, w2_scale, gate_bias=None, b1=None, b2=None, y=None,
                             routing_out=None):
        T = x.shape[0]
        if y is None:
            y = self._new((T, self.D), self.torch_dtype)
        ws, wsb = self._ws()
        _check(self.lib.moe_layer_forward_w8(self.h, _ptr(x), _ptr(wg), _ptr(gate_bias), _ptr(w1_q), _ptr(w2_q),
                                             _ptr(w1_scale), _ptr(w2_scale), _ptr(b1), _ptr(b2), T, _ptr(y),
                                             self._routing_struct(routing_out), ws, wsb, _stream()))
        return y

    def moe_quantize_mxfp4(self, w):
        """w [E, rows, cols] -> (q uint8 [E, rows * cols / 2], scale bytes uint8 [E, moe_mxfp4_scale_bytes]),
        both in the library's blocked layouts."""
        E, rows, cols = w.shape
        nb = int(self.lib.moe_mxfp4_scale_bytes(rows, cols))
        if nb < 0:
            _check(nb)
        q = self._new((E, rows * cols // 2), torch.uint8)
        scale = torch.full((E, nb), 127, dtype=torch.uint8, device=self.device)
        _check(self.lib.moe_quantize_mxfp4(self.h, _ptr(w), E, rows, cols, _ptr(q), _ptr(scale), _stream()))
        return q, scale

    def moe_expert_ffn_w4(self, xp, offsets, w1_q, w2_q, w1_scale, w2_scale, b1=None, b2=None):
        n_rows = xp.shape[0]
        yp = self._new((n_rows, self.D), self.torch_dtype)
        ws, wsb = self._ws()
        _check(self.lib.moe_expert_ffn_w4(self.h, _ptr(xp), _ptr(offsets), _ptr(w1_q), _ptr(w2_q), _ptr(w1_scale),
                                          _ptr(w2_scale), _ptr(b1), _ptr(b2), n_rows, _ptr(yp), ws, wsb, _stream()))
        return yp

    def moe_layer_forward_w4(self, x, wg, w1_q, w2_q, w1_scale, w2_scale, gate_bias=None, b1=None, b2=None, y=None,
                             routing_out=None):
        T = x.shape[0]
        if y is None:
            y = self._new((T, self.D), self.torch_dtype)
        ws, wsb = self._ws()
        _check(self.lib.moe_layer_forward_w4(self.h, _ptr(x), _ptr(wg), _ptr(gate_bias), _ptr(w1_q), _ptr(w2_q),
                                             _ptr(w1_scale), _ptr(w2_scale), _ptr(b1), _ptr(b2), T, _ptr(y),
                                             self._routing_struct(routing_out), ws, wsb, _stream()))
        return y

    def moe_profile_begin(self) -> None:
        _check(self.lib.moe_profile_begin(self.h))

    def moe_profile_end(self):
        """-> list of (kernel name, milliseconds) in launch order.  Waits for the device."""
        ms = (ctypes.c_float * 64)()
        n = ctypes.c_int32(0)
        _check(self.lib.moe_profile_end(self.h, ms, 64, ctypes.byref(n)))
        return [(self.lib.moe_profile_name(self.h, i).decode(), float(ms[i])) for i in range(n.value)]

    def moe_static_workspace_bytes(self, T: int, capacity: int, mode: int) -> int:
        n = int(self.lib.moe_static_workspace_bytes(self.h, T, capacity, mode))
        if n < 0:
            _check(n)
        return n

    def moe_layer_forward_static(self, x, wg, w1, w2, capacity: int, mode: int = MOE_STATIC_INDEXED,
                                 gate_bias=None, b1=None, b2=None, y=None, routing_out=None, workspace=None):
        T = x.shape[0]
        if y is None:
            y = self._new((T, self.D), self.torch_dtype)
        dropped = torch.zeros(4, dtype=torch.int32, device=self.device)
        if workspace is None:
            workspace = torch.empty(self.moe_static_workspace_bytes(T, capacity, mode), dtype=torch.uint8,
                                    device=self.device)
        _check(self.lib.moe_layer_forward_static(self.h, _ptr(x), _ptr(wg), _ptr(gate_bias), _ptr(w1), _ptr(w2),
                                                 _ptr(b1), _ptr(b2), T, capacity, mode, _ptr(y), _ptr(dropped),
                                                 self._routing_struct(routing_out), _ptr(workspace),
                                                 workspace.numel(), _stream()))
        return y, dropped[:1]


class CachePolicy:
    """moe_cache_policy_*: the cache management of Expert Buffering alone (host logic, no GPU)."""

    def __init__(self, E: int, slots: int):
        self.lib = load_library()
        self.E, self.slots = E, slots
        self.p = ctypes.c_void_p()
        _check(self.lib.moe_cache_policy_create(E, slots, ctypes.byref(self.p)))

    def __del__(self):
        if getattr(self, "p", None) is not None and self.p:
            self.lib.moe_cache_policy_destroy(self.p)
            self.p = None

    def reset(self) -> None:
        _check(self.lib.moe_cache_policy_reset(self.p))

    def step(self, counts):
        """counts: E host integers -> (slot_of, stage_of, loads, n_stages); loads = list of
        (expert, slot, victim, stage)."""
        E = self.E
        c = (ctypes.c_int32 * E)(*[int(v) for v in counts])
        slot_of, stage_of = (ctypes.c_int32 * E)(), (ctypes.c_int32 * E)()
        loads = (ctypes.c_int32 * (4 * E))()
        n_loads, n_stages = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(self.lib.moe_cache_policy_step(self.p, c, slot_of, stage_of, loads, E, ctypes.byref(n_loads),
                                              ctypes.byref(n_stages)))
        ll = [tuple(loads[4 * i + j] for j in range(4)) for i in range(n_loads.value)]
        return list(slot_of), list(stage_of), ll, n_stages.value

    def stats(self):
        """-> (hits, misses, expert held by every slot)."""
        h, m = ctypes.c_int64(0), ctypes.c_int64(0)
        se = (ctypes.c_int32 * self.slots)()
        _check(self.lib.moe_cache_policy_stats(self.p, ctypes.byref(h), ctypes.byref(m), se))
        return h.value, m.value, list(se)


class ExpertCache:
    """moe_expert_cache_*: `slots` device slots in front of expert parameters kept in pinned host
    memory (host_w1 [E,F,D], host_w2 [E,D,F], torch CPU tensors with pin_memory)."""

    def __init__(self, layer: "MoeLayer", slots: int, host_w1: torch.Tensor, host_w2: torch.Tensor, wbits: int = 0,
                 w1_scale: Optional[torch.Tensor] = None, w2_scale: Optional[torch.Tensor] = None):
        """wbits = 8 / 4: host_w1 / host_w2 hold the quantised bytes (moe_quantize_e4m3 / moe_quantize_mxfp4,
        copied to pinned host memory), w1_scale / w2_scale their scales, which stay on the device."""
        self.lib = layer.lib
        self.layer = layer
        self.slots = slots
        if host_w1.device.type != "cpu" or host_w2.device.type != "cpu":
            raise ValueError("host_w1 / host_w2 must be CPU tensors (pinned)")
        self.host_w1, self.host_w2 = host_w1, host_w2  # kept alive
        self.w1_scale, self.w2_scale = w1_scale, w2_scale
        nbytes = int(self.lib.moe_expert_cache_bytes_q(layer.h, slots, wbits))
        if nbytes < 0:
            _check(nbytes)
        self.device_mem = torch.empty(nbytes, dtype=torch.uint8, device=layer.device)
        self.c = ctypes.c_void_p()
        _check(self.lib.moe_expert_cache_create_q(layer.h, slots, wbits, host_w1.data_ptr(), host_w2.data_ptr(),
                                                  _ptr(w1_scale), _ptr(w2_scale), _ptr(self.device_mem), nbytes,
                                                  ctypes.byref(self.c)))

    def __del__(self):
        if getattr(self, "c", None) is not None and self.c:
            self.lib.moe_expert_cache_destroy(self.c)
            self.c = None

    def reset(self) -> None:
        _check(self.lib.moe_expert_cache_reset(self.c))

    def stats(self):
        """-> dict(hits, misses, bytes_copied, stages)."""
        v = [ctypes.c_int64(0) for _ in range(4)]
        _check(self.lib.moe_expert_cache_stats(self.c, *[ctypes.byref(x) for x in v]))
        return dict(hits=v[0].value, misses=v[1].value, bytes_copied=v[2].value, stages=v[3].value)

    def moe_layer_forward_buffered(self, x, wg, gate_bias=None, b1=None, b2=None, y=None, routing_out=None):
        L = self.layer
        T = x.shape[0]
        if y is None:
            y = L._new((T, L.D), L.torch_dtype)
        ws, wsb = L._ws()
        _check(self.lib.moe_layer_forward_buffered(L.h, self.c, _ptr(x), _ptr(wg), _ptr(gate_bias), _ptr(b1),
                                                   _ptr(b2), T, _ptr(y), L._routing_struct(routing_out), ws, wsb,
                                                   _stream()))
        return y


def _activation_array(A):
    E = len(A)
    B = len(A[0]) if E else 0
    flat = (ctypes.c_float * (E * B))(*[float(v) for row in A for v in row])
    return flat, E, B


def moe_placement_greedy(A, n_devices: int):
    """A: E rows of B activation fractions (host) -> device of every expert (Sec. 7.1)."""
    flat, E, B = _activation_array(A)
    out = (ctypes.c_int32 * max(E, 1))()
    _check(load_library().moe_placement_greedy(flat, E, B, n_devices, out))
    return list(out)[:E]


def moe_placement_anticorrelation(A, n_devices: int, corr_weight: float = 0.5):
    flat, E, B = _activation_array(A)
    out = (ctypes.c_int32 * max(E, 1))()
    _check(load_library().moe_placement_anticorrelation(flat, E, B, n_devices, corr_weight, out))
    return list(out)[:E]


def moe_placement_loads(A, device_of, n_devices: int):
    """-> (Max Load, Avg Max Load) of a placement on activation data A (Sec. 7.1)."""
    flat, E, B = _activation_array(A)
    d = (ctypes.c_int32 * max(E, 1))(*[int(v) for v in device_of])
    mx, av = ctypes.c_double(0), ctypes.c_double(0)
    _check(load_library().moe_placement_loads(flat, E, B, d, n_devices, ctypes.byref(mx), ctypes.byref(av)))
    return mx.value, av.value
