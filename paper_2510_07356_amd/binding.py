"""Thin ctypes binding of libgqa_decode.so (same names as include/gqa_decode.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the attention path runs in the library's kernels.
There is no fallback: if the library is missing, import fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# GQA_DECODE_LIBRARY selects another build of the same library (e.g. one compiled with other tunables)
LIB_PATH = os.environ.get("GQA_DECODE_LIBRARY") or os.path.join(_HERE, "libgqa_decode.so")

GQA_OK = 0
GQA_ERR_INVALID_ARG = -1
GQA_ERR_UNSUPPORTED = -2
GQA_ERR_WORKSPACE_TOO_SMALL = -3
GQA_ERR_LAUNCH = -4

GQA_ERR_SCRATCH_LIMIT = -5

EXPORTS = ("gqa_decode_version", "gqa_decode_strerror", "gqa_decode_init", "gqa_decode_workspace_bytes",
           "gqa_decode_plan_info", "gqa_decode_attn", "gqa_decode_attn_timed",
           "gqa_decode_static_scratch_bytes", "gqa_decode_attn_static",
           "gqa_prefill_attn", "gqa_prefill_attn_varlen", "gqa_decode_kv_append",
           "gqa_cascade_workspace_bytes", "gqa_decode_attn_shared_prefix",
           "gqa_decode_stream_read", "gqa_decode_stream_copy", "gqa_decode_stream_probe",
           "gqa_timer_create", "gqa_timer_destroy", "gqa_timer_read", "gqa_timer_read_calls")


class gqa_decode_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("max_kv_len", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("block_table_stride", ctypes.c_int32), ("chunk_tokens", ctypes.c_int32),
        ("scale", ctypes.c_float), ("kernel_variant", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_t", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_t", ctypes.c_int64),
    ]


class gqa_append_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("max_kv_len", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("block_table_stride", ctypes.c_int32), ("rope_positions", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_t", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_t", ctypes.c_int64),
    ]


class gqa_cascade_params(ctypes.Structure):
    _fields_ = [
        ("decode", gqa_decode_params),
        ("num_groups", ctypes.c_int32), ("max_prefix_len", ctypes.c_int32),
        ("kp_stride_g", ctypes.c_int64), ("kp_stride_h", ctypes.c_int64), ("kp_stride_t", ctypes.c_int64),
        ("vp_stride_g", ctypes.c_int64), ("vp_stride_h", ctypes.c_int64), ("vp_stride_t", ctypes.c_int64),
    ]


class gqa_prefill_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("scale", ctypes.c_float),
        ("q_stride_b", ctypes.c_int64), ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_t", ctypes.c_int64), ("k_stride_h", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_t", ctypes.c_int64), ("v_stride_h", ctypes.c_int64),
        ("o_stride_b", ctypes.c_int64), ("o_stride_t", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
    ]


class GqaError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"gqa_decode: {gqa_decode_strerror(status)} ({status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2510_07356_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(gqa_decode_params)
    vp, i32p = ctypes.c_void_p, ctypes.c_void_p
    lib.gqa_decode_version.restype = ctypes.c_int
    lib.gqa_decode_version.argtypes = []
    lib.gqa_decode_strerror.restype = ctypes.c_char_p
    lib.gqa_decode_strerror.argtypes = [ctypes.c_int]
    lib.gqa_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.gqa_decode_workspace_bytes.argtypes = [P]
    lib.gqa_decode_plan_info.restype = ctypes.c_int
    lib.gqa_decode_plan_info.argtypes = [P, i32p, ctypes.POINTER(ctypes.c_int32),
                                         ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)]
    attn_args = [P, vp, vp, vp, i32p, i32p, i32p, vp, vp, vp, ctypes.c_size_t, vp]
    lib.gqa_decode_attn.restype = ctypes.c_int
    lib.gqa_decode_attn.argtypes = attn_args
    lib.gqa_decode_attn_timed.restype = ctypes.c_int
    lib.gqa_decode_attn_timed.argtypes = attn_args + [vp]
    lib.gqa_decode_init.restype = ctypes.c_int
    lib.gqa_decode_init.argtypes = []
    lib.gqa_decode_static_scratch_bytes.restype = ctypes.c_size_t
    lib.gqa_decode_static_scratch_bytes.argtypes = []
    lib.gqa_decode_attn_static.restype = ctypes.c_int
    lib.gqa_decode_attn_static.argtypes = [P, vp, vp, vp, i32p, i32p, vp, vp, vp]
    lib.gqa_timer_create.restype = ctypes.c_int
    lib.gqa_timer_create.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p)]
    lib.gqa_timer_destroy.restype = None
    lib.gqa_timer_destroy.argtypes = [vp]
    lib.gqa_timer_read.restype = ctypes.c_int
    lib.gqa_timer_read.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)]
    lib.gqa_timer_read_calls.restype = ctypes.c_int
    lib.gqa_timer_read_calls.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                                         ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
    lib.gqa_cascade_workspace_bytes.restype = ctypes.c_size_t
    lib.gqa_cascade_workspace_bytes.argtypes = [ctypes.POINTER(gqa_cascade_params)]
    lib.gqa_decode_attn_shared_prefix.restype = ctypes.c_int
    lib.gqa_decode_attn_shared_prefix.argtypes = [ctypes.POINTER(gqa_cascade_params)] + [vp] * 13 + [ctypes.c_size_t, vp]
    lib.gqa_prefill_attn.restype = ctypes.c_int
    lib.gqa_prefill_attn.argtypes = [ctypes.POINTER(gqa_prefill_params)] + [vp] * 6
    lib.gqa_prefill_attn_varlen.restype = ctypes.c_int
    lib.gqa_prefill_attn_varlen.argtypes = [ctypes.POINTER(gqa_prefill_params)] + [vp] * 7
    lib.gqa_decode_kv_append.restype = ctypes.c_int
    lib.gqa_decode_kv_append.argtypes = [ctypes.POINTER(gqa_append_params)] + [vp] * 10
    lib.gqa_decode_stream_read.restype = ctypes.c_int
    lib.gqa_decode_stream_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int32, vp]
    lib.gqa_decode_stream_probe.restype = ctypes.c_int
    lib.gqa_decode_stream_probe.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int32, ctypes.c_int32, vp]
    lib.gqa_decode_stream_copy.restype = ctypes.c_int
    lib.gqa_decode_stream_copy.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int32, vp]
    return lib


_lib = _load()


def gqa_decode_version() -> int:
    return _lib.gqa_decode_version()


def gqa_decode_strerror(status: int) -> str:
    return _lib.gqa_decode_strerror(int(status)).decode()


def gqa_decode_init() -> None:
    """Per-device set-up for torch's current device (needed only before a HIP-graph capture)."""
    rc = _lib.gqa_decode_init()
    if rc != GQA_OK:
        raise GqaError(rc)


def gqa_decode_static_scratch_bytes() -> int:
    return int(_lib.gqa_decode_static_scratch_bytes())


def gqa_decode_workspace_bytes(params: gqa_decode_params) -> int:
    return int(_lib.gqa_decode_workspace_bytes(ctypes.byref(params)))


@dataclass
class PlanInfo:
    share_tokens: int
    workgroups: int
    partial_slots: int


def _host_lens_ptr(host_kv_lens):
    """host_kv_lens: None or a contiguous int32 CPU tensor / numpy array."""
    if host_kv_lens is None:
        return None, None
    if isinstance(host_kv_lens, torch.Tensor):
        assert host_kv_lens.device.type == "cpu" and host_kv_lens.dtype == torch.int32
        keep = host_kv_lens.contiguous()
        return keep.data_ptr(), keep
    import numpy as np
    keep = np.ascontiguousarray(host_kv_lens, dtype=np.int32)
    return keep.ctypes.data, keep


def gqa_decode_plan_info(params: gqa_decode_params, host_kv_lens=None) -> PlanInfo:
    c, w, m = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int64(0)
    ptr, _keep = _host_lens_ptr(host_kv_lens)
    rc = _lib.gqa_decode_plan_info(ctypes.byref(params), ptr, ctypes.byref(c), ctypes.byref(w), ctypes.byref(m))
    if rc != GQA_OK:
        raise GqaError(rc)
    return PlanInfo(c.value, w.value, m.value)


def make_params(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, max_kv_len: int, scale: float,
                page_size: int = 0, block_table: Optional[torch.Tensor] = None,
                chunk_tokens: int = 0, kernel_variant: int = 0) -> gqa_decode_params:
    """q [B, Hq, D]; k, v indexed [b | block, kv head, token | slot, d] (any strides with a dense last axis)."""
    p = gqa_decode_params()
    p.batch, p.num_q_heads, p.head_dim = q.shape
    p.num_kv_heads = k.shape[1]
    p.max_kv_len = int(max_kv_len)
    p.page_size = int(page_size)
    p.block_table_stride = int(block_table.stride(0)) if block_table is not None else 0
    p.chunk_tokens = int(chunk_tokens)
    p.scale = float(scale)
    p.kernel_variant = int(kernel_variant)
    p.q_stride_b, p.q_stride_h = q.stride(0), q.stride(1)
    p.k_stride_b, p.k_stride_h, p.k_stride_t = k.stride(0), k.stride(1), k.stride(2)
    p.v_stride_b, p.v_stride_h, p.v_stride_t = v.stride(0), v.stride(1), v.stride(2)
    return p


def _check_inputs(q, k, v, kv_lens, block_table, out, lse, workspace):
    for name, t, dt in (("q", q, torch.bfloat16), ("k", k, torch.bfloat16), ("v", v, torch.bfloat16),
                        ("kv_lens", kv_lens, torch.int32), ("out", out, torch.float32)):
        if not t.is_cuda or t.dtype != dt:
            raise TypeError(f"{name} must be a {dt} device tensor")
    if q.stride(-1) != 1 or k.stride(-1) != 1 or v.stride(-1) != 1:
        raise ValueError("the head_dim axis must be dense")
    if not out.is_contiguous() or (lse is not None and not lse.is_contiguous()):
        raise ValueError("out and lse must be dense")
    if block_table is not None and (not block_table.is_cuda or block_table.dtype != torch.int32
                                    or block_table.stride(1) != 1):
        raise TypeError("block_table must be an int32 device tensor with dense rows")
    if not workspace.is_cuda or workspace.dtype != torch.uint8:
        raise TypeError("workspace must be a uint8 device tensor")


class Timer:
    """gqa_timer: HIP events around the three kernels of up to max_calls calls."""

    def __init__(self, max_calls: int):
        self._h = ctypes.c_void_p()
        rc = _lib.gqa_timer_create(int(max_calls), ctypes.byref(self._h))
        if rc != GQA_OK:
            raise GqaError(rc)

    def read(self):
        """Wait for the recorded calls; returns (calls, (partial_ms, combine_ms) summed)."""
        n, ms = ctypes.c_int32(0), (ctypes.c_float * 2)()
        rc = _lib.gqa_timer_read(self._h, ctypes.byref(n), ms)
        if rc != GQA_OK:
            raise GqaError(rc)
        return n.value, tuple(ms)

    def read_calls(self, capacity: int):
        """Wait for the recorded calls; returns (partial_ms, combine_ms), one list entry per call."""
        n = ctypes.c_int32(0)
        a, b = (ctypes.c_float * capacity)(), (ctypes.c_float * capacity)()
        rc = _lib.gqa_timer_read_calls(self._h, int(capacity), ctypes.byref(n), a, b)
        if rc != GQA_OK:
            raise GqaError(rc)
        return list(a[:n.value]), list(b[:n.value])

    def close(self):
        if self._h:
            _lib.gqa_timer_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        self.close()


class Call:
    """Pre-marshalled argument list of one gqa_decode_attn call, so that a timed
    loop does nothing but cross the C ABI."""

    def __init__(self, params, q, k, v, kv_lens, block_table, host_kv_lens, out, lse, workspace,
                 stream: Optional[torch.cuda.Stream] = None):
        _check_inputs(q, k, v, kv_lens, block_table, out, lse, workspace)
        s = stream if stream is not None else torch.cuda.current_stream(q.device)
        hptr, self._keep = _host_lens_ptr(host_kv_lens)
        self._tensors = (q, k, v, kv_lens, block_table, out, lse, workspace, params)
        self.args = [ctypes.byref(params), q.data_ptr(), k.data_ptr(), v.data_ptr(), kv_lens.data_ptr(),
                     block_table.data_ptr() if block_table is not None else None, hptr,
                     out.data_ptr(), lse.data_ptr() if lse is not None else None,
                     workspace.data_ptr(), workspace.numel(), s.cuda_stream]

    def __call__(self, timer: Optional[Timer] = None) -> None:
        rc = _lib.gqa_decode_attn(*self.args) if timer is None \
            else _lib.gqa_decode_attn_timed(*self.args, timer._h)
        if rc != GQA_OK:
            raise GqaError(rc)


def gqa_decode_attn(params: gqa_decode_params, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                    kv_lens: torch.Tensor, block_table: Optional[torch.Tensor], host_kv_lens,
                    out: torch.Tensor, lse: Optional[torch.Tensor], workspace: torch.Tensor,
                    stream: Optional[torch.cuda.Stream] = None, timed: bool = False):
    """Enqueue one call on `stream` (default: torch's current stream).  With
    timed=True uses gqa_decode_attn_timed with a one-call timer, waits, and
    returns (partial_ms, combine_ms)."""
    _check_inputs(q, k, v, kv_lens, block_table, out, lse, workspace)
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    hptr, _keep = _host_lens_ptr(host_kv_lens)
    args = [ctypes.byref(params), q.data_ptr(), k.data_ptr(), v.data_ptr(), kv_lens.data_ptr(),
            block_table.data_ptr() if block_table is not None else None, hptr,
            out.data_ptr(), lse.data_ptr() if lse is not None else None,
            workspace.data_ptr(), workspace.numel(), s.cuda_stream]
    if timed:
        t = Timer(1)
        rc = _lib.gqa_decode_attn_timed(*args, t._h)
        if rc != GQA_OK:
            raise GqaError(rc)
        ms = t.read()[1]
        t.close()
        return ms
    rc = _lib.gqa_decode_attn(*args)
    if rc != GQA_OK:
        raise GqaError(rc)
    return None


def gqa_decode_attn_static(params: gqa_decode_params, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                           kv_lens: torch.Tensor, block_table: Optional[torch.Tensor],
                           out: torch.Tensor, lse: Optional[torch.Tensor],
                           stream: Optional[torch.cuda.Stream] = None) -> None:
    """gqa_decode_attn on the library's built-in scratch buffer: no workspace argument, no allocation."""
    for name, t, dt in (("q", q, torch.bfloat16), ("k", k, torch.bfloat16), ("v", v, torch.bfloat16),
                        ("kv_lens", kv_lens, torch.int32), ("out", out, torch.float32)):
        if not t.is_cuda or t.dtype != dt:
            raise TypeError(f"{name} must be a {dt} device tensor")
    if not out.is_contiguous() or (lse is not None and not lse.is_contiguous()):
        raise ValueError("out and lse must be dense")
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.gqa_decode_attn_static(ctypes.byref(params), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                     kv_lens.data_ptr(),
                                     block_table.data_ptr() if block_table is not None else None,
                                     out.data_ptr(), lse.data_ptr() if lse is not None else None, s.cuda_stream)
    if rc != GQA_OK:
        raise GqaError(rc)


def gqa_cascade_workspace_bytes(params: gqa_cascade_params) -> int:
    return int(_lib.gqa_cascade_workspace_bytes(ctypes.byref(params)))


def make_cascade_params(q, k, v, kp, vp, max_kv_len, max_prefix_len, num_groups, scale, page_size=0,
                        block_table=None, chunk_tokens=0) -> gqa_cascade_params:
    cp = gqa_cascade_params()
    cp.decode = make_params(q, k, v, max_kv_len, scale, page_size, block_table, chunk_tokens, 0)
    cp.num_groups, cp.max_prefix_len = int(num_groups), int(max_prefix_len)
    cp.kp_stride_g, cp.kp_stride_h, cp.kp_stride_t = kp.stride(0), kp.stride(1), kp.stride(2)
    cp.vp_stride_g, cp.vp_stride_h, cp.vp_stride_t = vp.stride(0), vp.stride(1), vp.stride(2)
    return cp


class CascadeCall:
    """Pre-marshalled gqa_decode_attn_shared_prefix call."""

    def __init__(self, cp, q, kp, vp, prefix_lens, group_start, host_group_start, k, v, kv_lens, block_table,
                 out, lse, workspace, stream: Optional[torch.cuda.Stream] = None):
        _check_inputs(q, k, v, kv_lens, block_table, out, lse, workspace)
        for t in (kp, vp):
            if not t.is_cuda or t.dtype != torch.bfloat16 or t.stride(-1) != 1:
                raise TypeError("prefix caches must be bf16 device tensors with a dense last axis")
        for t in (prefix_lens, group_start):
            if not t.is_cuda or t.dtype != torch.int32 or not t.is_contiguous():
                raise TypeError("prefix_lens / group_start must be dense int32 device tensors")
        hptr, self._keep = _host_lens_ptr(host_group_start)
        s = stream if stream is not None else torch.cuda.current_stream(q.device)
        self._tensors = (cp, q, kp, vp, prefix_lens, group_start, k, v, kv_lens, block_table, out, lse, workspace)
        self.args = [ctypes.byref(cp), q.data_ptr(), kp.data_ptr(), vp.data_ptr(), prefix_lens.data_ptr(),
                     group_start.data_ptr(), hptr, k.data_ptr(), v.data_ptr(), kv_lens.data_ptr(),
                     block_table.data_ptr() if block_table is not None else None,
                     out.data_ptr(), lse.data_ptr() if lse is not None else None,
                     workspace.data_ptr(), workspace.numel(), s.cuda_stream]

    def __call__(self) -> None:
        rc = _lib.gqa_decode_attn_shared_prefix(*self.args)
        if rc != GQA_OK:
            raise GqaError(rc)


def shared_prefix_to_device(sw, device="cuda:0"):
    dev = to_device(sw.base, device)
    dev["kp"] = _bf16_view(sw.kp).to(device)
    dev["vp"] = _bf16_view(sw.vp).to(device)
    dev["prefix_lens"] = torch.from_numpy(sw.prefix_lens).to(device)
    dev["group_start"] = torch.from_numpy(sw.group_start).to(device)
    return dev


def run_shared_prefix(sw, dev=None, chunk_tokens: int = 0, want_lse: bool = True):
    """One gqa_decode_attn_shared_prefix call on a workloads.SharedPrefixWorkload; returns (out, lse)."""
    w = sw.base
    dev = dev if dev is not None else shared_prefix_to_device(sw)
    cp = make_cascade_params(dev["q"], dev["k"], dev["v"], dev["kp"], dev["vp"], w.max_kv_len,
                             int(sw.prefix_lens.max(initial=0)), len(sw.prefix_lens), w.scale, w.page_size,
                             dev["block_table"], chunk_tokens)
    nbytes = gqa_cascade_workspace_bytes(cp)
    if nbytes == 0:
        raise GqaError(GQA_ERR_UNSUPPORTED)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=dev["q"].device)
    out = torch.full((w.batch, w.num_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device=dev["q"].device)
    lse = torch.full((w.batch, w.num_q_heads), float("nan"), dtype=torch.float32, device=dev["q"].device) if want_lse else None
    CascadeCall(cp, dev["q"], dev["kp"], dev["vp"], dev["prefix_lens"], dev["group_start"], sw.group_start,
                dev["k"], dev["v"], dev["kv_lens"], dev["block_table"], out, lse, ws)()
    return out, lse


def gqa_prefill_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scale: float, out: torch.Tensor,
                     lse: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                     seq_lens: Optional[torch.Tensor] = None) -> None:
    """q [B, T, Hq, D], k/v [B, T, Hkv, D] bf16 (any strides, dense last axis); out [B, T, Hq, D] fp32;
    lse [B, T, Hq] fp32 dense or None; seq_lens [B] int32 on the device or None (gqa_prefill_attn_varlen)."""
    if seq_lens is not None and (not seq_lens.is_cuda or seq_lens.dtype != torch.int32 or not seq_lens.is_contiguous()
                                 or seq_lens.numel() != q.shape[0]):
        raise TypeError("seq_lens must be a dense int32 device tensor with one entry per sequence")
    for t in (q, k, v):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.stride(-1) != 1:
            raise TypeError("bf16 device tensors with a dense last axis expected")
    if not out.is_cuda or out.dtype != torch.float32 or out.stride(-1) != 1:
        raise TypeError("out must be an fp32 device tensor with a dense last axis")
    if lse is not None and (lse.dtype != torch.float32 or not lse.is_contiguous()):
        raise TypeError("lse must be a dense fp32 tensor")
    p = gqa_prefill_params()
    p.batch, p.seq_len, p.num_q_heads, p.head_dim = q.shape
    p.num_kv_heads = k.shape[2]
    p.scale = float(scale)
    p.q_stride_b, p.q_stride_t, p.q_stride_h = q.stride(0), q.stride(1), q.stride(2)
    p.k_stride_b, p.k_stride_t, p.k_stride_h = k.stride(0), k.stride(1), k.stride(2)
    p.v_stride_b, p.v_stride_t, p.v_stride_h = v.stride(0), v.stride(1), v.stride(2)
    p.o_stride_b, p.o_stride_t, p.o_stride_h = out.stride(0), out.stride(1), out.stride(2)
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    if seq_lens is None:
        rc = _lib.gqa_prefill_attn(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                   lse.data_ptr() if lse is not None else None, s.cuda_stream)
    else:
        rc = _lib.gqa_prefill_attn_varlen(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                          seq_lens.data_ptr(), out.data_ptr(),
                                          lse.data_ptr() if lse is not None else None, s.cuda_stream)
    if rc != GQA_OK:
        raise GqaError(rc)


def gqa_decode_kv_append(q_in: torch.Tensor, q_out: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                         k_cache: torch.Tensor, v_cache: torch.Tensor, kv_lens: torch.Tensor, max_kv_len: int,
                         block_table: Optional[torch.Tensor] = None, page_size: int = 0,
                         cos_sin: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    """q_in/q_out [B, Hq, D] (same strides); k_new, v_new [B, Hkv, D] dense; caches indexed
    [b | block, kv head, token | slot, d]; cos_sin [positions, D] fp32 or None."""
    for t in (q_in, q_out, k_new, v_new, k_cache, v_cache):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.stride(-1) != 1:
            raise TypeError("bf16 device tensors with a dense last axis expected")
    if q_in.stride() != q_out.stride() or not k_new.is_contiguous() or not v_new.is_contiguous():
        raise ValueError("q_in/q_out must share strides; k_new/v_new must be dense")
    if cos_sin is not None and (cos_sin.dtype != torch.float32 or not cos_sin.is_contiguous() or not cos_sin.is_cuda):
        raise TypeError("cos_sin must be a dense fp32 device tensor")
    p = gqa_append_params()
    p.batch, p.num_q_heads, p.head_dim = q_in.shape
    p.num_kv_heads = k_new.shape[1]
    p.max_kv_len = int(max_kv_len)
    p.page_size = int(page_size)
    p.block_table_stride = int(block_table.stride(0)) if block_table is not None else 0
    p.rope_positions = int(cos_sin.shape[0]) if cos_sin is not None else 0
    p.q_stride_b, p.q_stride_h = q_in.stride(0), q_in.stride(1)
    p.k_stride_b, p.k_stride_h, p.k_stride_t = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    p.v_stride_b, p.v_stride_h, p.v_stride_t = v_cache.stride(0), v_cache.stride(1), v_cache.stride(2)
    s = stream if stream is not None else torch.cuda.current_stream(q_in.device)
    rc = _lib.gqa_decode_kv_append(ctypes.byref(p), q_in.data_ptr(), q_out.data_ptr(), k_new.data_ptr(),
                                   v_new.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), kv_lens.data_ptr(),
                                   block_table.data_ptr() if block_table is not None else None,
                                   cos_sin.data_ptr() if cos_sin is not None else None, s.cuda_stream)
    if rc != GQA_OK:
        raise GqaError(rc)


def gqa_decode_stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
    s = stream if stream is not None else torch.cuda.current_stream(src.device)
    nbytes = src.numel() * src.element_size()
    if sink.numel() * sink.element_size() < 4 * workgroups:
        raise ValueError("sink too small")
    rc = _lib.gqa_decode_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), int(workgroups), s.cuda_stream)
    if rc != GQA_OK:
        raise GqaError(rc)


def gqa_decode_stream_probe(src: torch.Tensor, sink: torch.Tensor, workgroups: int, mode: int,
                            stream: Optional[torch.cuda.Stream] = None) -> None:
    s = stream if stream is not None else torch.cuda.current_stream(src.device)
    if sink.numel() * sink.element_size() < 16 * workgroups:
        raise ValueError("sink too small")
    rc = _lib.gqa_decode_stream_probe(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                      int(workgroups), int(mode), s.cuda_stream)
    if rc != GQA_OK:
        raise GqaError(rc)


def gqa_decode_stream_copy(src: torch.Tensor, dst: torch.Tensor, workgroups: int,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
    s = stream if stream is not None else torch.cuda.current_stream(src.device)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    rc = _lib.gqa_decode_stream_copy(src.data_ptr(), dst.data_ptr(), nbytes, int(workgroups), s.cuda_stream)
    if rc != GQA_OK:
        raise GqaError(rc)


# ---------------------------------------------------------------------------
# Convenience used by tests, smoke and the benchmark: numpy workload -> device
# ---------------------------------------------------------------------------

def _bf16_view(bits_np) -> torch.Tensor:
    """uint16 bit patterns (numpy, maybe a strided view) -> bf16 CPU tensor with the same strides."""
    import numpy as np
    base = bits_np
    while isinstance(base.base, np.ndarray):
        base = base.base
    flat = torch.from_numpy(base.reshape(-1).view(np.int16)).view(torch.bfloat16)
    offset = (bits_np.__array_interface__["data"][0] - base.__array_interface__["data"][0]) // 2
    return torch.as_strided(flat, bits_np.shape, [s // 2 for s in bits_np.strides], offset)


def to_device(w, device="cuda:0"):
    """Copy a workloads.Workload to the device, keeping its memory layout.
    Returns dict(q, k, v, kv_lens, block_table)."""
    def put(bits):
        t = _bf16_view(bits)
        # move the underlying dense storage, then rebuild the same strided view
        dense = torch.empty(t.untyped_storage().size() // 2, dtype=torch.bfloat16, device=device)
        src = torch.as_strided(t, (dense.numel(),), (1,), 0)
        dense.copy_(src)
        return torch.as_strided(dense, t.shape, t.stride(), t.storage_offset())
    bt = torch.from_numpy(w.block_table).to(device) if w.block_table is not None else None
    return dict(q=put(w.q), k=put(w.k), v=put(w.v),
                kv_lens=torch.from_numpy(w.kv_lens).to(device), block_table=bt)


def run_workload(w, dev=None, chunk_tokens: int = 0, kernel_variant: int = 0, use_host_lens: bool = True,
                 want_lse: bool = True, timed: bool = False):
    """One library call on a workload; returns (out, lse[, kernel_ms]) as device tensors."""
    dev = dev if dev is not None else to_device(w)
    q, k, v = dev["q"], dev["k"], dev["v"]
    params = make_params(q, k, v, w.max_kv_len, w.scale, w.page_size, dev["block_table"],
                         chunk_tokens, kernel_variant)
    nbytes = gqa_decode_workspace_bytes(params)
    if nbytes == 0:
        raise GqaError(GQA_ERR_UNSUPPORTED)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=q.device)   # NaN poison: stale partials show up
    out = torch.full((w.batch, w.num_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device=q.device)
    lse = torch.full((w.batch, w.num_q_heads), float("nan"), dtype=torch.float32, device=q.device) if want_lse else None
    ms = gqa_decode_attn(params, q, k, v, dev["kv_lens"], dev["block_table"],
                         w.kv_lens if use_host_lens else None, out, lse, ws, timed=timed)
    return (out, lse, ms) if timed else (out, lse)


# ---------------------------------------------------------------------------
# Host-only metrics and curation rules of the paper (include/concur_curation.h)
# ---------------------------------------------------------------------------
CURATION_EXPORTS = ("concur_speedup", "concur_fast_p", "concur_exec_pass_at_k", "concur_fast1_pass_at_k",
                    "concur_arl", "concur_difficulty_bins", "concur_select")


def _np(a, dtype):
    import numpy as np
    return np.ascontiguousarray(a, dtype=dtype)


def _setup_curation():
    d, i64, vp = ctypes.c_double, ctypes.c_int64, ctypes.c_void_p
    _lib.concur_speedup.restype = ctypes.c_int
    _lib.concur_speedup.argtypes = [i64, vp, vp, vp, vp]
    _lib.concur_fast_p.restype = d
    _lib.concur_fast_p.argtypes = [i64, vp, d]
    _lib.concur_exec_pass_at_k.restype = d
    _lib.concur_exec_pass_at_k.argtypes = [i64, ctypes.c_int32, vp]
    _lib.concur_fast1_pass_at_k.restype = d
    _lib.concur_fast1_pass_at_k.argtypes = [i64, ctypes.c_int32, vp]
    _lib.concur_arl.restype = d
    _lib.concur_arl.argtypes = [i64, ctypes.c_int32, vp]
    _lib.concur_difficulty_bins.restype = ctypes.c_int
    _lib.concur_difficulty_bins.argtypes = [i64, vp, d, d, vp]
    _lib.concur_select.restype = i64
    _lib.concur_select.argtypes = [i64, vp, vp, vp, vp, d, i64, vp, vp]


_setup_curation()


def concur_speedup(t_torch, t_kernel, correct):
    import numpy as np
    tt, tk, c = _np(t_torch, np.float64), _np(t_kernel, np.float64), _np(correct, np.uint8)
    out = np.empty(len(tt), dtype=np.float64)
    if _lib.concur_speedup(len(tt), tt.ctypes.data, tk.ctypes.data, c.ctypes.data, out.ctypes.data) != 0:
        raise ValueError("concur_speedup: bad arguments")
    return out


def concur_fast_p(speedup, p):
    import numpy as np
    s = _np(speedup, np.float64)
    return float(_lib.concur_fast_p(len(s), s.ctypes.data, float(p)))


def concur_exec_pass_at_k(correct_rows):
    import numpy as np
    c = _np(correct_rows, np.uint8)
    return float(_lib.concur_exec_pass_at_k(c.shape[0], c.shape[1], c.ctypes.data))


def concur_fast1_pass_at_k(speedup_rows):
    import numpy as np
    s = _np(speedup_rows, np.float64)
    return float(_lib.concur_fast1_pass_at_k(s.shape[0], s.shape[1], s.ctypes.data))


def concur_arl(length_rows):
    import numpy as np
    L = _np(length_rows, np.int32)
    return float(_lib.concur_arl(L.shape[0], L.shape[1], L.ctypes.data))


def concur_difficulty_bins(task_arl, lo=4000.0, hi=8500.0):
    import numpy as np
    a = _np(task_arl, np.float64)
    out = np.empty(len(a), dtype=np.int32)
    if _lib.concur_difficulty_bins(len(a), a.ctypes.data, float(lo), float(hi), out.ctypes.data) != 0:
        raise ValueError("concur_difficulty_bins: bad arguments")
    return out


def concur_select(task_id, speedup, reasoning_len, single_op, threshold=5.0, quota=544):
    """Returns (flags uint8 per record, counts (a, b-only, c))."""
    import numpy as np
    t, s = _np(task_id, np.int64), _np(speedup, np.float64)
    r, o = _np(reasoning_len, np.int32), _np(single_op, np.uint8)
    flags = np.empty(len(t), dtype=np.uint8)
    counts = np.zeros(3, dtype=np.int64)
    rc = _lib.concur_select(len(t), t.ctypes.data, s.ctypes.data, r.ctypes.data, o.ctypes.data, float(threshold),
                            int(quota), flags.ctypes.data, counts.ctypes.data)
    if rc < 0:
        raise ValueError("concur_select: bad arguments")
    return flags, tuple(int(x) for x in counts)
