"""ctypes front end of oracle/gqa_oracle.c (test infrastructure only).

Argument marshalling and nothing else: all arithmetic lives in the C file,
whose header states the definition it follows.  Inputs are numpy arrays of
bf16 bit patterns (dtype uint16); strides are taken from the arrays, so any
layout whose last axis is dense can be passed as a view.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gqa_oracle.c")
_LIB = os.path.join(_HERE, "libgqa_oracle.so")
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("block_table_stride", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_t", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_t", ctypes.c_int64),
        ("scale", ctypes.c_double),
    ]


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the row loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        _lib = ctypes.CDLL(_LIB)
        _lib.gqa_oracle_decode_attn.restype = ctypes.c_int
        _lib.gqa_oracle_decode_attn.argtypes = [
            ctypes.POINTER(_Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int]
        _lib.gqa_oracle_kv_append.restype = ctypes.c_int
        _lib.gqa_oracle_kv_append.argtypes = [ctypes.POINTER(_Shape)] + [ctypes.c_void_p] * 9
    return _lib


@dataclass
class OracleResult:
    out: np.ndarray                 # [B, Hq, D] float64
    lse: np.ndarray                 # [B, Hq] float64
    weights: Optional[np.ndarray]   # [B, Hq, max L] float64 (zero beyond L_b) or None
    threads: int


def _u16(a: np.ndarray) -> np.ndarray:
    if a.dtype != np.uint16:
        raise TypeError("bf16 bit patterns must be passed as uint16 arrays")
    if a.strides[-1] != 2:
        raise ValueError("last axis must be dense")
    return a


def _base_ptr(a: np.ndarray) -> int:
    return a.__array_interface__["data"][0]


def decode_attn(q: np.ndarray, k: np.ndarray, v: np.ndarray, kv_lens: np.ndarray, scale: float,
                block_table: Optional[np.ndarray] = None, page_size: int = 0,
                want_weights: bool = False, threads: Optional[int] = None) -> OracleResult:
    """q: [B, Hq, D].  Contiguous cache: k, v indexed [b, g, t, d] (any strides,
    e.g. a transposed view of a token-major array).  Paged cache: k, v indexed
    [block, g, slot, d] and block_table [B, max_blocks] int32."""
    lib = _load()
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, Hq, D = q.shape
    Hkv = k.shape[1]
    if k.shape[3] != D or v.shape[3] != D or v.shape[1] != Hkv:
        raise ValueError("shape mismatch between q, k, v")
    kv_lens = np.ascontiguousarray(kv_lens, dtype=np.int32)
    if kv_lens.shape != (B,):
        raise ValueError("kv_lens must have shape [B]")
    sh = _Shape()
    sh.batch, sh.num_q_heads, sh.num_kv_heads, sh.head_dim = B, Hq, Hkv, D
    sh.page_size = int(page_size)
    sh.scale = float(scale)
    sh.q_stride_b, sh.q_stride_h = q.strides[0] // 2, q.strides[1] // 2
    sh.k_stride_b, sh.k_stride_h, sh.k_stride_t = (x // 2 for x in k.strides[:3])
    sh.v_stride_b, sh.v_stride_h, sh.v_stride_t = (x // 2 for x in v.strides[:3])
    bt_ptr = None
    if page_size:
        if block_table is None:
            raise ValueError("paged cache needs a block table")
        block_table = np.ascontiguousarray(block_table, dtype=np.int32)
        sh.block_table_stride = block_table.shape[1]
        bt_ptr = _base_ptr(block_table)
        need = -(-int(kv_lens.max(initial=0)) // page_size)
        if need > block_table.shape[1]:
            raise ValueError("block table too narrow for kv_lens")
        for b in range(B):
            nb = -(-int(kv_lens[b]) // page_size)
            if nb and (block_table[b, :nb].min() < 0 or block_table[b, :nb].max() >= k.shape[0]):
                raise ValueError("block table entry out of range")
    else:
        if int(kv_lens.max(initial=0)) > k.shape[2]:
            raise ValueError("kv_lens exceeds the cache length")
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    w = None
    wstride = 0
    if want_weights:
        wstride = max(int(kv_lens.max(initial=0)), 1)
        w = np.zeros((B, Hq, wstride), dtype=np.float64)
    if threads is None:
        threads = len(os.sched_getaffinity(0))
    used = lib.gqa_oracle_decode_attn(ctypes.byref(sh), _base_ptr(q), _base_ptr(k), _base_ptr(v),
                                      _base_ptr(kv_lens), bt_ptr, _base_ptr(out), _base_ptr(lse),
                                      _base_ptr(w) if w is not None else None, wstride, int(threads))
    if used < 0:
        raise ValueError("oracle rejected its arguments")
    return OracleResult(out=out, lse=lse, weights=w, threads=used)


def causal_attn_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray, b: int, rows, scale: float) -> OracleResult:
    """Rows `rows` of causal attention over sequence b of q [B, T, Hq, D], k, v [B, T, Hkv, D]:
    row t is, by definition, the attention of query t over keys and values 0 .. t, i.e. decode_attn
    with kv_len = t + 1.  One oracle "sequence" per requested row, all reading the same K/V of
    sequence b (a view with batch stride 0, nothing is copied).  Result: out [R, Hq, D], lse [R, Hq]."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    rows = np.asarray(rows, dtype=np.int64)
    if rows.ndim != 1 or (len(rows) and (rows.min() < 0 or rows.max() >= q.shape[1])):
        raise ValueError("rows out of range")
    qq = np.ascontiguousarray(q[b, rows])                        # [R, Hq, D]
    kb, vb = k[b].transpose(1, 0, 2), v[b].transpose(1, 0, 2)    # [Hkv, T, D] views
    kk = np.broadcast_to(kb[None], (len(rows),) + kb.shape)      # [R, Hkv, T, D], stride 0 over R
    vv = np.broadcast_to(vb[None], (len(rows),) + vb.shape)
    return decode_attn(qq, kk, vv, rows + 1, scale)


def shared_prefix_attn(q: np.ndarray, k_prefix: np.ndarray, v_prefix: np.ndarray, prefix_lens: np.ndarray,
                       group_start: np.ndarray, k: np.ndarray, v: np.ndarray, kv_lens: np.ndarray, scale: float,
                       block_table: Optional[np.ndarray] = None, page_size: int = 0) -> OracleResult:
    """Attention of every sequence over [prefix of its group ; its own suffix].  Group j holds the
    sequences group_start[j] .. group_start[j+1]-1 and its prefix is k_prefix[j, :, :prefix_lens[j]]
    (indexed [group, kv head, token, d]); k, v, kv_lens, block_table describe the suffix caches as
    in decode_attn.  The definition needs no sharing: every sequence gets a private contiguous cache
    holding the two pieces one after the other, and decode_attn runs on that."""
    q, k, v, kp, vp = _u16(q), _u16(k), _u16(v), _u16(k_prefix), _u16(v_prefix)
    B, Hkv, D = q.shape[0], kp.shape[1], q.shape[2]
    group_start = np.asarray(group_start, dtype=np.int64)
    prefix_lens = np.asarray(prefix_lens, dtype=np.int64)
    kv_lens = np.asarray(kv_lens, dtype=np.int64)
    if group_start[0] != 0 or group_start[-1] != B or np.any(np.diff(group_start) < 0):
        raise ValueError("group_start must rise from 0 to the batch size")
    total = np.zeros(B, dtype=np.int64)
    for j in range(len(prefix_lens)):
        total[group_start[j]:group_start[j + 1]] = prefix_lens[j]
    total += kv_lens
    cap = max(int(total.max(initial=0)), 1)
    kc = np.zeros((B, Hkv, cap, D), dtype=np.uint16)
    vc = np.zeros((B, Hkv, cap, D), dtype=np.uint16)
    for j in range(len(prefix_lens)):
        P = int(prefix_lens[j])
        for b in range(int(group_start[j]), int(group_start[j + 1])):
            kc[b, :, :P] = kp[j, :, :P]
            vc[b, :, :P] = vp[j, :, :P]
            S = int(kv_lens[b])
            if page_size:
                for t in range(S):
                    blk, slot = int(block_table[b, t // page_size]), t % page_size
                    kc[b, :, P + t] = k[blk, :, slot]
                    vc[b, :, P + t] = v[blk, :, slot]
            else:
                kc[b, :, P:P + S] = k[b, :, :S]
                vc[b, :, P:P + S] = v[b, :, :S]
    return decode_attn(q, kc, vc, total.astype(np.int32), scale)


def kv_append(q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
              kv_lens: np.ndarray, cos_sin: Optional[np.ndarray] = None,
              block_table: Optional[np.ndarray] = None, page_size: int = 0) -> np.ndarray:
    """Rotate q and the new key by position kv_lens[b] - 1 (if cos_sin [positions, D] fp32 is given)
    and write the new key/value rows into the caches IN PLACE at that position.
    q [B, Hq, D]; k_new, v_new [B, Hkv, D] dense; caches indexed as in decode_attn.
    Returns the rotated q (same shape and strides as a dense copy of q)."""
    lib = _load()
    q = np.ascontiguousarray(_u16(q))
    k_new, v_new = np.ascontiguousarray(_u16(k_new)), np.ascontiguousarray(_u16(v_new))
    k_cache, v_cache = _u16(k_cache), _u16(v_cache)
    if not (k_cache.flags.writeable and v_cache.flags.writeable):
        raise ValueError("caches must be writable")
    B, Hq, D = q.shape
    Hkv = k_new.shape[1]
    kv_lens = np.ascontiguousarray(kv_lens, dtype=np.int32)
    sh = _Shape()
    sh.batch, sh.num_q_heads, sh.num_kv_heads, sh.head_dim = B, Hq, Hkv, D
    sh.page_size = int(page_size)
    sh.q_stride_b, sh.q_stride_h = q.strides[0] // 2, q.strides[1] // 2
    sh.k_stride_b, sh.k_stride_h, sh.k_stride_t = (x // 2 for x in k_cache.strides[:3])
    sh.v_stride_b, sh.v_stride_h, sh.v_stride_t = (x // 2 for x in v_cache.strides[:3])
    bt_ptr = None
    if page_size:
        block_table = np.ascontiguousarray(block_table, dtype=np.int32)
        sh.block_table_stride = block_table.shape[1]
        bt_ptr = _base_ptr(block_table)
        for b in range(B):
            if kv_lens[b] > 0:
                blk = block_table[b, (int(kv_lens[b]) - 1) // page_size]
                if blk < 0 or blk >= k_cache.shape[0]:
                    raise ValueError("block table entry out of range")
    elif int(kv_lens.max(initial=0)) > k_cache.shape[2]:
        raise ValueError("kv_lens exceeds the cache length")
    cs_ptr = None
    if cos_sin is not None:
        cos_sin = np.ascontiguousarray(cos_sin, dtype=np.float32)
        if cos_sin.ndim != 2 or cos_sin.shape[1] != D or cos_sin.shape[0] < int(kv_lens.max(initial=0)):
            raise ValueError("cos_sin must be [positions >= max kv_len, D]")
        cs_ptr = _base_ptr(cos_sin)
    q_out = np.empty_like(q)
    rc = lib.gqa_oracle_kv_append(ctypes.byref(sh), _base_ptr(q), _base_ptr(q_out), _base_ptr(k_new),
                                  _base_ptr(v_new), _base_ptr(k_cache), _base_ptr(v_cache),
                                  _base_ptr(kv_lens), bt_ptr, cs_ptr)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return q_out
