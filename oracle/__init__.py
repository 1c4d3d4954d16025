"""CPU oracle (fp64) for decode attention -- TEST INFRASTRUCTURE ONLY.

ctypes binding of ``oracle_attn.c``.  Only ``tests/``, the smoke check and the
benchmark's CPU-baseline leg may import this package; the product package never
does, and this package imports nothing of the product.

All array arguments are numpy arrays of bf16 bit patterns (uint16); results are
float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .beam import beam_select  # noqa: F401,E402  (numpy only)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_attn.c")
_LIB_PATH = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle_attn.c (gcc, OpenMP, no fast-math, no contraction). Returns the library path."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        tmp = _LIB_PATH + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
             "-Wall", "-Wextra", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _bind(path: str):
    lib = ctypes.CDLL(path)
    vp, i32 = ctypes.c_void_p, ctypes.c_int
    lib.oracle_num_threads.restype = i32
    lib.oracle_attn.restype = i32
    lib.oracle_attn.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_float, vp, vp]
    lib.oracle_attn_weights.restype = i32
    lib.oracle_attn_weights.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_float,
                                        i32, i32, i32, vp]
    lib.oracle_merge.restype = i32
    lib.oracle_merge.argtypes = [vp, vp, i32, ctypes.c_long, i32, vp, vp]
    lib.oracle_write_kvcache.restype = i32
    lib.oracle_write_kvcache.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32]
    lib.oracle_mla.restype = i32
    lib.oracle_mla.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_float, vp, vp]
    lib.oracle_page_of.restype = None
    lib.oracle_page_of.argtypes = [ctypes.c_uint64] * 3 + [vp, vp]
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


class use_library:
    """Context manager for the oracle's own tests: route calls to another build of oracle_attn.c
    (a deliberately broken copy) to show that the pins catch it."""

    def __init__(self, path: str):
        self._path = path

    def __enter__(self):
        global _lib
        self._saved = _lib
        _lib = _bind(self._path)
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self._saved
        return False


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _marshal(q, ks, vs, kv_lens):
    q = np.ascontiguousarray(q, dtype=np.uint16)
    if q.ndim != 4:
        raise ValueError("q must be [batch, q_len, n_q_heads, head_dim]")
    B, T, Hq, D = q.shape
    if len(ks) != B or len(vs) != B or len(kv_lens) != B:
        raise ValueError("ks, vs, kv_lens must have one entry per sequence")
    ks = [np.ascontiguousarray(k, dtype=np.uint16) for k in ks]
    vs = [np.ascontiguousarray(v, dtype=np.uint16) for v in vs]
    Hkv = ks[0].shape[1] if B else 1
    for b in range(B):
        for a in (ks[b], vs[b]):
            if a.ndim != 3 or a.shape[1] != Hkv or a.shape[2] != D or a.shape[0] < kv_lens[b]:
                raise ValueError("K/V of sequence %d must be [>=kv_len, n_kv_heads, head_dim]" % b)
    lens = np.ascontiguousarray(kv_lens, dtype=np.int32)
    kp = (ctypes.c_void_p * max(B, 1))(*[k.ctypes.data for k in ks])
    vp = (ctypes.c_void_p * max(B, 1))(*[v.ctypes.data for v in vs])
    return q, ks, vs, lens, kp, vp, (B, T, Hq, Hkv, D)


def attn(q: np.ndarray, ks: Sequence[np.ndarray], vs: Sequence[np.ndarray], kv_lens: Sequence[int],
         scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """softmax(scale * Q K^T) V per (sequence, new token, query head), causal inside the new-token block.

    Returns (out float64 [B, T, Hq, D], lse float64 [B, T, Hq]); lse is the natural-log sum of exp of
    the scaled scores.
    """
    q, ks, vs, lens, kp, vp, (B, T, Hq, Hkv, D) = _marshal(q, ks, vs, kv_lens)
    out = np.empty((B, T, Hq, D), dtype=np.float64)
    lse = np.empty((B, T, Hq), dtype=np.float64)
    rc = _load().oracle_attn(q.ctypes.data, kp, vp, lens.ctypes.data, B, T, Hq, Hkv, D,
                             ctypes.c_float(scale), out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_attn rejected its arguments (kv_len < q_len, or heads not divisible)")
    return out, lse


def attn_weights(q, ks, vs, kv_lens, scale: float, b: int, t: int, h: int) -> np.ndarray:
    """Normalised softmax weights of one (b, t, h) row over its visible keys."""
    q, ks, vs, lens, kp, vp, (B, T, Hq, Hkv, D) = _marshal(q, ks, vs, kv_lens)
    w = np.empty(int(lens[b]) - T + t + 1, dtype=np.float64)
    rc = _load().oracle_attn_weights(q.ctypes.data, kp, vp, lens.ctypes.data, B, T, Hq, Hkv, D,
                                     ctypes.c_float(scale), b, t, h, w.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_attn_weights rejected its arguments")
    return w


def merge(out_parts: np.ndarray, lse_parts: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Aggregate partial results over disjoint key ranges.

    out_parts float64 [n_parts, ..., D], lse_parts float64 [n_parts, ...] -> (out [..., D], lse [...]).
    """
    out_parts = np.ascontiguousarray(out_parts, dtype=np.float64)
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    S, D = out_parts.shape[0], out_parts.shape[-1]
    lead = out_parts.shape[1:-1]
    rows = int(np.prod(lead)) if lead else 1
    if lse_parts.shape != (S,) + lead:
        raise ValueError("lse_parts shape must be out_parts shape without the last axis")
    out = np.empty(lead + (D,), dtype=np.float64)
    lse = np.empty(lead, dtype=np.float64)
    rc = _load().oracle_merge(out_parts.ctypes.data, lse_parts.ctypes.data, S, rows, D,
                              out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_merge rejected its arguments")
    return out, lse


def page_of(va: int, va_start: int, page_size: int) -> Tuple[int, int]:
    """(physical page index within the range, byte offset within the page) of a virtual address."""
    idx, off = ctypes.c_uint64(), ctypes.c_uint64()
    _load().oracle_page_of(va, va_start, page_size, ctypes.byref(idx), ctypes.byref(off))
    return int(idx.value), int(off.value)


def write_kvcache(k_new: np.ndarray, v_new: np.ndarray, ks: Sequence[np.ndarray], vs: Sequence[np.ndarray],
                  kv_lens: Sequence[int]) -> None:
    """Append in place: k_new/v_new uint16 [B, T, Hkv, D] go to rows [kv_len - T, kv_len) of ks[b] / vs[b]."""
    k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
    v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    B, T = k_new.shape[:2]
    row = int(np.prod(k_new.shape[2:]))
    for a in list(ks) + list(vs):
        if a.dtype != np.uint16 or not a.flags["C_CONTIGUOUS"] or int(np.prod(a.shape[1:])) != row:
            raise ValueError("K/V buffers must be contiguous uint16 [rows, Hkv, D]")
    for b in range(B):
        if ks[b].shape[0] < kv_lens[b] or vs[b].shape[0] < kv_lens[b]:
            raise ValueError("buffer of sequence %d is shorter than kv_len" % b)
    lens = np.ascontiguousarray(kv_lens, dtype=np.int32)
    kp = (ctypes.c_void_p * max(B, 1))(*[k.ctypes.data for k in ks])
    vp = (ctypes.c_void_p * max(B, 1))(*[v.ctypes.data for v in vs])
    rc = _load().oracle_write_kvcache(k_new.ctypes.data, v_new.ctypes.data, kp, vp, lens.ctypes.data, B, T, row)
    if rc != 0:
        raise ValueError("oracle_write_kvcache rejected its arguments")


def mla(q: np.ndarray, cs: Sequence[np.ndarray], kv_lens: Sequence[int], d_v: int, scale: float
        ) -> Tuple[np.ndarray, np.ndarray]:
    """Latent-KV attention: q uint16 [B, T, H, d_qk]; cs[b] uint16 [>= kv_len, d_qk] is key and (its first
    d_v columns) value of every head.  Returns (out float64 [B, T, H, d_v], lse float64 [B, T, H])."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    B, T, H, d_qk = q.shape
    cs = [np.ascontiguousarray(c, dtype=np.uint16) for c in cs]
    for b in range(B):
        if cs[b].ndim != 2 or cs[b].shape[1] != d_qk or cs[b].shape[0] < kv_lens[b]:
            raise ValueError("latent cache of sequence %d must be [>= kv_len, d_qk]" % b)
    lens = np.ascontiguousarray(kv_lens, dtype=np.int32)
    cp = (ctypes.c_void_p * max(B, 1))(*[c.ctypes.data for c in cs])
    out = np.empty((B, T, H, d_v), dtype=np.float64)
    lse = np.empty((B, T, H), dtype=np.float64)
    rc = _load().oracle_mla(q.ctypes.data, cp, lens.ctypes.data, B, T, H, d_qk, d_v, ctypes.c_float(scale),
                            out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_mla rejected its arguments")
    return out, lse
