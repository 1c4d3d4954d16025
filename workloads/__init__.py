"""Seeded synthetic workloads for decode attention over per-sequence KV ranges.

This module serves both the CPU oracle's callers and the GPU path's callers.  It
holds no attention arithmetic: only the five workload shapes, the length samplers
and the counter-based N(0,1) -> bf16 generator (``gen.c``).  Every draw depends
on ``(seed, stream, index)`` alone, so host and device consumers see identical
bytes and any sub-range can be regenerated on its own.

Streams of one workload seed:
    0          Q  [batch, q_len, n_q_heads, head_dim]
    1 + 2*b    K of sequence b  [kv_len, n_kv_heads, head_dim]
    2 + 2*b    V of sequence b
    2**40      the KV-length sampler
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, replace
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB_PATH = os.path.join(_HERE, "libwlgen.so")
_LEN_STREAM = 1 << 40
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.c into libwlgen.so (gcc, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        tmp = _LIB_PATH + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
             "-ffp-contract=off", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64 = ctypes.c_uint64
        lib.wl_normal_f64.restype = ctypes.c_double
        lib.wl_normal_f64.argtypes = [u64, u64, u64]
        lib.wl_normal_bf16.restype = None
        lib.wl_normal_bf16.argtypes = [u64, u64, u64, u64, ctypes.c_void_p]
        lib.wl_uniform_u64.restype = None
        lib.wl_uniform_u64.argtypes = [u64, u64, u64, u64, ctypes.c_void_p]
        _lib = lib
    return _lib


# --------------------------------------------------------------------------- bf16 plumbing
def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """float -> bf16 bit patterns (uint16), round-to-nearest-even; NaN stays NaN."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    r = np.where(nan, (u >> 16) | 0x40, r)
    return r.astype(np.uint16)


# --------------------------------------------------------------------------- raw draws
def normal_bf16(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n bf16 bit patterns of i.i.d. N(0,1) draws: elements offset..offset+n of a stream."""
    out = np.empty(int(n), dtype=np.uint16)
    if n:
        _load().wl_normal_bf16(seed, stream, offset, n, out.ctypes.data)
    return out


def normal_f64(seed: int, stream: int, i: int) -> float:
    return float(_load().wl_normal_f64(seed, stream, i))


def uniform_u64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    out = np.empty(int(n), dtype=np.uint64)
    if n:
        _load().wl_uniform_u64(seed, stream, offset, n, out.ctypes.data)
    return out


# --------------------------------------------------------------------------- workloads
@dataclass(frozen=True)
class Workload:
    """One decode-attention workload: shapes, the KV-length recipe and the seed."""
    name: str
    batch: int
    q_len: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seed: int
    len_kind: str                      # "fixed" | "uniform" | "lognormal"
    len_args: Tuple = ()               # fixed: the lengths; uniform: (lo, hi); lognormal: (median, sigma, lo, hi)
    xtensor: bool = False              # place K/V in randomly permuted 2 MiB chunks
    note: str = ""

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def scale(self) -> float:
        """1/sqrt(head_dim) rounded to fp32, as the caller passes it."""
        return float(np.float32(1.0 / math.sqrt(self.head_dim)))

    def kv_lens(self) -> np.ndarray:
        """int32[batch]: keys visible to the LAST query token (prefix + q_len new tokens)."""
        B = self.batch
        if self.len_kind == "fixed":
            lens = np.asarray(self.len_args, dtype=np.int64)
            assert lens.shape == (B,)
        elif self.len_kind == "uniform":
            lo, hi = self.len_args
            u = uniform_u64(self.seed, _LEN_STREAM, B)
            lens = lo + (u % np.uint64(hi - lo + 1)).astype(np.int64)
            lens = lens + (self.q_len if self.q_len > 1 else 0)   # recipe draws the cached prefix
        elif self.len_kind == "lognormal":
            median, sigma, lo, hi = self.len_args
            z = np.array([normal_f64(self.seed, _LEN_STREAM, i) for i in range(B)])
            lens = np.clip(np.rint(median * np.exp(sigma * z)), lo, hi).astype(np.int64)
        else:
            raise ValueError(self.len_kind)
        return lens.astype(np.int32)

    def row_elems(self) -> int:
        return self.n_kv_heads * self.head_dim

    def kv_bytes(self, lens: Optional[Sequence[int]] = None) -> int:
        """Algorithmic K+V bytes one pass reads: sum_b L_b * Hkv * D * 2 tensors * 2 B."""
        lens = self.kv_lens() if lens is None else lens
        return int(np.sum(np.asarray(lens, dtype=np.int64))) * self.row_elems() * 2 * 2

    def make_q(self) -> np.ndarray:
        n = self.batch * self.q_len * self.n_q_heads * self.head_dim
        return normal_bf16(self.seed, 0, n).reshape(self.batch, self.q_len, self.n_q_heads, self.head_dim)

    def make_k(self, b: int, length: int) -> np.ndarray:
        return normal_bf16(self.seed, 1 + 2 * b, length * self.row_elems()).reshape(
            length, self.n_kv_heads, self.head_dim)

    def make_v(self, b: int, length: int) -> np.ndarray:
        return normal_bf16(self.seed, 2 + 2 * b, length * self.row_elems()).reshape(
            length, self.n_kv_heads, self.head_dim)

    def make_kv(self, lens: Optional[Sequence[int]] = None) -> Tuple[List[np.ndarray], List[np.ndarray]]:
        lens = self.kv_lens() if lens is None else lens
        ks = [self.make_k(b, int(L)) for b, L in enumerate(lens)]
        vs = [self.make_v(b, int(L)) for b, L in enumerate(lens)]
        return ks, vs

    def scaled(self, name: str, batch: int, len_div: int) -> "Workload":
        """A smaller workload of the same structure: fewer sequences, lengths divided by len_div."""
        if self.len_kind == "uniform":
            lo, hi = self.len_args
            args = (max(1, lo // len_div), max(2, hi // len_div))
        elif self.len_kind == "lognormal":
            median, sigma, lo, hi = self.len_args
            args = (max(4, median // len_div), sigma, max(1, lo // len_div) if lo > 1 else lo, max(8, hi // len_div))
        else:
            args = tuple(self.len_args)[:batch]
        return replace(self, name=name, batch=batch, len_args=args)


@dataclass(frozen=True)
class MlaWorkload:
    """Latent-KV (MLA-shaped) decode: one cached row of d_latent + d_rope values per token, shared by all heads."""
    name: str
    batch: int
    q_len: int
    n_heads: int
    seed: int
    len_args: Tuple            # uniform (lo, hi) cached-prefix length
    d_latent: int = 512
    d_rope: int = 64
    xtensor: bool = True
    note: str = ""

    @property
    def d_qk(self) -> int:
        return self.d_latent + self.d_rope

    @property
    def scale(self) -> float:
        """1/sqrt(128 + 64): the softmax scale of a model whose un-absorbed head has 128 + 64 dimensions."""
        return float(np.float32(1.0 / math.sqrt(192.0)))

    def kv_lens(self) -> np.ndarray:
        lo, hi = self.len_args
        u = uniform_u64(self.seed, _LEN_STREAM, self.batch)
        lens = lo + (u % np.uint64(hi - lo + 1)).astype(np.int64)
        return (lens + (self.q_len if self.q_len > 1 else 0)).astype(np.int32)

    def kv_bytes(self, lens=None) -> int:
        lens = self.kv_lens() if lens is None else lens
        return int(np.sum(np.asarray(lens, dtype=np.int64))) * self.d_qk * 2

    def flops(self, lens=None) -> int:
        """2 * (d_qk + d_latent) per key, row and head (the causal trim of the last q_len - 1 keys ignored)."""
        lens = self.kv_lens() if lens is None else lens
        return int(np.sum(np.asarray(lens, dtype=np.int64))) * self.q_len * self.n_heads * 2 * (self.d_qk + self.d_latent)

    def make_q(self) -> np.ndarray:
        """Queries scaled so that scores have unit variance, as trained attention has: N(0,1) / sqrt(d_qk / 192)."""
        n = self.batch * self.q_len * self.n_heads * self.d_qk
        z = bf16_to_f32(normal_bf16(self.seed, 0, n)) * np.float32(math.sqrt(192.0 / self.d_qk))
        return f32_to_bf16(z).reshape(self.batch, self.q_len, self.n_heads, self.d_qk)

    def make_c(self, b: int, length: int) -> np.ndarray:
        return normal_bf16(self.seed, 1 + b, length * self.d_qk).reshape(length, self.d_qk)

    def make_cache(self, lens=None):
        lens = self.kv_lens() if lens is None else lens
        return [self.make_c(b, int(L)) for b, L in enumerate(lens)]

    def scaled(self, name: str, batch: int, len_div: int, n_heads: Optional[int] = None) -> "MlaWorkload":
        lo, hi = self.len_args
        return replace(self, name=name, batch=batch, len_args=(max(1, lo // len_div), max(2, hi // len_div)),
                       n_heads=self.n_heads if n_heads is None else n_heads)

@dataclass(frozen=True)
class BeamWorkload:
    """One beam-search selection step of a generative-recommendation request batch (host side): per
    live sequence the top_k next-token log-probabilities of a softmax over `vocab` logits."""
    name: str
    n_req: int
    beam_width: int
    top_k: int
    seed: int
    vocab: int = 8192
    logit_std: float = 2.5      # spread of the synthetic logits: the softmax is neither flat nor one-hot
    note: str = ""

    def make(self):
        """(beam_lp [R, W] float32 descending, cand_lp [R, W, K] float32 descending along K, cand_tok int32).
        The log-softmax and the top-k are the sampler's job, upstream of the selection: input preparation."""
        R, W, K, V = self.n_req, self.beam_width, self.top_k, self.vocab
        cand_lp = np.empty((R, W, K), np.float32)
        cand_tok = np.empty((R, W, K), np.int32)
        for r in range(R):
            z = bf16_to_f32(normal_bf16(self.seed, 1 + r, W * V)).astype(np.float64).reshape(W, V) * self.logit_std
            lse = np.log(np.sum(np.exp(z - z.max(axis=1, keepdims=True)), axis=1, keepdims=True)) + z.max(axis=1, keepdims=True)
            lp = (z - lse).astype(np.float32)
            idx = np.argsort(-lp, axis=1, kind="stable")[:, :K]
            cand_tok[r] = idx.astype(np.int32)
            cand_lp[r] = np.take_along_axis(lp, idx, axis=1)
        u = uniform_u64(self.seed, 0, R * W).astype(np.float64) / float(1 << 64)
        beam_lp = -np.sort(2.0 + 6.0 * u.reshape(R, W), axis=1).astype(np.float32)     # in [-8, -2], descending
        return beam_lp, cand_lp, cand_tok


BEAM_CONFIGS = {
    "beam_small": BeamWorkload("beam_small", 2, 4, 8, seed=7, vocab=512, note="smallest beam width the paper plots"),
    "beam_128": BeamWorkload("beam_128", 8, 128, 128, seed=8, note="largest beam width the paper plots, top_k = beam width"),
    "beam_128x512": BeamWorkload("beam_128x512", 8, 128, 512, seed=9, note="large top_k: the host-bound regime"),
}


MLA_CONFIGS = {
    "mla_decode": MlaWorkload("mla_decode", 64, 1, 128, seed=5, len_args=(1024, 8192),
                              note="DeepSeek-style latent KV, 128 heads under DP attention, plain decode"),
    "mla_verify": MlaWorkload("mla_verify", 64, 2, 128, seed=6, len_args=(1024, 8192),
                              note="one speculated token (MTP): 2 query tokens per sequence"),
}

CONFIGS = {
    "tiny": Workload("tiny", 4, 1, 8, 2, 128, seed=0, len_kind="fixed", len_args=(17, 64, 100, 256),
                     note="parity / latency only"),
    "qwen3_8b_decode": Workload("qwen3_8b_decode", 64, 1, 32, 8, 128, seed=1, len_kind="uniform",
                                len_args=(512, 4096), xtensor=True,
                                note="Qwen3-8B-shaped plain decode"),
    "long_context": Workload("long_context", 16, 1, 64, 8, 128, seed=2, len_kind="uniform",
                             len_args=(16384, 32768), note="split-KV stress"),
    "spec_verify": Workload("spec_verify", 128, 4, 32, 8, 128, seed=3, len_kind="uniform",
                            len_args=(1024, 8192), note="3 draft tokens + 1, causal inside the block"),
    "skewed_xtensor": Workload("skewed_xtensor", 256, 1, 40, 8, 128, seed=4, len_kind="lognormal",
                               len_args=(1024, 1.2, 16, 65536), xtensor=True,
                               note="skewed batch on randomly ordered 2 MiB physical chunks"),
}
CONFIG_ORDER = ["tiny", "qwen3_8b_decode", "long_context", "spec_verify", "skewed_xtensor"]
