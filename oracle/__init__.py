"""CPU oracle for the chunk-wise KV-cache context-switch path (arXiv 2403.11805).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  The product package never imports it and it
never imports the product package.  The arithmetic lives in kvoracle.c (plain
C, compiled here with gcc) and hostlogic.py (integer bookkeeping in plain
Python); this file only builds the C part and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from .hostlogic import (  # noqa: F401  (re-exported)
    LctruModel,
    bits_from_scores,
    bits_optimise,
    build_gather,
    chunk_offsets,
    fit_line,
    pipeline_delay,
    pipeline_split,
    plan_pipeline,
    record_bytes,
)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvoracle.c")
_LIB = os.path.join(_HERE, "libkvoracle.so")

NORM_VISIBLE = 0
NORM_NONE = 1


class _CShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("L", "Hkv", "Hq", "D", "N", "T", "G", "fmt")]


@dataclass(frozen=True)
class Shape:
    """Geometry of one KV cache: [L][2][Hkv][N][D] fp16, chunks of T tokens,
    quantisation groups of G consecutive head_dim elements."""
    L: int
    Hkv: int
    Hq: int
    D: int
    N: int
    T: int
    G: int
    fmt: int = 0    # 0: fp16 cache, groups of G along head_dim (3: binary16 parameters); 1: int8 cache, channel-wise;
                    # 2: as 1 with binary16 parameters

    @property
    def n_chunks(self) -> int:
        return self.N // self.T

    @property
    def slabs(self) -> int:
        return self.L * 2 * self.Hkv

    def c(self) -> _CShape:
        return _CShape(self.L, self.Hkv, self.Hq, self.D, self.N, self.T, self.G, self.fmt)


def build(force: bool = False) -> str:
    """Compile kvoracle.c into libkvoracle.so (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-fno-fast-math", "-fexcess-precision=standard",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_half_to_float.restype = ctypes.c_float
        _lib.orc_half_to_float.argtypes = [ctypes.c_uint16]
        _lib.orc_float_to_half.restype = ctypes.c_uint16
        _lib.orc_float_to_half.argtypes = [ctypes.c_float]
        _lib.orc_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(lib().orc_threads())


def set_threads(n: int) -> None:
    """Threads the C loops use from now on (the benchmark times the oracle on one core as well)."""
    lib().orc_set_threads(ctypes.c_int(int(n)))


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    """fp16 array (numpy float16 or uint16 bit patterns) -> contiguous uint16 view."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def half_to_float(bits: int) -> float:
    return float(lib().orc_half_to_float(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().orc_float_to_half(float(x)))


def attention(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """A = softmax(mask(Q K^T / sqrt(D))) for one head; q [R][D], k [N][D] fp16 -> float64 [R][N]."""
    q, k = _u16(q), _u16(k)
    R, D = q.shape
    N = k.shape[0]
    assert k.shape[1] == D and R <= N
    A = np.empty((R, N), dtype=np.float64)
    lib().orc_attention(_p(q), _p(k), ctypes.c_int(R), ctypes.c_int(N), ctypes.c_int(D), _p(A))
    return A


def column_density(A: np.ndarray, T: int, norm_mode: int = NORM_VISIBLE) -> np.ndarray:
    """Per-chunk mass of one attention matrix (float64 [R][N]) -> float64 [N/T]."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    R, N = A.shape
    assert N % T == 0
    out = np.empty(N // T, dtype=np.float64)
    lib().orc_column_density(_p(A), ctypes.c_int(R), ctypes.c_int(N), ctypes.c_int(T),
                             ctypes.c_int(norm_mode), _p(out))
    return out


def score_head(shape: Shape, q, kv, layer: int, head: int,
               norm_mode: int = NORM_VISIBLE) -> np.ndarray:
    """Chunk mass of one (layer, query head) -> float64 [n_chunks]."""
    q, kv = _u16(q), _u16(kv)
    R = q.shape[2]
    assert q.shape == (shape.L, shape.Hq, R, shape.D)
    assert kv.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    out = np.empty(shape.n_chunks, dtype=np.float64)
    cs = shape.c()
    rc = lib().orc_score_head(ctypes.byref(cs), _p(q), ctypes.c_int(R), _p(kv),
                              ctypes.c_int(layer), ctypes.c_int(head),
                              ctypes.c_int(norm_mode), _p(out))
    assert rc == 0
    return out


def score_chunks(shape: Shape, q, kv, norm_mode: int = NORM_VISIBLE):
    """Eq. 1 over a whole context -> (chunk_mass fp32 [L][Hq][n_chunks], density fp32 [n_chunks])."""
    q, kv = _u16(q), _u16(kv)
    R = q.shape[2]
    assert q.shape == (shape.L, shape.Hq, R, shape.D)
    assert kv.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    cm = np.empty((shape.L, shape.Hq, shape.n_chunks), dtype=np.float32)
    dens = np.empty(shape.n_chunks, dtype=np.float32)
    cs = shape.c()
    rc = lib().orc_score_chunks(ctypes.byref(cs), _p(q), ctypes.c_int(R), _p(kv),
                                ctypes.c_int(norm_mode), _p(cm), _p(dens))
    assert rc == 0
    return cm, dens


def score_chunks_valid(shape: Shape, q, kv, n_valid: int, norm_mode: int = NORM_VISIBLE):
    """Eq. 1 for a context of n_valid tokens held in a cache padded to shape.N tokens: the valid
    prefix is scored as the context it is (the R query rows are its last R tokens, the padding is
    seen by no row), chunk i holds its tokens [iT, min((i+1)T, n_valid)), and the density is the
    mean per token the chunk really has (0 for a chunk made of padding only).
    -> (chunk_mass float64 [L][Hq][n_chunks], density float64 [n_chunks])."""
    q, kv = _u16(q), _u16(kv)
    R = q.shape[2]
    assert q.shape == (shape.L, shape.Hq, R, shape.D)
    assert kv.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    assert R <= n_valid <= shape.N
    T, n_chunks = shape.T, shape.n_chunks
    cm = np.zeros((shape.L, shape.Hq, n_chunks), dtype=np.float64)
    per_kv = shape.Hq // shape.Hkv
    for l in range(shape.L):
        for h in range(shape.Hq):
            A = attention(q[l, h], kv[l, 0, h // per_kv, :n_valid])
            col = column_density(A, 1, norm_mode)               # per-token mass of the valid prefix
            for i in range(n_chunks):
                cm[l, h, i] = col[i * T:min((i + 1) * T, n_valid)].sum()
    count = np.clip(n_valid - np.arange(n_chunks) * T, 0, T).astype(np.float64)
    total = cm.sum(axis=(0, 1))
    dens = np.where(count > 0, total / (np.maximum(count, 1) * shape.L * shape.Hq), 0.0)
    return cm, dens


def compress_chunks(shape: Shape, kv, bits: np.ndarray, off: np.ndarray) -> np.ndarray:
    """Quantise + pack all chunks -> uint8 pool of off[-1] bytes."""
    kv = _u16(kv)
    assert kv.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    off = np.ascontiguousarray(off, dtype=np.uint64)
    assert bits.shape == (shape.n_chunks,) and off.shape == (shape.n_chunks + 1,)
    packed = np.zeros(int(off[-1]), dtype=np.uint8)
    cs = shape.c()
    rc = lib().orc_compress_chunks(ctypes.byref(cs), _p(kv), _p(bits), _p(off), _p(packed))
    assert rc == 0, rc
    return packed


def swapin_chunks(shape: Shape, packed: np.ndarray, src_off, dst_tok, sel_bits,
                  kv_out: np.ndarray) -> np.ndarray:
    """Unpack + dequantise the listed records into kv_out (uint16/float16, modified in place)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    src_off = np.ascontiguousarray(src_off, dtype=np.uint64)
    dst_tok = np.ascontiguousarray(dst_tok, dtype=np.int32)
    sel_bits = np.ascontiguousarray(sel_bits, dtype=np.uint8)
    assert kv_out.flags["C_CONTIGUOUS"] and kv_out.dtype in (np.uint16, np.float16)
    assert kv_out.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    n_sel = len(src_off)
    assert len(dst_tok) == n_sel and len(sel_bits) == n_sel
    cs = shape.c()
    rc = lib().orc_swapin_chunks(ctypes.byref(cs), _p(packed), _p(src_off), _p(dst_tok),
                                 _p(sel_bits), ctypes.c_int(n_sel), _p(kv_out))
    assert rc == 0, rc
    return kv_out


def swapin_layers(shape: Shape, packed, src_off, dst_tok, sel_bits, layer_begin: int, layer_end: int,
                  kv_out: np.ndarray) -> np.ndarray:
    """Layer-wise Load (Sec. 3.3: the chunks of one layer are loaded while another is recomputed): what
    the Load of the listed records puts into the layers [layer_begin, layer_end); every other layer of
    kv_out keeps its contents.  Written as its definition: the whole Load into a copy, of which the
    layers in range are taken.  Any format (the cache's dtype says which)."""
    assert 0 <= layer_begin <= layer_end <= shape.L
    whole = kv_out.copy()
    if shape.fmt in (0, 3):
        swapin_chunks(shape, packed, src_off, dst_tok, sel_bits, whole)
    else:
        swapin_chunks_i8(shape, packed, src_off, dst_tok, sel_bits, whole)
    kv_out[layer_begin:layer_end] = whole[layer_begin:layer_end]
    return kv_out


def compress_chunks_i8(shape: Shape, kv, bits: np.ndarray, off: np.ndarray) -> np.ndarray:
    """Channel-wise quantise + pack of an int8 cache (format 1) -> uint8 pool."""
    kv = np.ascontiguousarray(kv, dtype=np.int8)
    assert shape.fmt in (1, 2) and kv.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    off = np.ascontiguousarray(off, dtype=np.uint64)
    assert bits.shape == (shape.n_chunks,) and off.shape == (shape.n_chunks + 1,)
    packed = np.zeros(int(off[-1]), dtype=np.uint8)
    cs = shape.c()
    rc = lib().orc_compress_chunks_i8(ctypes.byref(cs), _p(kv), _p(bits), _p(off), _p(packed))
    assert rc == 0, rc
    return packed


def swapin_chunks_i8(shape: Shape, packed, src_off, dst_tok, sel_bits, kv_out: np.ndarray) -> np.ndarray:
    """Unpack + dequantise listed records into an int8 cache (format 1), in place."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    src_off = np.ascontiguousarray(src_off, dtype=np.uint64)
    dst_tok = np.ascontiguousarray(dst_tok, dtype=np.int32)
    sel_bits = np.ascontiguousarray(sel_bits, dtype=np.uint8)
    assert shape.fmt in (1, 2) and kv_out.flags["C_CONTIGUOUS"] and kv_out.dtype == np.int8
    assert kv_out.shape == (shape.L, 2, shape.Hkv, shape.N, shape.D)
    cs = shape.c()
    rc = lib().orc_swapin_chunks_i8(ctypes.byref(cs), _p(packed), _p(src_off), _p(dst_tok),
                                    _p(sel_bits), ctypes.c_int(len(src_off)), _p(kv_out))
    assert rc == 0, rc
    return kv_out
