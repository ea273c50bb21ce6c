"""ctypes binding of libkvswitch: same names as the C ABI, argument marshalling only.

Every computation runs in the library's HIP kernels (device entry points) or its
C++ host code.  There is no Python or CPU fallback: if the shared library has
not been built, importing a function from here raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvswitch.so")

KV_OK, KV_EINVAL, KV_ESHAPE, KV_EBITS, KV_EINDEX, KV_ENOMEM, KV_EHIP = 0, -1, -2, -3, -4, -5, -6
KV_NORM_VISIBLE, KV_NORM_NONE = 0, 1
KV_FMT_F16_GROUPS, KV_FMT_I8_CHANNELS, KV_FMT_I8_CHANNELS_H, KV_FMT_F16_GROUPS_H = 0, 1, 2, 3
KV_OBJ_BITS_TO_DENSE, KV_OBJ_AS_PRINTED = 0, 1


class KvError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libkvswitch error {code}: {text}")
        self.code = code


class kv_shape_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "n_kv_heads", "n_q_heads", "head_dim", "n_tokens", "chunk_tokens", "group",
                 "format")]


class Shape(NamedTuple):
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    n_tokens: int
    chunk_tokens: int
    group: int
    format: int = 0      # KV_FMT_F16_GROUPS, KV_FMT_I8_CHANNELS, KV_FMT_I8_CHANNELS_H or KV_FMT_F16_GROUPS_H

    @property
    def cache_dtype(self):
        return torch.int8 if self.format in (KV_FMT_I8_CHANNELS, KV_FMT_I8_CHANNELS_H) else torch.float16

    @property
    def n_chunks(self) -> int:
        return self.n_tokens // self.chunk_tokens

    @property
    def slabs(self) -> int:
        return self.n_layers * 2 * self.n_kv_heads

    @property
    def kv_dims(self):
        return (self.n_layers, 2, self.n_kv_heads, self.n_tokens, self.head_dim)

    def c(self) -> kv_shape_t:
        return kv_shape_t(*self)


_lib = None
_vp, _i32, _u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64

_SIGNATURES = {
    "kv_last_error": (ctypes.c_char_p, []),
    "kv_record_bytes": (_u64, [_vp, _i32]),
    "kv_chunk_offsets": (_i32, [_vp, _vp, _vp]),
    "kv_bits_from_scores": (_i32, [_vp, _i32, _i32, _i32, _i32, _vp]),
    "kv_bits_optimise": (_i32, [_vp, _i32, _i32, _i32, _i32, _vp, _vp]),
    "kv_fit_line": (_i32, [_vp, _vp, _i32, _vp, _vp]),
    "kv_plan_pipeline": (_i32, [_vp, _vp, _vp, _vp, _vp]),
    "kv_pipeline_split": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "kv_build_gather": (_i32, [_vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]),
    "kv_score_workspace_bytes": (_u64, [_vp, _i32]),
    "kv_score_chunks": (_i32, [_vp, _vp, _i32, _vp, _i32, _vp, _u64, _vp, _vp, _vp]),
    "kv_score_chunks_valid": (_i32, [_vp, _vp, _i32, _vp, _i32, _i32, _vp, _u64, _vp, _vp, _vp]),
    "kv_score_chunks_static": (_i32, [_vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp]),
    "kv_compress_chunks": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "kv_swapin_chunks": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "kv_swapin_layers": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp]),
    "kv_compress_selected": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "kv_load_chunks": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "kv_plan_chunks_dev": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp]),
    "kv_plan_optimise_dev": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp]),
    "kv_swapin_pinned": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _u64, _i32, _vp, _vp, _vp]),
    "kv_loader_create": (_vp, []),
    "kv_loader_destroy": (None, [_vp]),
    "kv_swapin_stream": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _u64, _i32, _vp, _vp, _vp]),
    "kv_swapout_aot": (_i32, [_vp, _vp, _u64, _u64, _vp, _vp]),
    "kv_recompute_create": (_vp, []),
    "kv_recompute_destroy": (None, [_vp]),
    "kv_recompute_workspace_bytes": (_u64, [_vp, _vp, _i32]),
    "kv_recompute_tune": (_i32, [_vp, _vp, _vp, _vp, _i32, _vp, _u64, _vp, _vp]),
    "kv_recompute_layer": (_i32, [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _u64, _vp]),
    "kv_lctru_create": (_vp, []),
    "kv_lctru_destroy": (None, [_vp]),
    "kv_lctru_insert": (_i32, [_vp, _i32, _i32, _i32, _u64, _u64]),
    "kv_lctru_touch_ctx": (_i32, [_vp, _i32, _u64]),
    "kv_lctru_lock": (_i32, [_vp, _i32]),
    "kv_lctru_unlock": (_i32, [_vp, _i32]),
    "kv_lctru_evict": (_i32, [_vp, _u64, _vp, _vp, _i32, _vp]),
    "kv_lctru_order": (_i32, [_vp, _vp, _vp, _i32, _vp]),
    "kv_lctru_remove_ctx": (_i32, [_vp, _i32]),
    "kv_lctru_size": (_i32, [_vp, _vp, _vp]),
}


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2403_11805_amd.build); "
                "there is no fallback path")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def kv_last_error() -> str:
    return lib().kv_last_error().decode()


def _check(rc: int) -> None:
    if rc != KV_OK:
        raise KvError(rc, kv_last_error())


def _np(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _hp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dev(t: torch.Tensor, dtype=None) -> int:
    if not t.is_cuda:
        raise TypeError("expected a device tensor")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _dev_or_pinned(t: torch.Tensor, dtype=None) -> int:
    """A record pool: device memory, or pinned host memory that the kernels read over the host link."""
    if t.is_cuda:
        return _dev(t, dtype)
    if not t.is_pinned():
        raise TypeError("expected a device tensor or a pinned host tensor")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


# ------------------------------------------------- recompute of interleaved chunks

class kv_layer_dims_t(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("rope_base", ctypes.c_float), ("rms_eps", ctypes.c_float)]


LAYER_WEIGHTS = ("w_norm1", "wq", "wk", "wv", "wo", "w_norm2", "w_gate", "w_up", "w_down")


class kv_layer_weights_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in LAYER_WEIGHTS]


class LayerDims(NamedTuple):
    d_model: int
    d_ff: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5

    def c(self) -> kv_layer_dims_t:
        return kv_layer_dims_t(*self)


def kv_recompute_workspace_bytes(shape: Shape, dims: LayerDims, n_missing: int) -> int:
    s, d = shape.c(), dims.c()
    n = int(lib().kv_recompute_workspace_bytes(ctypes.byref(s), ctypes.byref(d), n_missing))
    if n == 0:
        raise KvError(KV_EINVAL, kv_last_error())
    return n


class Recompute:
    """Handle of the recompute path (kv_recompute_create / kv_recompute_destroy)."""

    def __init__(self):
        self._h = lib().kv_recompute_create()
        if not self._h:
            raise KvError(KV_EHIP, kv_last_error())

    def close(self):
        if self._h:
            lib().kv_recompute_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def tune(self, shape: Shape, dims: LayerDims, weights: dict, n_missing: int, workspace: torch.Tensor,
             stream=None) -> int:
        """kv_recompute_tune: synchronises the stream; returns the number of GEMM shapes that got another kernel."""
        s, d = shape.c(), dims.c()
        w = kv_layer_weights_t(*[_dev(weights[n], torch.float16) for n in LAYER_WEIGHTS])
        improved = ctypes.c_int32(0)
        _check(lib().kv_recompute_tune(self._h, ctypes.byref(s), ctypes.byref(d), ctypes.byref(w), n_missing,
                                       _dev(workspace), workspace.numel() * workspace.element_size(),
                                       _stream(stream), ctypes.byref(improved)))
        return improved.value

    def layer(self, shape: Shape, dims: LayerDims, weights: dict, layer: int, chunk_idx_dev: torch.Tensor,
              x_in: torch.Tensor, kv: torch.Tensor, x_out: torch.Tensor, workspace: torch.Tensor,
              stream=None) -> None:
        """kv_recompute_layer: argument marshalling only."""
        s, d = shape.c(), dims.c()
        n_missing = chunk_idx_dev.numel()
        rows = n_missing * shape.chunk_tokens
        if tuple(x_in.shape) != (rows, dims.d_model) or tuple(x_out.shape) != (rows, dims.d_model):
            raise ValueError("x_in / x_out must be [n_missing * chunk_tokens][d_model]")
        if tuple(kv.shape) != shape.kv_dims:
            raise ValueError("kv must be [L][2][Hkv][N][D]")
        w = kv_layer_weights_t(*[_dev(weights[n], torch.float16) for n in LAYER_WEIGHTS])
        _check(lib().kv_recompute_layer(self._h, ctypes.byref(s), ctypes.byref(d), ctypes.byref(w), layer,
                                        _dev(chunk_idx_dev, torch.int32), n_missing,
                                        _dev(x_in, torch.float16), _dev(kv, torch.float16),
                                        _dev(x_out, torch.float16), _dev(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)))


# ------------------------------------------------------------------ host, pure

def kv_record_bytes(shape: Shape, bits: int) -> int:
    s = shape.c()
    n = int(lib().kv_record_bytes(ctypes.byref(s), bits))
    if n == 0:
        raise KvError(KV_EINVAL, kv_last_error())
    return n


def kv_chunk_offsets(shape: Shape, bits) -> np.ndarray:
    s = shape.c()
    bits = _np(bits, np.uint8)
    if bits.shape != (shape.n_chunks,):
        raise ValueError("bits must have n_chunks entries")
    off = np.empty(shape.n_chunks + 1, dtype=np.uint64)
    _check(lib().kv_chunk_offsets(ctypes.byref(s), _hp(bits), _hp(off)))
    return off


def kv_bits_from_scores(density, num8: int, num4: int, den: int) -> np.ndarray:
    density = _np(density, np.float32)
    bits = np.empty(len(density), dtype=np.uint8)
    _check(lib().kv_bits_from_scores(_hp(density), len(density), num8, num4, den, _hp(bits)))
    return bits


def kv_bits_optimise(density, ratio_num: int, ratio_den: int, objective: int = KV_OBJ_BITS_TO_DENSE):
    """-> (bits uint8 [n], (k8, k4, k2))."""
    density = _np(density, np.float32)
    bits = np.empty(len(density), dtype=np.uint8)
    counts = np.zeros(3, dtype=np.int32)
    _check(lib().kv_bits_optimise(_hp(density), len(density), ratio_num, ratio_den, objective,
                                  _hp(bits), _hp(counts)))
    return bits, tuple(int(c) for c in counts)


class kv_pipeline_model_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("re_per_chunk", "re_fixed", "io_per_byte", "io_fixed")]


def kv_fit_line(x, t):
    """-> (slope, intercept) of the least-squares line through the points."""
    x, t = _np(x, np.float64), _np(t, np.float64)
    if len(x) != len(t):
        raise ValueError("x and t differ in length")
    a, b = ctypes.c_double(), ctypes.c_double()
    _check(lib().kv_fit_line(_hp(x), _hp(t), len(x), ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def kv_plan_pipeline(model, missing, record_bytes):
    """model = (re_per_chunk, re_fixed, io_per_byte, io_fixed) -> (recompute[3], delay)."""
    m = kv_pipeline_model_t(*[float(v) for v in model])
    missing, record_bytes = _np(missing, np.int32), _np(record_bytes, np.uint64)
    if missing.shape != (3,) or record_bytes.shape != (3,):
        raise ValueError("missing and record_bytes have three entries (8, 4, 2 bits)")
    out = np.zeros(3, dtype=np.int32)
    d = ctypes.c_double()
    _check(lib().kv_plan_pipeline(ctypes.byref(m), _hp(missing), _hp(record_bytes), _hp(out), ctypes.byref(d)))
    return tuple(int(v) for v in out), d.value


def kv_pipeline_split(shape: Shape, bits, missing_idx, recompute):
    """-> (recompute_idx, load_idx), both int32 ascending."""
    s = shape.c()
    bits, missing_idx = _np(bits, np.uint8), _np(missing_idx, np.int32)
    if len(bits) != shape.n_chunks:
        raise ValueError("bits must have n_chunks entries")
    plan = _np(recompute, np.int32)
    if len(plan) != 3:
        raise ValueError("recompute must have 3 entries")
    n = len(missing_idx)
    re_idx, io_idx = np.empty(max(n, 1), dtype=np.int32), np.empty(max(n, 1), dtype=np.int32)
    n_re, n_io = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().kv_pipeline_split(ctypes.byref(s), _hp(bits), _hp(missing_idx), n, _hp(plan), _hp(re_idx),
                                   ctypes.byref(n_re), _hp(io_idx), ctypes.byref(n_io)))
    return re_idx[:n_re.value].copy(), io_idx[:n_io.value].copy()


def kv_build_gather(shape: Shape, off, bits, chunk_idx):
    s = shape.c()
    off, bits, idx = _np(off, np.uint64), _np(bits, np.uint8), _np(chunk_idx, np.int32)
    if off.shape != (shape.n_chunks + 1,) or bits.shape != (shape.n_chunks,):
        raise ValueError("off/bits have the wrong length")
    n = len(idx)
    src_off = np.empty(n, dtype=np.uint64)
    dst_tok = np.empty(n, dtype=np.int32)
    sel_bits = np.empty(n, dtype=np.uint8)
    _check(lib().kv_build_gather(ctypes.byref(s), _hp(off), _hp(bits), _hp(idx), n,
                                 _hp(src_off), _hp(dst_tok), _hp(sel_bits)))
    return src_off, dst_tok, sel_bits


# ------------------------------------------------------------------ device, async

def kv_score_workspace_bytes(shape: Shape, n_queries: int) -> int:
    s = shape.c()
    n = int(lib().kv_score_workspace_bytes(ctypes.byref(s), n_queries))
    if n == 0:
        raise KvError(KV_ESHAPE, kv_last_error())
    return n


def kv_score_chunks(shape: Shape, q: torch.Tensor, kv: torch.Tensor, norm_mode: int,
                    workspace: torch.Tensor, chunk_mass: torch.Tensor, density: torch.Tensor,
                    stream=None) -> None:
    s = shape.c()
    n_queries = q.shape[2]
    if tuple(q.shape) != (shape.n_layers, shape.n_q_heads, n_queries, shape.head_dim):
        raise ValueError("q must be [L][Hq][R][D]")
    if tuple(kv.shape) != shape.kv_dims:
        raise ValueError("kv must be [L][2][Hkv][N][D]")
    if chunk_mass.numel() != shape.n_layers * shape.n_q_heads * shape.n_chunks or \
            density.numel() != shape.n_chunks:
        raise ValueError("chunk_mass/density have the wrong size")
    _check(lib().kv_score_chunks(ctypes.byref(s), _dev(q, torch.float16), n_queries,
                                 _dev(kv, torch.float16), norm_mode, _dev(workspace),
                                 workspace.numel() * workspace.element_size(),
                                 _dev(chunk_mass, torch.float32), _dev(density, torch.float32),
                                 _stream(stream)))


def kv_score_chunks_valid(shape: Shape, q: torch.Tensor, kv: torch.Tensor, n_valid: int, norm_mode: int,
                          workspace: torch.Tensor, chunk_mass: torch.Tensor, density: torch.Tensor,
                          stream=None) -> None:
    s = shape.c()
    n_queries = q.shape[2]
    if tuple(q.shape) != (shape.n_layers, shape.n_q_heads, n_queries, shape.head_dim):
        raise ValueError("q must be [L][Hq][R][D]")
    if tuple(kv.shape) != shape.kv_dims:
        raise ValueError("kv must be [L][2][Hkv][N][D]")
    if chunk_mass.numel() != shape.n_layers * shape.n_q_heads * shape.n_chunks or \
            density.numel() != shape.n_chunks:
        raise ValueError("chunk_mass/density have the wrong size")
    _check(lib().kv_score_chunks_valid(ctypes.byref(s), _dev(q, torch.float16), n_queries,
                                       _dev(kv, torch.float16), int(n_valid), norm_mode, _dev(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _dev(chunk_mass, torch.float32), _dev(density, torch.float32),
                                       _stream(stream)))


KV_SCORE_STATIC_BYTES = 32 << 20
KV_RECOMPUTE_OWN_GEMM_ROWS = 512


def kv_score_chunks_static(shape: Shape, q: torch.Tensor, kv: torch.Tensor, norm_mode: int,
                           chunk_mass: torch.Tensor, density: torch.Tensor, stream=None) -> None:
    s = shape.c()
    n_queries = q.shape[2]
    if tuple(q.shape) != (shape.n_layers, shape.n_q_heads, n_queries, shape.head_dim):
        raise ValueError("q must be [L][Hq][R][D]")
    if tuple(kv.shape) != shape.kv_dims:
        raise ValueError("kv must be [L][2][Hkv][N][D]")
    if chunk_mass.numel() != shape.n_layers * shape.n_q_heads * shape.n_chunks or \
            density.numel() != shape.n_chunks:
        raise ValueError("chunk_mass/density have the wrong size")
    _check(lib().kv_score_chunks_static(ctypes.byref(s), _dev(q, torch.float16), n_queries,
                                        _dev(kv, torch.float16), norm_mode,
                                        _dev(chunk_mass, torch.float32), _dev(density, torch.float32),
                                        _stream(stream)))


def kv_compress_chunks(shape: Shape, kv: torch.Tensor, bits_dev: torch.Tensor,
                       off_dev: torch.Tensor, packed_out: torch.Tensor, stream=None) -> None:
    s = shape.c()
    if tuple(kv.shape) != shape.kv_dims:
        raise ValueError("kv must be [L][2][Hkv][N][D]")
    if bits_dev.numel() != shape.n_chunks or off_dev.numel() != shape.n_chunks + 1:
        raise ValueError("bits_dev/off_dev have the wrong length")
    _check(lib().kv_compress_chunks(ctypes.byref(s), _dev(kv, shape.cache_dtype),
                                    _dev(bits_dev, torch.uint8), _dev(off_dev, torch.int64),
                                    _dev(packed_out, torch.uint8), _stream(stream)))


def kv_compress_selected(shape: Shape, kv: torch.Tensor, bits_dev: torch.Tensor, off_dev: torch.Tensor,
                         chunk_idx_dev: torch.Tensor, packed_out: torch.Tensor, stream=None) -> None:
    s = shape.c()
    if tuple(kv.shape) != shape.kv_dims:
        raise ValueError("kv must be [L][2][Hkv][N][D]")
    if bits_dev.numel() != shape.n_chunks or off_dev.numel() != shape.n_chunks + 1:
        raise ValueError("need bits of n_chunks entries and off of n_chunks + 1")
    n_sel = chunk_idx_dev.numel()
    if n_sel == 0:
        return
    _check(lib().kv_compress_selected(ctypes.byref(s), _dev(kv, shape.cache_dtype), _dev(bits_dev, torch.uint8),
                                      _dev(off_dev, torch.int64), _dev(chunk_idx_dev, torch.int32), n_sel,
                                      _dev(packed_out, torch.uint8), _stream(stream)))


def kv_plan_chunks_dev(shape: Shape, density_dev: torch.Tensor, num8: int, num4: int, den: int,
                       bits_dev: torch.Tensor, off_dev: torch.Tensor, dst_tok_dev: torch.Tensor,
                       stream=None) -> None:
    s = shape.c()
    n = shape.n_chunks
    if density_dev.numel() != n or bits_dev.numel() != n or dst_tok_dev.numel() != n or off_dev.numel() != n + 1:
        raise ValueError("need density/bits/dst_tok of n_chunks entries and off of n_chunks + 1")
    _check(lib().kv_plan_chunks_dev(ctypes.byref(s), _dev(density_dev, torch.float32), num8, num4, den,
                                    _dev(bits_dev, torch.uint8), _dev(off_dev, torch.int64),
                                    _dev(dst_tok_dev, torch.int32), _stream(stream)))


def kv_plan_optimise_dev(shape: Shape, density_dev: torch.Tensor, ratio_num: int, ratio_den: int, objective: int,
                         bits_dev: torch.Tensor, off_dev: torch.Tensor, dst_tok_dev: torch.Tensor,
                         counts_dev: torch.Tensor = None, stream=None) -> None:
    s = shape.c()
    n = shape.n_chunks
    if density_dev.numel() != n or bits_dev.numel() != n or dst_tok_dev.numel() != n or off_dev.numel() != n + 1:
        raise ValueError("need density/bits/dst_tok of n_chunks entries and off of n_chunks + 1")
    if counts_dev is not None and counts_dev.numel() != 3:
        raise ValueError("counts_dev must have 3 entries")
    _check(lib().kv_plan_optimise_dev(ctypes.byref(s), _dev(density_dev, torch.float32), ratio_num, ratio_den,
                                      objective, _dev(bits_dev, torch.uint8), _dev(off_dev, torch.int64),
                                      _dev(dst_tok_dev, torch.int32),
                                      None if counts_dev is None else _dev(counts_dev, torch.int32),
                                      _stream(stream)))


def kv_swapin_chunks(shape: Shape, packed: torch.Tensor, src_off_dev: torch.Tensor,
                     dst_tok_dev: torch.Tensor, sel_bits_dev: torch.Tensor, kv_out: torch.Tensor,
                     stream=None) -> None:
    s = shape.c()
    n_sel = src_off_dev.numel()
    if dst_tok_dev.numel() != n_sel or sel_bits_dev.numel() != n_sel:
        raise ValueError("gather lists differ in length")
    if tuple(kv_out.shape) != shape.kv_dims:
        raise ValueError("kv_out must be [L][2][Hkv][N][D]")
    if n_sel == 0:
        return
    _check(lib().kv_swapin_chunks(ctypes.byref(s), _dev_or_pinned(packed, torch.uint8),
                                  _dev(src_off_dev, torch.int64), _dev(dst_tok_dev, torch.int32),
                                  _dev(sel_bits_dev, torch.uint8), n_sel,
                                  _dev(kv_out, shape.cache_dtype), _stream(stream)))


def kv_swapin_layers(shape: Shape, packed: torch.Tensor, src_off_dev: torch.Tensor,
                     dst_tok_dev: torch.Tensor, sel_bits_dev: torch.Tensor, layer_begin: int,
                     layer_end: int, kv_out: torch.Tensor, stream=None) -> None:
    s = shape.c()
    n_sel = src_off_dev.numel()
    if dst_tok_dev.numel() != n_sel or sel_bits_dev.numel() != n_sel:
        raise ValueError("gather lists differ in length")
    if tuple(kv_out.shape) != shape.kv_dims:
        raise ValueError("kv_out must be [L][2][Hkv][N][D]")
    _check(lib().kv_swapin_layers(ctypes.byref(s), _dev_or_pinned(packed, torch.uint8) if n_sel else None,
                                  _dev(src_off_dev, torch.int64) if n_sel else None,
                                  _dev(dst_tok_dev, torch.int32) if n_sel else None,
                                  _dev(sel_bits_dev, torch.uint8) if n_sel else None, n_sel,
                                  int(layer_begin), int(layer_end),
                                  _dev(kv_out, shape.cache_dtype), _stream(stream)))


def kv_load_chunks(shape: Shape, packed: torch.Tensor, off, bits, chunk_idx, kv_out: torch.Tensor,
                   stream=None) -> None:
    s = shape.c()
    off, bits, chunk_idx = _np(off, np.uint64), _np(bits, np.uint8), _np(chunk_idx, np.int32)
    if len(off) != shape.n_chunks + 1 or len(bits) != shape.n_chunks:
        raise ValueError("need off of n_chunks + 1 entries and bits of n_chunks entries")
    if tuple(kv_out.shape) != shape.kv_dims:
        raise ValueError("kv_out must be [L][2][Hkv][N][D]")
    _check(lib().kv_load_chunks(ctypes.byref(s), _dev_or_pinned(packed, torch.uint8), _hp(off), _hp(bits),
                                _hp(chunk_idx), len(chunk_idx), _dev(kv_out, shape.cache_dtype),
                                _stream(stream)))


def kv_swapin_pinned(shape: Shape, packed_pinned: torch.Tensor, src_off, dst_tok, sel_bits,
                     staging_dev: torch.Tensor, n_buffers: int, kv_out: torch.Tensor,
                     copy_stream, compute_stream) -> None:
    s = shape.c()
    if packed_pinned.is_cuda or not packed_pinned.is_pinned():
        raise TypeError("packed_pinned must be a pinned host tensor")
    src_off, dst_tok, sel_bits = _np(src_off, np.uint64), _np(dst_tok, np.int32), _np(sel_bits, np.uint8)
    n_sel = len(src_off)
    if len(dst_tok) != n_sel or len(sel_bits) != n_sel:
        raise ValueError("gather lists differ in length")
    if tuple(kv_out.shape) != shape.kv_dims:
        raise ValueError("kv_out must be [L][2][Hkv][N][D]")
    _check(lib().kv_swapin_pinned(ctypes.byref(s), packed_pinned.data_ptr(), _hp(src_off),
                                  _hp(dst_tok), _hp(sel_bits), n_sel, _dev(staging_dev),
                                  staging_dev.numel() * staging_dev.element_size(), n_buffers,
                                  _dev(kv_out, shape.cache_dtype), _stream(copy_stream),
                                  _stream(compute_stream)))


class Loader:
    """Owner of a kv_loader_t handle (kv_loader_create / kv_loader_destroy); swapin_stream is
    kv_swapin_stream."""

    def __init__(self):
        self._h = lib().kv_loader_create()
        if not self._h:
            raise KvError(KV_EHIP, kv_last_error())

    def close(self):
        if self._h:
            lib().kv_loader_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def swapin_stream(self, shape: Shape, packed_pinned: torch.Tensor, src_off, dst_tok, sel_bits,
                      staging_dev: torch.Tensor, n_buffers: int, kv_out: torch.Tensor,
                      copy_stream, compute_stream) -> None:
        s = shape.c()
        if packed_pinned.is_cuda or not packed_pinned.is_pinned():
            raise TypeError("packed_pinned must be a pinned host tensor")
        src_off, dst_tok, sel_bits = _np(src_off, np.uint64), _np(dst_tok, np.int32), _np(sel_bits, np.uint8)
        n_sel = len(src_off)
        if len(dst_tok) != n_sel or len(sel_bits) != n_sel:
            raise ValueError("gather lists differ in length")
        if kv_out.numel() != int(np.prod(shape.kv_dims)):
            raise ValueError("kv_out must hold [L][2][Hkv][N][D]")
        _check(lib().kv_swapin_stream(self._h, ctypes.byref(s), packed_pinned.data_ptr(), _hp(src_off),
                                      _hp(dst_tok), _hp(sel_bits), n_sel, _dev(staging_dev),
                                      staging_dev.numel() * staging_dev.element_size(), n_buffers,
                                      _dev(kv_out, shape.cache_dtype), _stream(copy_stream),
                                      _stream(compute_stream)))


def kv_swapout_aot(packed_dev: torch.Tensor, packed_pinned: torch.Tensor, begin: int, end: int,
                   producer_stream, copy_stream) -> None:
    if packed_pinned.is_cuda or not packed_pinned.is_pinned():
        raise TypeError("packed_pinned must be a pinned host tensor")
    nbytes = packed_dev.numel() * packed_dev.element_size()
    if end > nbytes or end > packed_pinned.numel() * packed_pinned.element_size():
        raise ValueError("range exceeds a buffer")
    _check(lib().kv_swapout_aot(_dev(packed_dev), packed_pinned.data_ptr(), begin, end,
                                _stream(producer_stream), _stream(copy_stream)))


# ------------------------------------------------------------------ host lifecycle

class Lctru:
    """Thin owner of a kv_lctru_t handle; methods are the kv_lctru_* calls."""

    def __init__(self):
        self._h = lib().kv_lctru_create()
        if not self._h:
            raise MemoryError("kv_lctru_create failed")

    def close(self):
        if self._h:
            lib().kv_lctru_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def insert(self, ctx, chunk, bits, nbytes, now):
        _check(lib().kv_lctru_insert(self._h, ctx, chunk, bits, nbytes, now))

    def touch_ctx(self, ctx, now):
        _check(lib().kv_lctru_touch_ctx(self._h, ctx, now))

    def lock(self, ctx):
        _check(lib().kv_lctru_lock(self._h, ctx))

    def unlock(self, ctx):
        _check(lib().kv_lctru_unlock(self._h, ctx))

    def remove_ctx(self, ctx):
        _check(lib().kv_lctru_remove_ctx(self._h, ctx))

    def size(self):
        n = ctypes.c_int32()
        b = ctypes.c_uint64()
        _check(lib().kv_lctru_size(self._h, ctypes.byref(n), ctypes.byref(b)))
        return n.value, b.value

    def _lists(self, fn, *head):
        cap = self.size()[0]
        ctx = np.empty(max(cap, 1), dtype=np.int32)
        chunk = np.empty(max(cap, 1), dtype=np.int32)
        n = ctypes.c_int32()
        rc = fn(self._h, *head, _hp(ctx), _hp(chunk), cap, ctypes.byref(n))
        return rc, list(zip(ctx[:n.value].tolist(), chunk[:n.value].tolist()))

    def order(self):
        rc, out = self._lists(lib().kv_lctru_order)
        _check(rc)
        return out

    def evict(self, bytes_needed):
        """Popped (ctx, chunk) pairs, or None if the unlocked chunks cannot free that much."""
        rc, out = self._lists(lib().kv_lctru_evict, bytes_needed)
        if rc == KV_ENOMEM:
            return None
        _check(rc)
        return out
