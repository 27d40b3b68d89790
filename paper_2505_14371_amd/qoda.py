"""Thin ctypes binding over libqoda.so (the C ABI of include/qoda.h).

Argument marshalling only: every step of the hot path runs in the library's HIP kernels.  Device memory is
passed as integer addresses (``tensor.data_ptr()``) and streams as ``torch.cuda.Stream.cuda_stream`` integers;
there is no CPU fallback -- a missing library is an ImportError-like failure at first use.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqoda.so")

OK, EINVAL, ENOMEM, EHIP, ENONFINITE, ETINYNORM = 0, -1, -2, -3, -4, -5
BUF_SUMSQ, BUF_NORM, BUF_INV, BUF_DELTA, BUF_HIST, BUF_POOLED = range(6)
NUM_KERNELS = 24
SCOPE_LAYER, SCOPE_VECTOR, SCOPE_BUCKET = 0, 1, 2
NORM_LINF, NORM_L1, NORM_L2 = 0, 1, 2
HIST_BINS, GRID_POINTS = 2048, 257

_lib = None


class QodaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"qoda error {code}: {msg}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("layer_size", C.POINTER(C.c_int64)), ("layer_type", C.POINTER(C.c_int32)),
                ("num_types", C.c_int32), ("type_points", C.POINTER(C.c_int32)), ("num_nodes", C.c_int32),
                ("norm_kind", C.c_int32), ("seed", C.c_uint64), ("norm_scope", C.c_int32)]


class _State(C.Structure):
    _fields_ = [("x1_dev", C.POINTER(C.c_void_p)), ("y_dev", C.POINTER(C.c_void_p)),
                ("x_half_dev", C.POINTER(C.c_void_p)), ("x_next_dev", C.POINTER(C.c_void_p)),
                ("acc_dev", C.c_void_p), ("eta_dev", C.c_void_p)]


class _AltState(C.Structure):
    _fields_ = [("x1_dev", C.POINTER(C.c_void_p)), ("y_dev", C.POINTER(C.c_void_p)),
                ("x_half_dev", C.POINTER(C.c_void_p)), ("x_next_dev", C.POINTER(C.c_void_p)),
                ("sums_dev", C.c_void_p), ("eta_dev", C.c_void_p)]


class _CodeLength(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("fixed_bits", "paper_bits", "entropy_bits", "huffman_bits", "nonzeros",
                                          "coordinates", "message_bits")]


def load():
    """Open libqoda.so (built by ``paper_2505_14371_amd.build``); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise QodaError(EINVAL, f"{LIB_PATH} is missing: build it with `python -m paper_2505_14371_amd.build` "
                                "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, pp = C.c_void_p, C.POINTER(C.c_void_p)
    L.qoda_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
    L.qoda_destroy.argtypes = [vp]
    L.qoda_message_bytes.argtypes = [vp]
    L.qoda_message_bytes.restype = C.c_size_t
    L.qoda_message_layout.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.qoda_set_levels.argtypes = [vp, C.c_int32, C.POINTER(C.c_float), vp]
    L.qoda_get_levels.argtypes = [vp, C.c_int32, C.POINTER(C.c_float), vp]
    L.qoda_fit_levels.argtypes = [vp, pp, C.c_uint32, vp]
    L.qoda_fit_levels_keep_norms.argtypes = [vp, pp, C.c_uint32, vp]
    L.qoda_gather_statistics.argtypes = [vp, C.c_int32]
    L.qoda_quantize.argtypes = [vp, C.c_int32, pp, C.c_uint32, vp, vp, vp]
    L.qoda_quantize_noalloc.argtypes = [vp, C.c_int32, pp, C.c_uint32, vp, vp, vp]
    L.qoda_quantize_all.argtypes = [vp, pp, C.c_uint32, pp, pp, vp]
    L.qoda_dequant_aggregate.argtypes = [vp, pp, pp, vp]
    L.qoda_step.argtypes = [vp, pp, C.POINTER(_State), vp]
    L.qoda_step_alt.argtypes = [vp, pp, C.POINTER(_AltState), C.c_double, vp]
    L.qoda_step_rates.argtypes = [vp, pp, C.POINTER(_State), vp, vp]
    L.qoda_extrapolate.argtypes = [vp, pp, pp, pp, vp, vp]
    L.qoda_index_counts.argtypes = [vp, pp, C.POINTER(C.c_uint64), vp]
    L.qoda_code_length.argtypes = [vp, C.POINTER(C.c_uint64), C.c_uint32, C.POINTER(_CodeLength)]
    L.qoda_read_buffer.argtypes = [vp, C.c_int32, vp, C.c_size_t, vp]
    L.qoda_status.argtypes = [vp, vp]
    L.qoda_profile_enable.argtypes = [vp, C.c_uint32]
    L.qoda_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), vp]
    L.qoda_kernel_name.argtypes = [C.c_int32]
    L.qoda_kernel_name.restype = C.c_char_p
    L.qoda_copy_calibration.argtypes = [vp, vp, vp, C.c_size_t, vp]
    L.qoda_stream_calibration.argtypes = [vp, vp, vp, C.c_size_t, C.c_int32, vp]
    L.qoda_last_error.argtypes = [vp]
    L.qoda_last_error.restype = C.c_char_p
    for name in ("qoda_create", "qoda_destroy", "qoda_message_layout", "qoda_set_levels", "qoda_get_levels",
                 "qoda_fit_levels", "qoda_fit_levels_keep_norms", "qoda_gather_statistics", "qoda_quantize", "qoda_quantize_noalloc", "qoda_quantize_all", "qoda_dequant_aggregate", "qoda_step", "qoda_step_alt",
                 "qoda_step_rates", "qoda_extrapolate", "qoda_index_counts", "qoda_code_length",
                 "qoda_read_buffer", "qoda_status", "qoda_profile_enable", "qoda_profile_read", "qoda_copy_calibration",
                 "qoda_stream_calibration"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _addr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptrs(xs) -> C.Array:
    if isinstance(xs, C.Array):          # built once by the caller with pointer_array(): passed through
        return xs
    arr = (C.c_void_p * len(xs))()
    for i, x in enumerate(xs):
        arr[i] = _addr(x)
    return arr


def pointer_array(xs: Sequence) -> C.Array:
    """A host array of device pointers in the form the library takes, for callers that pass the same set every
    round and do not want it rebuilt on every call (tensors or integer addresses; None -> NULL)."""
    return _ptrs(list(xs))


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class Context:
    """One model: layer sizes, layer -> type map, grid points per type, K nodes, generator seed."""

    def __init__(self, layer_size: Sequence[int], layer_type: Sequence[int], type_points: Sequence[int],
                 num_nodes: int, seed: int, norm_scope: int = SCOPE_LAYER, norm_kind: int = NORM_L2):
        self._lib = load()
        self.norm_scope = int(norm_scope)
        self.norm_kind = int(norm_kind)
        self.layer_size = np.ascontiguousarray(layer_size, dtype=np.int64)
        self.layer_type = np.ascontiguousarray(layer_type, dtype=np.int32)
        self.type_points = np.ascontiguousarray(type_points, dtype=np.int32)
        self.L, self.M, self.K = int(self.layer_size.size), int(self.type_points.size), int(num_nodes)
        cfg = _Config(self.L, self.layer_size.ctypes.data_as(C.POINTER(C.c_int64)),
                      self.layer_type.ctypes.data_as(C.POINTER(C.c_int32)), self.M,
                      self.type_points.ctypes.data_as(C.POINTER(C.c_int32)), self.K, self.norm_kind, seed, self.norm_scope)
        h = C.c_void_p()
        rc = self._lib.qoda_create(C.byref(cfg), C.byref(h))
        if rc != OK:
            raise QodaError(rc, "qoda_create failed (bad configuration, or no usable GPU)")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.qoda_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != OK:
            raise QodaError(rc, self._lib.qoda_last_error(self._h).decode())

    # -- layout
    def message_bytes(self) -> int:
        return int(self._lib.qoda_message_bytes(self._h))

    def message_layout(self):
        h = np.zeros(self.L, dtype=np.int64)
        b = np.zeros(self.L, dtype=np.int64)
        self._check(self._lib.qoda_message_layout(self._h, h.ctypes.data_as(C.POINTER(C.c_int64)),
                                                  b.ctypes.data_as(C.POINTER(C.c_int64))))
        return h, b

    # -- levels
    def set_levels(self, type_: int, levels, stream=None):
        lev = np.ascontiguousarray(levels, dtype=np.float32)
        if lev.size != self.type_points[type_]:
            raise QodaError(EINVAL, "set_levels: wrong number of levels")
        self._check(self._lib.qoda_set_levels(self._h, type_, lev.ctypes.data_as(C.POINTER(C.c_float)), _stream(stream)))

    def get_levels(self, type_: int, stream=None) -> np.ndarray:
        lev = np.zeros(int(self.type_points[type_]), dtype=np.float32)
        self._check(self._lib.qoda_get_levels(self._h, type_, lev.ctypes.data_as(C.POINTER(C.c_float)), _stream(stream)))
        return lev

    def fit_levels(self, grads: Optional[Sequence], round_: int, stream=None):
        """grads: K*L device tensors/addresses, entry k*L+l; None (bucket scope): fit from the statistics gathered by
        the last quantize pass."""
        assert grads is None or len(grads) == self.K * self.L
        self._check(self._lib.qoda_fit_levels(self._h, None if grads is None else _ptrs(grads), round_, _stream(stream)))

    def fit_levels_keep_norms(self, grads: Sequence, round_: int, stream=None):
        """fit_levels on the round's own vectors: declares that the quantize calls of ``round_`` get the same buffers
        unchanged, so that they reuse the norms computed here."""
        assert len(grads) == self.K * self.L
        self._check(self._lib.qoda_fit_levels_keep_norms(self._h, _ptrs(grads), round_, _stream(stream)))

    def gather_statistics(self, enable: bool):
        """Bucket scope: whether quantize passes gather the histogram for the next statistics-based fit."""
        self._check(self._lib.qoda_gather_statistics(self._h, 1 if enable else 0))

    # -- hot path
    def quantize(self, node: int, grads: Sequence, round_: int, msg, msg_prev=None, stream=None):
        assert len(grads) == self.L
        self._check(self._lib.qoda_quantize(self._h, node, _ptrs(grads), round_, _addr(msg), _addr(msg_prev),
                                            _stream(stream)))

    def quantize_noalloc(self, node: int, grads: Sequence, round_: int, msg, msg_prev=None, stream=None):
        """quantize() for callers that cannot allocate: the kernels' scratch is the library's static device array."""
        assert len(grads) == self.L
        self._check(self._lib.qoda_quantize_noalloc(self._h, node, _ptrs(grads), round_, _addr(msg), _addr(msg_prev),
                                                    _stream(stream)))

    def quantize_all(self, grads: Sequence, round_: int, msgs: Sequence, msgs_prev: Optional[Sequence] = None,
                     stream=None):
        assert len(grads) == self.K * self.L and len(msgs) == self.K
        prev = None if msgs_prev is None else _ptrs(msgs_prev)
        self._check(self._lib.qoda_quantize_all(self._h, _ptrs(grads), round_, _ptrs(msgs), prev, _stream(stream)))

    def dequant_aggregate(self, msgs: Sequence, mean_out: Sequence, stream=None):
        assert len(msgs) == self.K and len(mean_out) == self.L
        self._check(self._lib.qoda_dequant_aggregate(self._h, _ptrs(msgs), _ptrs(mean_out), _stream(stream)))

    def step(self, msgs: Sequence, x1: Sequence, y: Sequence, x_half: Sequence, acc, x_next: Optional[Sequence] = None,
             eta=None, stream=None):
        assert len(msgs) == self.K
        st = _State(_ptrs(x1), _ptrs(y), _ptrs(x_half), None if x_next is None else _ptrs(x_next), _addr(acc), _addr(eta))
        self._check(self._lib.qoda_step(self._h, _ptrs(msgs), C.byref(st), _stream(stream)))

    def step_rates(self, msgs: Sequence, x1: Sequence, y: Sequence, x_half: Sequence, rates,
                   x_next: Optional[Sequence] = None, stream=None):
        """The fused step with the caller's two rates (device float[2]: eta_{t+1}, gamma_{t+1})."""
        assert len(msgs) == self.K
        st = _State(_ptrs(x1), _ptrs(y), _ptrs(x_half), None if x_next is None else _ptrs(x_next), None, None)
        self._check(self._lib.qoda_step_rates(self._h, _ptrs(msgs), C.byref(st), _addr(rates), _stream(stream)))

    def step_alt(self, msgs: Sequence, x1: Sequence, y: Sequence, x_half: Sequence, sums, eta, q_hat: float,
                 x_next: Optional[Sequence] = None, stream=None):
        assert len(msgs) == self.K
        st = _AltState(_ptrs(x1), _ptrs(y), _ptrs(x_half), None if x_next is None else _ptrs(x_next), _addr(sums),
                       _addr(eta))
        self._check(self._lib.qoda_step_alt(self._h, _ptrs(msgs), C.byref(st), float(q_hat), _stream(stream)))

    def extrapolate(self, msgs: Sequence, x: Sequence, out: Sequence, gamma, stream=None):
        assert len(msgs) == self.K and len(x) == self.L and len(out) == self.L
        self._check(self._lib.qoda_extrapolate(self._h, _ptrs(msgs), _ptrs(x), _ptrs(out), _addr(gamma), _stream(stream)))

    def index_counts(self, msgs: Sequence, stream=None) -> np.ndarray:
        """Occurrences of every level index per type over the K messages: uint64 [M, 256]."""
        assert len(msgs) == self.K
        out = np.zeros((self.M, 256), dtype=np.uint64)
        self._check(self._lib.qoda_index_counts(self._h, _ptrs(msgs), out.ctypes.data_as(C.POINTER(C.c_uint64)),
                                                _stream(stream)))
        return out

    def code_length(self, counts: np.ndarray, num_messages: Optional[int] = None) -> dict:
        c = np.ascontiguousarray(counts, dtype=np.uint64)
        assert c.shape == (self.M, 256)
        rep = _CodeLength()
        self._check(self._lib.qoda_code_length(self._h, c.ctypes.data_as(C.POINTER(C.c_uint64)),
                                               self.K if num_messages is None else int(num_messages), C.byref(rep)))
        return {n: getattr(rep, n) for n, _ in _CodeLength._fields_}

    # -- diagnostics
    def read_buffer(self, which: int, stream=None) -> np.ndarray:
        KL = self.K * self.L
        shape, dt = {BUF_SUMSQ: ((self.K, self.L), np.float64), BUF_NORM: ((self.K, self.L), np.float32),
                     BUF_INV: ((self.K, self.L), np.float32), BUF_DELTA: ((self.K,), np.float64),
                     BUF_HIST: ((self.K, self.L, HIST_BINS), np.uint32),
                     BUF_POOLED: ((self.M, GRID_POINTS), np.uint64)}[which]
        out = np.zeros(shape, dtype=dt)
        del KL
        self._check(self._lib.qoda_read_buffer(self._h, which, out.ctypes.data, out.nbytes, _stream(stream)))
        return out

    def status(self, stream=None) -> int:
        return int(self._lib.qoda_status(self._h, _stream(stream)))

    # -- measurement aids
    def profile_enable(self, classes=True):
        """classes: True (all kernel classes), False (off), or an iterable of kernel names to time."""
        if classes is True:
            mask = 0xFFFFFFFF
        elif not classes:
            mask = 0
        else:
            names = [kernel_name(i) for i in range(NUM_KERNELS)]
            mask = 0
            for n in classes:
                mask |= 1 << names.index(n)
        self._check(self._lib.qoda_profile_enable(self._h, mask))

    def profile_read(self, stream=None):
        """{kernel name: (total ms, launches)} since the last read."""
        ms = (C.c_double * NUM_KERNELS)()
        n = (C.c_int64 * NUM_KERNELS)()
        self._check(self._lib.qoda_profile_read(self._h, ms, n, _stream(stream)))
        return {kernel_name(i): (float(ms[i]), int(n[i])) for i in range(NUM_KERNELS) if n[i]}

    def copy_calibration(self, src, dst, nbytes: int, stream=None):
        self._check(self._lib.qoda_copy_calibration(self._h, _addr(src), _addr(dst), nbytes, _stream(stream)))

    def stream_calibration(self, src, dst, nbytes: int, stores_per_16_loads: int, stream=None):
        self._check(self._lib.qoda_stream_calibration(self._h, _addr(src), _addr(dst), nbytes, stores_per_16_loads,
                                                      _stream(stream)))


def kernel_name(i: int) -> str:
    return load().qoda_kernel_name(i).decode()
