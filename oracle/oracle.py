"""ctypes marshalling for the C++ oracle (argument conversion only; no arithmetic of the method here)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qoda_oracle.cpp")
_LIB = os.path.join(_HERE, "libqoda_oracle.so")
_CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]

HIST_BINS = 2048
GRID_POINTS = 257
GRID_BASE = 760
BLOCK = 256
OCTET = 2048
CHUNK = 16384
BUCKET = 128
TYPE_SKIP = 0x7FFFFFFF   # "no weight scale for this type"
SCOPE_LAYER, SCOPE_VECTOR, SCOPE_BUCKET = 0, 1, 2   # what one norm covers: a layer, the whole vector, 128 coordinates
NORM_LINF, NORM_L1, NORM_L2 = 0, 1, 2                # the q of the L^q normalisation (0 stands for q -> infinity)

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (always when ``force``; otherwise only if stale or missing)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["g++", *_CXXFLAGS, _SRC, "-o", _LIB])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u8p, u32p, u64p, i32p, i64p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint32, C.c_uint64, C.c_int32, C.c_int64))
        fp, dp = C.POINTER(C.c_float), C.POINTER(C.c_double)
        pp = C.POINTER(C.c_void_p)
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_draw16.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
        L.oracle_draw16.restype = C.c_uint32
        L.oracle_sqrt_floor.argtypes = [C.c_double]
        L.oracle_sqrt_floor.restype = C.c_float
        L.oracle_rcp_floor.argtypes = [C.c_float]
        L.oracle_rcp_floor.restype = C.c_float
        L.oracle_level_index.argtypes = [fp, C.c_int32, C.c_float]
        L.oracle_level_index.restype = C.c_int32
        L.oracle_index_bits.argtypes = [C.c_int32]
        L.oracle_index_bits.restype = C.c_int32
        L.oracle_sumsq.argtypes = [fp, C.c_int64]
        L.oracle_sumsq.restype = C.c_double
        L.oracle_quantize_range.argtypes = [fp, C.c_int64, C.c_int64, C.c_float, fp, C.c_int32, C.c_uint64, C.c_uint32,
                                            C.c_uint32, C.c_uint32, u8p, u8p]
        L.oracle_quantize_range.restype = None
        L.oracle_quantize_with_draws.argtypes = [fp, C.c_int64, C.c_float, fp, C.c_int32, u32p, u8p, u8p]
        L.oracle_quantize_with_draws.restype = None
        L.oracle_decode.argtypes = [u8p, u8p, C.c_int64, C.c_float, fp, C.c_int32, fp]
        L.oracle_decode.restype = None
        L.oracle_message_bytes.argtypes = [C.c_int32, i64p, i32p, C.c_int32]
        L.oracle_message_bytes.restype = C.c_int64
        L.oracle_header_bytes.argtypes = [C.c_int32, i64p, i32p, C.c_int32]
        L.oracle_header_bytes.restype = C.c_int64
        L.oracle_layout.argtypes = [C.c_int32, i64p, i32p, C.c_int32, i64p, i64p]
        L.oracle_layout.restype = None
        L.oracle_pack_layer.argtypes = [u8p, u8p, C.c_int64, C.c_int32, C.c_int32, fp, u8p]
        L.oracle_pack_layer.restype = None
        L.oracle_unpack_layer.argtypes = [u8p, C.c_int64, C.c_int32, C.c_int32, u8p, u8p, fp]
        L.oracle_bucket_sumsq.argtypes = [fp, C.c_int64]
        L.oracle_bucket_sumsq.restype = C.c_double
        L.oracle_unpack_layer.restype = None
        L.oracle_quantize.argtypes = [C.c_int32, i64p, i32p, pp, pp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int32, u8p, u8p,
                                      dp, dp, i32p, u64p, dp, C.c_int32]
        L.oracle_quantize.restype = C.c_int32
        L.oracle_delta_from_messages.argtypes = [C.c_int32, i64p, i32p, C.c_int32, u8p, u8p]
        L.oracle_delta_from_messages.restype = C.c_double
        L.oracle_dequant_aggregate.argtypes = [C.c_int32, i64p, i32p, C.c_int32, C.c_int32, pp, pp]
        L.oracle_dequant_aggregate.restype = None
        L.oracle_step_size.argtypes = [C.c_int32, dp, dp, fp]
        L.oracle_step_size.restype = None
        L.oracle_oda_update.argtypes = [C.c_int64, fp, fp, fp, fp, fp, C.c_float, C.c_float]
        L.oracle_oda_update.restype = None
        L.oracle_index_counts.argtypes = [C.c_int32, i64p, i32p, i32p, C.c_int32, u8p, u64p]
        L.oracle_index_counts.restype = None
        L.oracle_huffman_bits.argtypes = [u64p, C.c_int32]
        L.oracle_huffman_bits.restype = C.c_double
        L.oracle_code_length.argtypes = [C.c_int32, i32p, u64p, C.c_double, dp]
        L.oracle_code_length.restype = None
        L.oracle_extrapolate.argtypes = [C.c_int64, fp, fp, C.c_float, fp]
        L.oracle_extrapolate.restype = None
        L.oracle_alt_step_size.argtypes = [C.c_double, C.c_double, C.c_double, fp, fp]
        L.oracle_alt_step_size.restype = None
        L.oracle_alt_advance.argtypes = [C.c_int32, dp, C.c_double, dp, dp]
        L.oracle_alt_advance.restype = None
        L.oracle_oda_update_alt.argtypes = [C.c_int32, i64p, pp, pp, pp, pp, pp, C.c_float, C.c_float, C.c_float]
        L.oracle_oda_update_alt.restype = C.c_double
        L.oracle_histogram.argtypes = [fp, C.c_int64, u32p]
        L.oracle_histogram.restype = None
        L.oracle_fit_objective.argtypes = [u64p, fp, C.c_int32]
        L.oracle_fit_objective.restype = C.c_double
        L.oracle_fit_dp.argtypes = [u64p, C.c_int32, fp]
        L.oracle_fit_dp.restype = None
        L.oracle_fit_levels.argtypes = [C.c_int32, i64p, i32p, C.c_int32, i32p, C.c_int32, C.c_int32, pp, pp, u32p, u64p,
                                        C.c_int32]
        L.oracle_fit_levels.restype = C.c_int32
        L.oracle_fit_from_stats.argtypes = [C.c_int32, i32p, C.c_int32, i32p, C.c_int32, u64p, dp, i32p, pp, u64p, C.c_int32]
        L.oracle_fit_from_stats.restype = C.c_int32
        L.oracle_delta_plain.argtypes = [C.c_int32, i64p, i32p, C.c_int32, u8p, u8p]
        L.oracle_delta_plain.restype = C.c_double
        L.oracle_sumsq_plain.argtypes = [fp, C.c_int64]
        L.oracle_sumsq_plain.restype = C.c_double
        L.oracle_variance_plain.argtypes = [fp, C.c_int64, fp, C.c_int32, C.c_int32]
        L.oracle_variance_plain.restype = C.c_double
        L.oracle_mqv_objective_plain.argtypes = [C.c_int32, i64p, i32p, i32p, C.c_int32, C.c_int32, pp, pp, C.c_int32]
        L.oracle_mqv_objective_plain.restype = C.c_double
        L.oracle_norm_stat.argtypes = [fp, C.c_int64, C.c_int32]
        L.oracle_norm_stat.restype = C.c_double
        L.oracle_bucket_stat.argtypes = [fp, C.c_int64, C.c_int32]
        L.oracle_bucket_stat.restype = C.c_double
        L.oracle_norm_of.argtypes = [C.c_double, C.c_int32]
        L.oracle_norm_of.restype = C.c_float
        L.oracle_weight_of.argtypes = [C.c_double, C.c_int32]
        L.oracle_weight_of.restype = C.c_double
        _lib = L
    return _lib


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    out = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


# ------------------------------------------------------------------ scalars
def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def draw16(seed: int, round_: int, node: int, layer: int, e: int) -> int:
    return int(lib().oracle_draw16(seed, round_, node, layer, e))


def sqrt_floor(s: float) -> np.float32:
    return np.float32(lib().oracle_sqrt_floor(float(s)))


def rcp_floor(x) -> np.float32:
    return np.float32(lib().oracle_rcp_floor(C.c_float(float(x))))


def level_index(levels, u) -> int:
    lev = _f32(levels)
    return int(lib().oracle_level_index(_p(lev, C.c_float), len(lev), C.c_float(float(u))))


def index_bits(S: int) -> int:
    return int(lib().oracle_index_bits(S))


def sumsq(v) -> float:
    v = _f32(v)
    return float(lib().oracle_sumsq(_p(v, C.c_float), v.size))


def norm_stat(v, norm_kind: int = NORM_L2) -> float:
    """The reduced statistic of one layer: sum of squares, sum of magnitudes or largest magnitude."""
    v = _f32(v)
    return float(lib().oracle_norm_stat(_p(v, C.c_float), v.size, norm_kind))


def bucket_stat(v, norm_kind: int = NORM_L2) -> float:
    v = _f32(v)
    assert v.size <= BUCKET
    return float(lib().oracle_bucket_stat(_p(v, C.c_float), v.size, norm_kind))


def norm_of(s: float, norm_kind: int = NORM_L2) -> np.float32:
    """The fp32 norm a statistic yields (0 if the statistic is out of range)."""
    return np.float32(lib().oracle_norm_of(float(s), norm_kind))


def weight_of(s: float, norm_kind: int = NORM_L2) -> float:
    return float(lib().oracle_weight_of(float(s), norm_kind))


def norm_and_inv(v):
    n = sqrt_floor(sumsq(v))
    return n, rcp_floor(n)


# ------------------------------------------------------------------ one layer, unpacked
def quantize_range(v, e0: int, e1: int, inv, levels, seed: int, round_: int, node: int, layer: int):
    v = _f32(v)
    lev = _f32(levels)
    sign = np.zeros(e1 - e0, dtype=np.uint8)
    idx = np.zeros(e1 - e0, dtype=np.uint8)
    lib().oracle_quantize_range(_p(v, C.c_float), e0, e1, C.c_float(float(inv)), _p(lev, C.c_float), len(lev), seed,
                                round_, node, layer, _p(sign, C.c_uint8), _p(idx, C.c_uint8))
    return sign, idx


def quantize_with_draws(v, inv, levels, w16):
    v = _f32(v)
    lev = _f32(levels)
    w = np.ascontiguousarray(w16, dtype=np.uint32)
    sign = np.zeros(v.size, dtype=np.uint8)
    idx = np.zeros(v.size, dtype=np.uint8)
    lib().oracle_quantize_with_draws(_p(v, C.c_float), v.size, C.c_float(float(inv)), _p(lev, C.c_float), len(lev),
                                     _p(w, C.c_uint32), _p(sign, C.c_uint8), _p(idx, C.c_uint8))
    return sign, idx


def decode(sign, idx, norm, levels) -> np.ndarray:
    sign = np.ascontiguousarray(sign, dtype=np.uint8)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    lev = _f32(levels)
    out = np.zeros(sign.size, dtype=np.float32)
    lib().oracle_decode(_p(sign, C.c_uint8), _p(idx, C.c_uint8), sign.size, C.c_float(float(norm)), _p(lev, C.c_float),
                        len(lev), _p(out, C.c_float))
    return out


# ------------------------------------------------------------------ layout
def _dims(sizes, points):
    d = np.ascontiguousarray(sizes, dtype=np.int64)
    S = np.ascontiguousarray(points, dtype=np.int32)
    assert d.size == S.size
    return d, S


def message_bytes(sizes, points, scope: int = SCOPE_LAYER) -> int:
    d, S = _dims(sizes, points)
    return int(lib().oracle_message_bytes(d.size, _p(d, C.c_int64), _p(S, C.c_int32), scope))


def header_bytes(sizes, points, scope: int = SCOPE_LAYER) -> int:
    d, S = _dims(sizes, points)
    return int(lib().oracle_header_bytes(d.size, _p(d, C.c_int64), _p(S, C.c_int32), scope))


def layout(sizes, points, scope: int = SCOPE_LAYER):
    d, S = _dims(sizes, points)
    h = np.zeros(d.size, dtype=np.int64)
    m = np.zeros(d.size, dtype=np.int64)
    lib().oracle_layout(d.size, _p(d, C.c_int64), _p(S, C.c_int32), scope, _p(h, C.c_int64), _p(m, C.c_int64))
    return h, m


def octet_bytes(S: int, scope: int = SCOPE_LAYER) -> int:
    """Bytes of one octet (2048 coordinates) of a layer's body."""
    return 256 * (1 + index_bits(S)) + (64 if scope == SCOPE_BUCKET else 0)


def pack_layer(sign, idx, S: int, scope: int = SCOPE_LAYER, bucket_norms=None) -> np.ndarray:
    sign = np.ascontiguousarray(sign, dtype=np.uint8)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    d = sign.size
    region = np.zeros(((d + OCTET - 1) // OCTET) * octet_bytes(S, scope), dtype=np.uint8)
    bn = None if bucket_norms is None else _f32(bucket_norms)
    lib().oracle_pack_layer(_p(sign, C.c_uint8), _p(idx, C.c_uint8), d, S, scope,
                            None if bn is None else _p(bn, C.c_float), _p(region, C.c_uint8))
    return region


def unpack_layer(region, d: int, S: int, scope: int = SCOPE_LAYER):
    """Returns (sign, index), plus the bucket norms under bucket scope."""
    region = np.ascontiguousarray(region, dtype=np.uint8)
    sign = np.zeros(d, dtype=np.uint8)
    idx = np.zeros(d, dtype=np.uint8)
    bn = np.zeros((d + BUCKET - 1) // BUCKET, dtype=np.float32) if scope == SCOPE_BUCKET else None
    lib().oracle_unpack_layer(_p(region, C.c_uint8), d, S, scope, _p(sign, C.c_uint8), _p(idx, C.c_uint8),
                              None if bn is None else _p(bn, C.c_float))
    return (sign, idx) if bn is None else (sign, idx, bn)


def bucket_sumsq(v) -> float:
    v = _f32(v)
    assert v.size <= BUCKET
    return float(lib().oracle_bucket_sumsq(_p(v, C.c_float), v.size))


# ------------------------------------------------------------------ whole messages
def quantize(sizes, points, levels: Sequence[np.ndarray], grads: Sequence[np.ndarray], seed: int, round_: int,
             node: int, msg_prev: Optional[np.ndarray] = None, scope: int = SCOPE_LAYER, stats_exp=None,
             norm_kind: int = NORM_L2):
    """ENCODE(Q(V_k)) for one node.  Returns (msg bytes, sumsq per layer, delta, status); with ``stats_exp`` (the
    weight scale of every layer's type, bucket scope) also the gathered (grid histograms [L, 257], largest sampled
    bucket sums [L])."""
    d, S = _dims(sizes, points)
    lev = [_f32(a) for a in levels]
    g = [_f32(a) for a in grads]
    for l in range(d.size):
        assert g[l].size == d[l] and lev[l].size == S[l]
    msg = np.zeros(message_bytes(d, S, scope), dtype=np.uint8)
    ss = np.zeros(d.size, dtype=np.float64)
    delta = np.zeros(1, dtype=np.float64)
    prev = None
    if msg_prev is not None:
        prev = np.ascontiguousarray(msg_prev, dtype=np.uint8)
        assert prev.size == msg.size
    if stats_exp is not None:
        sexp = np.ascontiguousarray(stats_exp, dtype=np.int32)
        assert sexp.size == d.size
        shist = np.zeros((d.size, GRID_POINTS), dtype=np.uint64)
        smax = np.zeros(d.size, dtype=np.float64)
    st = lib().oracle_quantize(d.size, _p(d, C.c_int64), _p(S, C.c_int32), _ptr_array(lev), _ptr_array(g), seed, round_,
                               node, scope, _p(msg, C.c_uint8), None if prev is None else _p(prev, C.c_uint8),
                               _p(ss, C.c_double), _p(delta, C.c_double),
                               None if stats_exp is None else _p(sexp, C.c_int32),
                               None if stats_exp is None else _p(shist, C.c_uint64),
                               None if stats_exp is None else _p(smax, C.c_double), norm_kind)
    if stats_exp is None:
        return msg, ss, float(delta[0]), int(st)
    return msg, ss, float(delta[0]), int(st), shist, smax


def delta_from_messages(sizes, points, msg, msg_prev=None, scope: int = SCOPE_LAYER) -> float:
    d, S = _dims(sizes, points)
    m = np.ascontiguousarray(msg, dtype=np.uint8)
    p = None if msg_prev is None else np.ascontiguousarray(msg_prev, dtype=np.uint8)
    return float(lib().oracle_delta_from_messages(d.size, _p(d, C.c_int64), _p(S, C.c_int32), scope, _p(m, C.c_uint8),
                                                  None if p is None else _p(p, C.c_uint8)))


def dequant_aggregate(sizes, points, msgs: Sequence[np.ndarray], scope: int = SCOPE_LAYER) -> List[np.ndarray]:
    d, S = _dims(sizes, points)
    ms = [np.ascontiguousarray(m, dtype=np.uint8) for m in msgs]
    out = [np.zeros(int(n), dtype=np.float32) for n in d]
    lib().oracle_dequant_aggregate(d.size, _p(d, C.c_int64), _p(S, C.c_int32), scope, len(ms), _ptr_array(ms),
                                   _ptr_array(out))
    return out


def step_size(delta: Sequence[float], acc: float):
    """Returns (new acc, eta)."""
    dl = np.ascontiguousarray(delta, dtype=np.float64)
    a = np.array([acc], dtype=np.float64)
    eta = np.zeros(1, dtype=np.float32)
    lib().oracle_step_size(dl.size, _p(dl, C.c_double), _p(a, C.c_double), _p(eta, C.c_float))
    return float(a[0]), np.float32(eta[0])


def oda_update(mean, x1, y, eta, gamma, want_next: bool = True):
    """In place on ``y``.  Returns (x_next or None, x_half)."""
    mean = _f32(mean)
    x1 = _f32(x1)
    assert y.dtype == np.float32 and y.flags.c_contiguous
    xn = np.zeros_like(y) if want_next else None
    xh = np.zeros_like(y)
    lib().oracle_oda_update(y.size, _p(mean, C.c_float), _p(x1, C.c_float), _p(y, C.c_float),
                            None if xn is None else _p(xn, C.c_float), _p(xh, C.c_float), C.c_float(float(eta)),
                            C.c_float(float(gamma)))
    return xn, xh


def index_counts(sizes, points, layer_type, num_types: int, msgs: Sequence[np.ndarray], scope: int = SCOPE_LAYER):
    """Occurrences of every level index per type over the given messages: uint64 [num_types, 256]."""
    d, S = _dims(sizes, points)
    lt = np.ascontiguousarray(layer_type, dtype=np.int32)
    counts = np.zeros((num_types, 256), dtype=np.uint64)
    for m in msgs:
        m = np.ascontiguousarray(m, dtype=np.uint8)
        lib().oracle_index_counts(d.size, _p(d, C.c_int64), _p(S, C.c_int32), _p(lt, C.c_int32), scope, _p(m, C.c_uint8),
                                  _p(counts, C.c_uint64))
    return counts


def huffman_bits(counts) -> float:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    return float(lib().oracle_huffman_bits(_p(c, C.c_uint64), c.size))


def code_length(type_points, counts, num_norms: float) -> dict:
    tp = np.ascontiguousarray(type_points, dtype=np.int32)
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    assert c.shape == (tp.size, 256)
    out = np.zeros(6, dtype=np.float64)
    lib().oracle_code_length(tp.size, _p(tp, C.c_int32), _p(c, C.c_uint64), float(num_norms), _p(out, C.c_double))
    return dict(zip(("fixed_bits", "paper_bits", "entropy_bits", "huffman_bits", "nonzeros", "coordinates"), out.tolist()))


def extrapolate(mean, x, gamma) -> np.ndarray:
    """x - gamma * mean (one leg of an extra-gradient round)."""
    mean, x = _f32(mean), _f32(x)
    out = np.zeros_like(x)
    lib().oracle_extrapolate(x.size, _p(mean, C.c_float), _p(x, C.c_float), C.c_float(float(gamma)), _p(out, C.c_float))
    return out


def alt_step_size(lam: float, mu: float, q_hat: float):
    """eq. (Alt): returns (eta, gamma) from the lagged sums."""
    eta = np.zeros(1, dtype=np.float32)
    gamma = np.zeros(1, dtype=np.float32)
    lib().oracle_alt_step_size(float(lam), float(mu), float(q_hat), _p(eta, C.c_float), _p(gamma, C.c_float))
    return np.float32(eta[0]), np.float32(gamma[0])


def alt_advance(delta: Sequence[float], dx2: float, lam: float, mu: float):
    """Returns the sums (lambda, mu) after a round."""
    dl = np.ascontiguousarray(delta, dtype=np.float64)
    a = np.array([lam], dtype=np.float64)
    b = np.array([mu], dtype=np.float64)
    lib().oracle_alt_advance(dl.size, _p(dl, C.c_double), float(dx2), _p(a, C.c_double), _p(b, C.c_double))
    return float(a[0]), float(b[0])


def oda_update_alt(sizes, mean, x1, y, eta_prev, eta, gamma, want_next: bool = True):
    """All layers, in place on the ``y`` arrays.  Returns (x_next list or None, x_half list, ||X_t - X_{t+1}||^2)."""
    d = np.ascontiguousarray(sizes, dtype=np.int64)
    mean = [_f32(a) for a in mean]
    x1 = [_f32(a) for a in x1]
    for a in y:
        assert a.dtype == np.float32 and a.flags.c_contiguous
    xn = [np.zeros_like(a) for a in y] if want_next else None
    xh = [np.zeros_like(a) for a in y]
    dx2 = lib().oracle_oda_update_alt(d.size, _p(d, C.c_int64), _ptr_array(mean), _ptr_array(x1), _ptr_array(y),
                                      None if xn is None else _ptr_array(xn), _ptr_array(xh),
                                      C.c_float(float(eta_prev)), C.c_float(float(eta)), C.c_float(float(gamma)))
    return xn, xh, float(dx2)


# ------------------------------------------------------------------ level fit
def histogram(v) -> np.ndarray:
    v = _f32(v)
    h = np.zeros(HIST_BINS, dtype=np.uint32)
    lib().oracle_histogram(_p(v, C.c_float), v.size, _p(h, C.c_uint32))
    return h


def fit_objective(W, levels) -> float:
    W = np.ascontiguousarray(W, dtype=np.uint64)
    assert W.size == GRID_POINTS
    lev = _f32(levels)
    return float(lib().oracle_fit_objective(_p(W, C.c_uint64), _p(lev, C.c_float), lev.size))


def fit_dp(W, S: int) -> np.ndarray:
    W = np.ascontiguousarray(W, dtype=np.uint64)
    assert W.size == GRID_POINTS
    lev = np.zeros(S, dtype=np.float32)
    lib().oracle_fit_dp(_p(W, C.c_uint64), S, _p(lev, C.c_float))
    return lev


def fit_levels(sizes, layer_type, type_points, K: int, grads: Sequence[np.ndarray], levels: Sequence[np.ndarray],
               scope: int = SCOPE_LAYER, norm_kind: int = NORM_L2):
    """grads: K*L arrays (entry k*L+l).  levels: M arrays, updated copies returned with (hist, pooled, status)."""
    d = np.ascontiguousarray(sizes, dtype=np.int64)
    lt = np.ascontiguousarray(layer_type, dtype=np.int32)
    tp = np.ascontiguousarray(type_points, dtype=np.int32)
    L, M = d.size, tp.size
    g = [_f32(a) for a in grads]
    assert len(g) == K * L
    lev = [_f32(a).copy() for a in levels]
    hist = np.zeros(K * L * HIST_BINS, dtype=np.uint32)
    pooled = np.zeros(M * GRID_POINTS, dtype=np.uint64)
    st = lib().oracle_fit_levels(L, _p(d, C.c_int64), _p(lt, C.c_int32), M, _p(tp, C.c_int32), K, scope,
                                 _ptr_array(g), _ptr_array(lev), _p(hist, C.c_uint32), _p(pooled, C.c_uint64), norm_kind)
    return lev, hist.reshape(K, L, HIST_BINS), pooled.reshape(M, GRID_POINTS), int(st)


def fit_from_stats(layer_type, type_points, K: int, hist, bmax, exps, levels: Sequence[np.ndarray],
                   norm_kind: int = NORM_L2):
    """hist: [K, L, 257] uint64, bmax: [K, L] float64, exps: [M] int32 (the scales the histograms were gathered with).
    Returns (levels, pooled [M, 257], new exps [M], status)."""
    lt = np.ascontiguousarray(layer_type, dtype=np.int32)
    tp = np.ascontiguousarray(type_points, dtype=np.int32)
    L, M = lt.size, tp.size
    h = np.ascontiguousarray(hist, dtype=np.uint64)
    b = np.ascontiguousarray(bmax, dtype=np.float64)
    assert h.shape == (K, L, GRID_POINTS) and b.shape == (K, L)
    ex = np.ascontiguousarray(exps, dtype=np.int32).copy()
    lev = [_f32(a).copy() for a in levels]
    pooled = np.zeros(M * GRID_POINTS, dtype=np.uint64)
    st = lib().oracle_fit_from_stats(L, _p(lt, C.c_int32), M, _p(tp, C.c_int32), K, _p(h, C.c_uint64), _p(b, C.c_double),
                                     _p(ex, C.c_int32), _ptr_array(lev), _p(pooled, C.c_uint64), norm_kind)
    return lev, pooled.reshape(M, GRID_POINTS), ex, int(st)


# ------------------------------------------------------------------ plain definitions (references, no contract)
def delta_plain(sizes, points, msg, msg_prev=None, scope: int = SCOPE_LAYER) -> float:
    """sum_i (Vhat_i - Vhat_prev_i)^2 of two stored messages in fp64, plain order (eq. (general_stepsize))."""
    d, S = _dims(sizes, points)
    m = np.ascontiguousarray(msg, dtype=np.uint8)
    p = None if msg_prev is None else np.ascontiguousarray(msg_prev, dtype=np.uint8)
    return float(lib().oracle_delta_plain(d.size, _p(d, C.c_int64), _p(S, C.c_int32), scope, _p(m, C.c_uint8),
                                          None if p is None else _p(p, C.c_uint8)))


def sumsq_plain(v) -> float:
    v = _f32(v)
    return float(lib().oracle_sumsq_plain(_p(v, C.c_float), v.size))


def variance_plain(v, levels, norm_kind: int = NORM_L2) -> float:
    """eq. (Var) for one vector and one level sequence, from the definition in fp64."""
    v, lev = _f32(v), _f32(levels)
    return float(lib().oracle_variance_plain(_p(v, C.c_float), v.size, _p(lev, C.c_float), lev.size, norm_kind))


def mqv_objective_plain(sizes, layer_type, type_points, K: int, grads: Sequence[np.ndarray],
                        levels: Sequence[np.ndarray], scope: int = SCOPE_LAYER, norm_kind: int = NORM_L2) -> float:
    """eq. (MQV): total quantization variance of the K nodes' vectors (grads: K*L arrays) under per-type levels."""
    d = np.ascontiguousarray(sizes, dtype=np.int64)
    lt = np.ascontiguousarray(layer_type, dtype=np.int32)
    tp = np.ascontiguousarray(type_points, dtype=np.int32)
    g = [_f32(a) for a in grads]
    lev = [_f32(a) for a in levels]
    assert len(g) == K * d.size and len(lev) == tp.size
    return float(lib().oracle_mqv_objective_plain(d.size, _p(d, C.c_int64), _p(lt, C.c_int32), _p(tp, C.c_int32), K, scope,
                                                  _ptr_array(g), _ptr_array(lev), norm_kind))


def grid_values() -> np.ndarray:
    """The 257 normalised grid points g_j as float32 (bit pattern (j + 760) << 20)."""
    return ((np.arange(GRID_POINTS, dtype=np.uint32) + GRID_BASE) << 20).view(np.float32)


def grid_mids() -> np.ndarray:
    m = (((np.arange(GRID_POINTS, dtype=np.uint32) + GRID_BASE) << 20) | (1 << 19)).view(np.float32).astype(np.float64)
    m[-1] = 1.0
    return m
