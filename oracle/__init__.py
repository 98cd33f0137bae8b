"""CPU oracle for the sketch-query + linear path (TEST INFRASTRUCTURE ONLY).

Thin numpy wrappers over ``sketch_oracle.c`` (plain C, built with gcc) plus
the importance-aware width allocation of Sec. 3.2.  Nothing in the GPU
library imports this package and this package imports nothing of the GPU
library.  Callers: tests/, the smoke check, and the benchmark's CPU leg
(offline sketch generator + cpu_baseline timing).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sketch_oracle.c")
# SKETCH_ORACLE_LIB: an already built library to load instead (the sanitizer run of the test suite uses it)
_LIB = os.environ.get("SKETCH_ORACLE_LIB") or os.path.join(_HERE, "libsketch_oracle.so")

_u32p = ctypes.POINTER(ctypes.c_uint32)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2, no intrinsics, no OpenMP)."""
    if os.environ.get("SKETCH_ORACLE_LIB"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _bind(L):
    """Declare the C signatures on a loaded oracle library."""
    L.ora_half_to_double.restype = ctypes.c_double
    L.ora_half_to_double.argtypes = [ctypes.c_uint16]
    L.ora_bf16_to_double.restype = ctypes.c_double
    L.ora_bf16_to_double.argtypes = [ctypes.c_uint16]
    L.ora_select.restype = ctypes.c_uint32
    L.ora_select.argtypes = [ctypes.c_uint32] * 4
    L.ora_count_states.restype = ctypes.c_uint64
    L.ora_count_states.argtypes = [ctypes.c_uint32] * 5 + [_u32p]
    geom = [ctypes.c_uint32] * 5 + [_u32p, _u32p, _u32p]
    L.ora_update.restype = ctypes.c_int
    L.ora_update.argtypes = geom + [_u16p, _u16p, ctypes.c_uint64]
    L.ora_query.restype = ctypes.c_int
    L.ora_query.argtypes = geom + [_u16p, ctypes.c_uint64, _u16p]
    L.ora_query_mode.restype = ctypes.c_int
    L.ora_query_mode.argtypes = geom + [_u16p, ctypes.c_uint64, ctypes.c_int, _u16p]
    _i8p = ctypes.POINTER(ctypes.c_int8)
    qgeom = [ctypes.c_uint32] * 5 + [_u32p]
    L.ora_quantize_states.restype = ctypes.c_int
    L.ora_quantize_states.argtypes = qgeom + [_u16p, ctypes.c_uint64, ctypes.c_int, _i8p, _u16p]
    L.ora_dequantize_states.restype = ctypes.c_int
    L.ora_dequantize_states.argtypes = qgeom + [ctypes.c_int, _i8p, _u16p, _u16p, ctypes.c_uint64]
    L.ora_linear.restype = ctypes.c_int
    L.ora_linear.argtypes = [ctypes.c_uint32, ctypes.c_uint32, _u16p, _u16p, ctypes.c_int,
                             ctypes.c_uint32, ctypes.c_uint64, _u32p, ctypes.c_uint32, _f64p]
    return L


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(ctypes.CDLL(_LIB))
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(ty)


def _u32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint32))


def _u16(a):
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    return np.ascontiguousarray(a, dtype=np.uint16)


@dataclass
class Sketch:
    """A sketched linear layer: geometry, hash parameters, widths, states.

    ``states`` holds binary16 bit patterns, group-major, then sketch row,
    then index inside the row (Sec. 3.1 sketch state S, one per group)."""
    in_features: int
    out_features: int
    tile_in: int
    tile_out: int
    d: int
    hash_a: np.ndarray
    hash_c: np.ndarray
    group_width: np.ndarray
    states: np.ndarray

    @property
    def n_groups(self):
        return (self.in_features // self.tile_in) * (self.out_features // self.tile_out)

    @property
    def bits_per_weight(self):
        return 16.0 * self.states.size / (self.in_features * self.out_features)


@dataclass
class QuantSketch(Sketch):
    """A sketch whose states are kept as low-bit codes (Sec. 3.3, last paragraph): ``codes`` holds one
    signed integer per state (int8, also for 4 bit), ``scales`` one binary16 pattern per (group, sketch
    row); ``states`` are the binary16 states the codes stand for, so query and linear apply unchanged."""
    bits: int = 8
    codes: np.ndarray = None
    scales: np.ndarray = None

    @property
    def bits_per_weight(self):
        return (self.bits * self.codes.size + 16.0 * self.scales.size) / (self.in_features * self.out_features)


def half_to_double(bits) -> np.ndarray:
    L = _load()
    b = np.asarray(bits, dtype=np.uint16).ravel()
    return np.array([L.ora_half_to_double(int(v)) for v in b]).reshape(np.shape(bits))


def select(A: int, C: int, K: int, a: int) -> int:
    """Eq. (3): row-local state index of the weight at group offset ``a``."""
    return int(_load().ora_select(A, C, K, a))


def count_states(in_f, out_f, tj, to, d, width) -> int:
    w = _u32(width)
    return int(_load().ora_count_states(in_f, out_f, tj, to, d, _p(w, _u32p)))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed: code {rc} "
                         f"({ {1: 'bad argument', 2: 'non-finite value'}.get(rc, '?')})")


def update(W, tile_in, tile_out, d, hash_a, hash_c, group_width) -> Sketch:
    """Eq. (4): build the sketch states of W ([in][out] binary16)."""
    Wb = _u16(W)
    in_f, out_f = Wb.shape
    A, C, wd = _u32(hash_a), _u32(hash_c), _u32(group_width).ravel()
    assert A.size == d and C.size == d
    n = count_states(in_f, out_f, tile_in, tile_out, d, wd)
    if n == 0:
        raise ValueError("bad geometry")
    states = np.empty(n, dtype=np.uint16)
    rc = _load().ora_update(in_f, out_f, tile_in, tile_out, d, _p(A, _u32p), _p(C, _u32p),
                            _p(wd, _u32p), _p(Wb, _u16p), _p(states, _u16p), n)
    _check(rc, "update")
    return Sketch(in_f, out_f, tile_in, tile_out, d, A, C, wd, states)


QUERY_ABS_MAX, QUERY_SIGNED_MAX = 0, 1


def query(sk: Sketch, mode: int = QUERY_ABS_MAX) -> np.ndarray:
    """Eq. (5): reconstruct W_hat ([in][out] binary16 bit patterns).  mode 0: Max by magnitude (default
    reading); mode 1: Max of the signed values, Eq. (5) as printed."""
    W_hat = np.empty((sk.in_features, sk.out_features), dtype=np.uint16)
    st = _u16(sk.states)
    rc = _load().ora_query_mode(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d,
                                _p(_u32(sk.hash_a), _u32p), _p(_u32(sk.hash_c), _u32p),
                                _p(_u32(sk.group_width), _u32p), _p(st, _u16p), st.size, int(mode),
                                _p(W_hat, _u16p))
    _check(rc, "query")
    return W_hat


def dequantize_states(in_f, out_f, tile_in, tile_out, d, group_width, bits, codes, scales) -> np.ndarray:
    """The binary16 states that low-bit codes stand for: q * scale / qmax, rounded once (nearest even)."""
    wd = _u32(group_width).ravel()
    cd = np.ascontiguousarray(np.asarray(codes, dtype=np.int8))
    sc = _u16(scales).ravel()
    n = count_states(in_f, out_f, tile_in, tile_out, d, wd)
    assert cd.size == n and sc.size == wd.size * d
    states = np.empty(n, dtype=np.uint16)
    rc = _load().ora_dequantize_states(in_f, out_f, tile_in, tile_out, d, _p(wd, _u32p), bits,
                                       _p(cd, ctypes.POINTER(ctypes.c_int8)), _p(sc, _u16p), _p(states, _u16p), n)
    _check(rc, "dequantize_states")
    return states


def quantize(sk: Sketch, bits: int) -> QuantSketch:
    """Low-bit copy of a sketch: per (group, sketch row) scale = largest state magnitude, codes =
    round-half-even(state * qmax / scale), qmax = 127 (8 bit) or 7 (4 bit)."""
    st = _u16(sk.states)
    wd = _u32(sk.group_width).ravel()
    codes = np.empty(st.size, dtype=np.int8)
    scales = np.empty(wd.size * sk.d, dtype=np.uint16)
    rc = _load().ora_quantize_states(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d,
                                     _p(wd, _u32p), _p(st, _u16p), st.size, bits,
                                     _p(codes, ctypes.POINTER(ctypes.c_int8)), _p(scales, _u16p))
    _check(rc, "quantize_states")
    deq = dequantize_states(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d, wd, bits, codes, scales)
    return QuantSketch(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d, sk.hash_a, sk.hash_c,
                       wd, deq, bits, codes, scales)


def linear(W_hat, x, x_kind: str = "f16", cols=None) -> np.ndarray:
    """y = x W_hat in binary64 (Eq. (1)/(2): y = xW, W is d_in x d_out).

    ``x``: [batch][in] bit patterns (uint16) or float16 array; ``x_kind``
    'f16' or 'bf16' says how to read uint16 bit patterns.  ``cols`` limits
    the result to the listed output channels."""
    Wb = _u16(W_hat)
    in_f, out_f = Wb.shape
    xb = _u16(x)
    if xb.ndim == 1:
        xb = xb[None, :]
    batch, ldx = xb.shape
    assert ldx == in_f
    kind = {"f16": 0, "bf16": 1}[x_kind]
    if cols is None:
        y = np.empty((batch, out_f), dtype=np.float64)
        rc = _load().ora_linear(in_f, out_f, _p(Wb, _u16p), _p(xb, _u16p), kind, batch, ldx,
                                None, 0, _p(y, _f64p))
    else:
        cc = _u32(cols)
        y = np.empty((batch, cc.size), dtype=np.float64)
        rc = _load().ora_linear(in_f, out_f, _p(Wb, _u16p), _p(xb, _u16p), kind, batch, ldx,
                                _p(cc, _u32p), cc.size, _p(y, _f64p))
    _check(rc, "linear")
    return y


def allocate_widths(importance, budget_states: int, d: int) -> np.ndarray:
    """Importance-aware space allocation (Sec. 3.2): unit i receives the share
    I_i / sum(I) of the total sketch space.  ``budget_states`` is the total
    number of states of the layer, split evenly over the d sketch rows; the
    per-row width is the floor of the share, at least 1."""
    imp = np.asarray(importance, dtype=np.float64).ravel()
    if imp.size == 0 or np.any(imp < 0) or not np.all(np.isfinite(imp)) or imp.sum() <= 0:
        raise ValueError("importance must be finite, non-negative, not all zero")
    share = imp / imp.sum()
    k = np.floor(share * (budget_states / d)).astype(np.int64)
    k = np.clip(k, 1, 65535)
    return k.astype(np.uint32)


def row_importance(activations) -> np.ndarray:
    """Importance of the input channels of a layer (Sec. 3.2): I_j = E[a_j^2], the mean over the sampled
    activation vectors (rows of ``activations``) of the squared j-th component, in binary64."""
    a = np.asarray(activations, dtype=np.float64)
    if a.ndim != 2 or a.shape[0] == 0:
        raise ValueError("activations must be [samples][channels] with at least one sample")
    return (a * a).sum(axis=0) / a.shape[0]


def layer_importance(row_imp) -> float:
    """Layer-wise importance (Sec. 3.2): the mean of the layer's row-wise values."""
    r = np.asarray(row_imp, dtype=np.float64).ravel()
    if r.size == 0:
        raise ValueError("no rows")
    return float(r.sum() / r.size)


def allocate_layer_budgets(layer_imp, total_states: int, sizes=None) -> np.ndarray:
    """Sketch space per layer (Sec. 3.2): layer l receives the share I_l / sum(I) of the total space,
    rounded down to whole states.  The paper's formula has no size term; its units (the rows of one
    matrix) are all of one size.  For layers of different sizes ``sizes`` (weights per layer) may be
    given: the share is then I_l n_l / sum(I n), i.e. the bits per weight of a layer are proportional
    to its importance; with equal sizes this is the paper's formula."""
    imp = np.asarray(layer_imp, dtype=np.float64).ravel()
    if imp.size == 0 or np.any(imp < 0) or not np.all(np.isfinite(imp)) or imp.sum() <= 0:
        raise ValueError("importance must be finite, non-negative, not all zero")
    w = imp if sizes is None else imp * np.asarray(sizes, dtype=np.float64).ravel()
    if w.shape != imp.shape:
        raise ValueError("one size per layer")
    return np.floor(w / w.sum() * float(total_states)).astype(np.int64)


def gate_up(gate, up) -> np.ndarray:
    """First half of the feed-forward block, Eq. (2): Activation(x W_gate) * (x W_up), element-wise, in
    binary64.  The paper leaves the activation open; the Llama-shaped configurations use SiLU,
    SiLU(a) = a / (1 + exp(-a))."""
    a = np.asarray(gate, dtype=np.float64)
    return a / (1.0 + np.exp(-a)) * np.asarray(up, dtype=np.float64)
