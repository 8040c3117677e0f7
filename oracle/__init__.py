"""CPU oracle (test infrastructure only) for ADT pack/unpack, AWP statistics and
the AWP rule of arXiv 2004.02297.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may use
this package.  It is a ctypes front end to ``adt_oracle.c`` (plain scalar C,
single thread); it imports nothing from the GPU package and the GPU package
imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adt_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

NSTATS = 3  # sumsq, l2, absmax


def build(force: bool = False) -> str:
    """Compile adt_oracle.c with gcc into liboracle.so (next to the source)."""
    if force or (not os.path.exists(_LIB)
                 or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra",
                               "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load(path=None):
    """Load liboracle.so (or, for tests that plant mistakes in a copy of the
    source, another build of it) and declare the C signatures."""
    global _lib
    if _lib is None or path is not None:
        if path is None:
            build()
        lib = ctypes.CDLL(path or _LIB)
        P = ctypes.c_void_p
        lib.oracle_pack.restype = ctypes.c_int64
        lib.oracle_pack.argtypes = [P, P, P, ctypes.c_int, P]
        lib.oracle_unpack.restype = ctypes.c_int64
        lib.oracle_unpack.argtypes = [P, P, P, ctypes.c_int, P]
        lib.oracle_stats.restype = None
        lib.oracle_stats.argtypes = [P, P, ctypes.c_int, P]
        lib.oracle_group_norms.restype = None
        lib.oracle_group_norms.argtypes = [P, P, P, ctypes.c_int, P]
        lib.oracle_awp_update.restype = None
        lib.oracle_awp_update.argtypes = [P, P, P, P, P, ctypes.c_int,
                                          ctypes.c_double, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_int]
        if path is not None:
            return lib
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _tables(layer_offsets, bytes_per_layer=None):
    off = np.ascontiguousarray(layer_offsets, dtype=np.int64)
    if off.ndim != 1 or off.size < 1:
        raise ValueError("layer_offsets must have n_layers+1 entries")
    L = off.size - 1
    if off[0] != 0 or np.any(np.diff(off) < 0):
        raise ValueError("layer_offsets must start at 0 and be non-decreasing")
    if bytes_per_layer is None:
        return off, None, L
    rb = np.ascontiguousarray(bytes_per_layer, dtype=np.uint8)
    if rb.shape != (L,):
        raise ValueError("bytes_per_layer must have n_layers entries")
    if L and (rb.min() < 1 or rb.max() > 4):
        raise ValueError("bytes_per_layer entries must be in 1..4")
    return off, rb, L


def packed_size(layer_offsets, bytes_per_layer) -> int:
    off, rb, _ = _tables(layer_offsets, bytes_per_layer)
    return int(np.sum(np.diff(off) * rb.astype(np.int64)))


def pack(weights: np.ndarray, layer_offsets, bytes_per_layer) -> np.ndarray:
    off, rb, L = _tables(layer_offsets, bytes_per_layer)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    if w.size != off[-1]:
        raise ValueError("weights size does not match layer_offsets[-1]")
    out = np.empty(packed_size(off, rb), dtype=np.uint8)
    n = _load().oracle_pack(_ptr(w), _ptr(off), _ptr(rb), L, _ptr(out))
    assert n == out.size
    return out


def unpack(packed: np.ndarray, layer_offsets, bytes_per_layer) -> np.ndarray:
    off, rb, L = _tables(layer_offsets, bytes_per_layer)
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    if p.size != packed_size(off, rb):
        raise ValueError("packed size does not match the tables")
    out = np.empty(int(off[-1]), dtype=np.float32)
    n = _load().oracle_unpack(_ptr(p), _ptr(off), _ptr(rb), L, _ptr(out))
    assert n == p.size
    return out


def unpack16(packed: np.ndarray, layer_offsets, bytes_per_layer, fmt: str) -> np.ndarray:
    """Bitunpack followed by a conversion to a 16-bit format, as uint16 bit
    patterns: "bf16" keeps the top 16 bits of each unpacked word, "fp16" is the
    IEEE binary16 value nearest to it (ties to even; numpy's conversion).  A NaN
    has no nearest value: it becomes the quiet NaN 0x7E00 with the word's sign
    (the paper proposes half-precision decompression without going into such
    detail; this is the library header's rule)."""
    w = unpack(packed, layer_offsets, bytes_per_layer)
    if fmt == "bf16":
        return (w.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    if fmt == "fp16":
        with np.errstate(over="ignore", invalid="ignore"):
            half = w.astype(np.float16).view(np.uint16).copy()
        words = w.view(np.uint32)
        is_nan = (words & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        sign = ((words >> np.uint32(16)) & np.uint32(0x8000)).astype(np.uint16)
        half[is_nan] = sign[is_nan] | np.uint16(0x7E00)
        return half
    raise ValueError("fmt must be 'bf16' or 'fp16'")


def stats(weights: np.ndarray, layer_offsets) -> np.ndarray:
    """float64[L, 3]: sum of squares, l2-norm, largest magnitude per layer."""
    off, _, L = _tables(layer_offsets)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    if w.size != off[-1]:
        raise ValueError("weights size does not match layer_offsets[-1]")
    out = np.empty((L, NSTATS), dtype=np.float64)
    _load().oracle_stats(_ptr(w), _ptr(off), L, _ptr(out))
    return out


def group_norms(weights: np.ndarray, layer_offsets, group_offsets) -> np.ndarray:
    """float64[G]: l2-norm over all weights of each run of layers."""
    off, _, L = _tables(layer_offsets)
    grp = np.ascontiguousarray(group_offsets, dtype=np.int32)
    if grp[0] != 0 or grp[-1] != L or np.any(np.diff(grp) < 0):
        raise ValueError("group_offsets must run from 0 to n_layers without decreasing")
    w = np.ascontiguousarray(weights, dtype=np.float32)
    out = np.empty(grp.size - 1, dtype=np.float64)
    _load().oracle_group_norms(_ptr(w), _ptr(off), _ptr(grp), grp.size - 1, _ptr(out))
    return out


class AwpState:
    """Per-layer AWP state: bit counts, interval counters, previous norms."""

    def __init__(self, n_layers: int, init_bits: int = 8):
        self.n_layers = n_layers
        self.bits = np.full(n_layers, init_bits, dtype=np.int32)
        self.counter = np.zeros(n_layers, dtype=np.int32)
        self.l2_prev = np.zeros(n_layers, dtype=np.float64)
        self.bytes = np.zeros(n_layers, dtype=np.uint8)
        self.first = True


def awp_update(state: AwpState, l2_now, T: float, interval: int,
               n_bits: int = 8) -> np.ndarray:
    """One batch of the AWP rule; returns the per-layer byte counts."""
    l2 = np.ascontiguousarray(l2_now, dtype=np.float64)
    assert l2.shape == (state.n_layers,)
    _load().oracle_awp_update(_ptr(l2), _ptr(state.l2_prev), _ptr(state.counter),
                              _ptr(state.bits), _ptr(state.bytes),
                              state.n_layers, float(T), int(interval),
                              int(n_bits), 1 if state.first else 0)
    state.first = False
    return state.bytes.copy()
