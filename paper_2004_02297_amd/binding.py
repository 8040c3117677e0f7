"""ctypes binding of libadt.so: argument marshalling only.

Function names and argument order follow include/adt.h.  Device buffers are
torch CUDA(HIP) tensors; the per-layer tables are host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import _build

AWP_NSTATS = 3
ADT_NKERNELS = 10
_lib = None


class _KernelTime(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_int64), ("total_ms", ctypes.c_double),
                ("min_ms", ctypes.c_double), ("max_ms", ctypes.c_double)]


class AdtError(RuntimeError):
    def __init__(self, status: int, text: str, detail: str):
        super().__init__(f"libadt status {status} ({text}): {detail}")
        self.status = status
        self.detail = detail


def lib_path() -> str:
    return _build.LIB


_DIGEST_MARKER = b"adt-source-digest:"


def _built_digest(path: str):
    """Source digest a built library file carries, read from the file's bytes:
    the file is not mapped, because a library that has been mapped once stays
    mapped under its path and a rebuilt file would not replace it.  None: the
    file carries no digest."""
    with open(path, "rb") as f:
        data = f.read()
    at = data.find(_DIGEST_MARKER)
    if at < 0:
        return None
    start = at + len(_DIGEST_MARKER)
    return data[start:data.index(b"\0", start)].decode()


def load_library():
    """Load the in-tree libadt.so.  It is built if no built library exists, and
    built again if the one found was compiled from other sources than the
    tree holds now (the library carries a digest of its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_library()
    want = _build.source_digest()
    if _built_digest(_build.LIB) != want:
        _build.build_library()
        digest = _built_digest(_build.LIB)
        if digest != want:
            raise RuntimeError("libadt.so at %s was built from other sources (digest %r, the "
                               "tree has %r) and rebuilding did not change that"
                               % (_build.LIB, digest, want))
    lib = ctypes.CDLL(_build.LIB)
    lib.adt_source_digest.restype = ctypes.c_char_p
    lib.adt_source_digest.argtypes = []
    if lib.adt_source_digest().decode() != want:
        raise RuntimeError("libadt.so at %s reports digest %r after loading, the tree has %r: another "
                           "build of it is already mapped in this process"
                           % (_build.LIB, lib.adt_source_digest().decode(), want))
    P, I, I64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.adt_packed_size.restype = I64
    lib.adt_packed_size.argtypes = [P, P, I]
    lib.adt_pack.restype = I
    lib.adt_pack.argtypes = [P, P, P, I, P, P]
    lib.adt_unpack.restype = I
    lib.adt_unpack.argtypes = [P, P, P, I, P, P]
    lib.adt_unpack16.restype = I
    lib.adt_unpack16.argtypes = [P, P, P, I, P, I, P]
    lib.adt_pack_unpack.restype = I
    lib.adt_pack_unpack.argtypes = [P, P, P, I, P, P, P]
    lib.awp_layer_stats.restype = I
    lib.awp_layer_stats.argtypes = [P, P, I, P, P]
    lib.awp_layer_stats_noalloc.restype = I
    lib.awp_layer_stats_noalloc.argtypes = [P, P, I, P, P]
    lib.awp_update.restype = I
    lib.awp_update.argtypes = [P, P, P, P, P, I, ctypes.c_double, I, I, I]
    lib.adt_strerror.restype = ctypes.c_char_p
    lib.adt_strerror.argtypes = [I]
    lib.adt_last_error.restype = ctypes.c_char_p
    lib.adt_last_error.argtypes = []
    lib.adt_timing_enable.restype = I
    lib.adt_timing_enable.argtypes = [I, I]
    lib.adt_timing_read.restype = I
    lib.adt_timing_read.argtypes = [P]
    lib.adt_kernel_name.restype = ctypes.c_char_p
    lib.adt_kernel_name.argtypes = [I]
    lib.awp_plan_create.restype = I
    lib.awp_plan_create.argtypes = [P, I, P, ctypes.c_double, I, I, ctypes.POINTER(P)]
    lib.awp_plan_create_grouped.restype = I
    lib.awp_plan_create_grouped.argtypes = [P, I, P, I, P, ctypes.c_double, I, I,
                                            ctypes.POINTER(P)]
    lib.awp_group_norms.restype = I
    lib.awp_group_norms.argtypes = [P, P, I, P]
    lib.awp_expand_group_bytes.restype = I
    lib.awp_expand_group_bytes.argtypes = [P, P, I, P]
    lib.awp_adt_step.restype = I
    lib.awp_adt_step.argtypes = [P, P, P, I64, P, P]
    lib.awp_adt_step16.restype = I
    lib.awp_adt_step16.argtypes = [P, P, P, I64, P, I, P]
    lib.awp_plan_read.restype = I
    lib.awp_plan_read.argtypes = [P, P, P, P, P, P]
    lib.awp_plan_flush.restype = I
    lib.awp_plan_flush.argtypes = [P]
    lib.awp_plan_get_state.restype = I
    lib.awp_plan_get_state.argtypes = [P, P, P, P, P]
    lib.awp_plan_set_state.restype = I
    lib.awp_plan_set_state.argtypes = [P, P, P, P, ctypes.c_int32]
    lib.awp_plan_destroy.restype = I
    lib.awp_plan_destroy.argtypes = [P]
    lib.adt_ablation.restype = I
    lib.adt_ablation.argtypes = [I, I, P, P, P, I, P, P]
    lib.adt_launch_shape.restype = I
    lib.adt_launch_shape.argtypes = [I, I, I]
    lib.adt_stream_cache_limit.restype = I64
    lib.adt_stream_cache_limit.argtypes = [I, I64]
    lib.adt_shutdown.restype = I
    lib.adt_shutdown.argtypes = []
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status < 0:
        lib = load_library()
        raise AdtError(status, lib.adt_strerror(status).decode(),
                       lib.adt_last_error().decode())


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _hptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dev_tensor(t, dtype, name):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} tensor")
    return t


def adt_packed_size(layer_offsets, bytes_per_layer) -> int:
    off = _host(layer_offsets, np.int64)
    rb = _host(bytes_per_layer, np.uint8)
    n = load_library().adt_packed_size(_hptr(off), _hptr(rb), off.size - 1)
    _check(n)
    return int(n)


def adt_pack(weights, layer_offsets, bytes_per_layer, out=None, stream=None):
    """adt_pack: device float32[N] -> device uint8[packed size]."""
    import torch
    off = _host(layer_offsets, np.int64)
    rb = _host(bytes_per_layer, np.uint8)
    L = off.size - 1
    if rb.size != L:
        raise ValueError("bytes_per_layer must have n_layers entries")
    w = _dev_tensor(weights, torch.float32, "weights")
    size = adt_packed_size(off, rb)
    if w.numel() != int(off[-1]):
        raise ValueError("weights size does not match layer_offsets[-1]")
    if out is None:
        out = torch.empty(size, dtype=torch.uint8, device=w.device)
    else:
        _dev_tensor(out, torch.uint8, "out")
        if out.numel() < size:
            raise ValueError("out is smaller than the packed size")
    _check(load_library().adt_pack(w.data_ptr() or None, _hptr(off), _hptr(rb), L,
                                   out.data_ptr() or None, _stream(stream)))
    return out


def adt_unpack(packed, layer_offsets, bytes_per_layer, out=None, stream=None):
    """adt_unpack: device uint8 stream -> device float32[N]."""
    import torch
    off = _host(layer_offsets, np.int64)
    rb = _host(bytes_per_layer, np.uint8)
    L = off.size - 1
    if rb.size != L:
        raise ValueError("bytes_per_layer must have n_layers entries")
    p = _dev_tensor(packed, torch.uint8, "packed")
    if p.numel() < adt_packed_size(off, rb):
        raise ValueError("packed is smaller than the packed size")
    n = int(off[-1])
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=p.device)
    else:
        _dev_tensor(out, torch.float32, "out")
        if out.numel() != n:
            raise ValueError("out size does not match layer_offsets[-1]")
    _check(load_library().adt_unpack(p.data_ptr() or None, _hptr(off), _hptr(rb), L,
                                     out.data_ptr() or None, _stream(stream)))
    return out


def adt_unpack16(packed, layer_offsets, bytes_per_layer, fmt: str, out=None, stream=None):
    """adt_unpack16: device uint8 stream -> device bfloat16 / float16 [N]."""
    import torch
    dtype, code = {"bf16": (torch.bfloat16, 1), "fp16": (torch.float16, 2)}[fmt]
    off = _host(layer_offsets, np.int64)
    rb = _host(bytes_per_layer, np.uint8)
    L = off.size - 1
    if rb.size != L:
        raise ValueError("bytes_per_layer must have n_layers entries")
    p = _dev_tensor(packed, torch.uint8, "packed")
    if p.numel() < adt_packed_size(off, rb):
        raise ValueError("packed is smaller than the packed size")
    n = int(off[-1])
    if out is None:
        out = torch.empty(n, dtype=dtype, device=p.device)
    elif _dev_tensor(out, dtype, "out").numel() != n:
        raise ValueError("out size does not match layer_offsets[-1]")
    _check(load_library().adt_unpack16(p.data_ptr() or None, _hptr(off), _hptr(rb), L,
                                       out.data_ptr() or None, code, _stream(stream)))
    return out


def adt_pack_unpack(weights, layer_offsets, bytes_per_layer, out=None, weights_out=None,
                    stream=None):
    """adt_pack_unpack: one kernel; returns (packed stream, truncated FP32 weights)."""
    import torch
    off = _host(layer_offsets, np.int64)
    rb = _host(bytes_per_layer, np.uint8)
    L = off.size - 1
    if rb.size != L:
        raise ValueError("bytes_per_layer must have n_layers entries")
    w = _dev_tensor(weights, torch.float32, "weights")
    size = adt_packed_size(off, rb)
    if w.numel() != int(off[-1]):
        raise ValueError("weights size does not match layer_offsets[-1]")
    if out is None:
        out = torch.empty(size, dtype=torch.uint8, device=w.device)
    elif _dev_tensor(out, torch.uint8, "out").numel() < size:
        raise ValueError("out is smaller than the packed size")
    if weights_out is None:
        weights_out = torch.empty_like(w)
    elif _dev_tensor(weights_out, torch.float32, "weights_out").numel() != w.numel():
        raise ValueError("weights_out size does not match")
    _check(load_library().adt_pack_unpack(w.data_ptr() or None, _hptr(off), _hptr(rb), L,
                                          out.data_ptr() or None,
                                          weights_out.data_ptr() or None, _stream(stream)))
    return out, weights_out


def awp_layer_stats(weights, layer_offsets, out=None, stream=None):
    """awp_layer_stats: device float32[N] -> device float64[L, 3]."""
    import torch
    off = _host(layer_offsets, np.int64)
    L = off.size - 1
    w = _dev_tensor(weights, torch.float32, "weights")
    if w.numel() != int(off[-1]):
        raise ValueError("weights size does not match layer_offsets[-1]")
    if out is None:
        out = torch.empty((L, AWP_NSTATS), dtype=torch.float64, device=w.device)
    else:
        _dev_tensor(out, torch.float64, "out")
        if out.numel() != L * AWP_NSTATS:
            raise ValueError("out must hold n_layers * 3 doubles")
    _check(load_library().awp_layer_stats(w.data_ptr() or None, _hptr(off), L,
                                          out.data_ptr() or None, _stream(stream)))
    return out


def awp_layer_stats_noalloc(weights, layer_offsets, out, stream=None):
    """awp_layer_stats_noalloc: as awp_layer_stats, scratch in the library's fixed
    device array; `out` (device float64[L, 3]) must be passed in, nothing is allocated."""
    import torch
    off = _host(layer_offsets, np.int64)
    L = off.size - 1
    w = _dev_tensor(weights, torch.float32, "weights")
    if w.numel() != int(off[-1]):
        raise ValueError("weights size does not match layer_offsets[-1]")
    _dev_tensor(out, torch.float64, "out")
    if out.numel() != L * AWP_NSTATS:
        raise ValueError("out must hold n_layers * 3 doubles")
    _check(load_library().awp_layer_stats_noalloc(w.data_ptr() or None, _hptr(off), L,
                                                  out.data_ptr() or None, _stream(stream)))
    return out


class AwpState:
    """Host arrays the AWP rule carries from batch to batch."""

    def __init__(self, n_layers: int, init_bits: int = 8):
        self.n_layers = n_layers
        self.bits = np.full(n_layers, init_bits, dtype=np.int32)
        self.counter = np.zeros(n_layers, dtype=np.int32)
        self.l2_prev = np.zeros(n_layers, dtype=np.float64)
        self.bytes = np.zeros(n_layers, dtype=np.uint8)
        self.first = True


def awp_update(state: AwpState, l2_now, T: float, interval: int, n_bits: int = 8):
    """awp_update: one batch of the rule on host arrays; returns bytes per layer."""
    l2 = _host(l2_now, np.float64)
    if l2.shape != (state.n_layers,):
        raise ValueError("l2_now must have n_layers entries")
    _check(load_library().awp_update(_hptr(l2), _hptr(state.l2_prev), _hptr(state.counter),
                                     _hptr(state.bits), _hptr(state.bytes), state.n_layers,
                                     float(T), int(interval), int(n_bits),
                                     1 if state.first else 0))
    state.first = False
    return state.bytes.copy()


def adt_timing_enable(on: bool, reserve_launches: int = 0) -> None:
    """adt_timing_enable: exact per-launch kernel durations on / off."""
    _check(load_library().adt_timing_enable(1 if on else 0, int(reserve_launches)))


def adt_launch_shape(kernel: str, waves: int, extra_lds_bytes: int = 0) -> None:
    """adt_launch_shape: waves per block and unused dynamic LDS of "pack_kernel",
    "pack_unpack_kernel" or "fused_kernel"; waves = 0 returns to the default."""
    _check(load_library().adt_launch_shape(_kernel_index(kernel), int(waves), int(extra_lds_bytes)))


def _kernel_index(kernel: str) -> int:
    lib = load_library()
    return [lib.adt_kernel_name(k).decode() for k in range(ADT_NKERNELS)].index(kernel)


def adt_stream_cache_limit(kernel: str, nbytes: int = -1) -> int:
    """adt_stream_cache_limit: set (nbytes >= 0) or read the size limit below which
    "pack_kernel", or "pack_unpack_kernel" / "fused_kernel", write the packed stream with
    cache-friendly stores; returns the previous value."""
    n = int(load_library().adt_stream_cache_limit(_kernel_index(kernel), int(nbytes)))
    _check(n)
    return n


def adt_timing_read() -> dict:
    """adt_timing_read: {kernel name: {launches, total_ms, min_ms, max_ms}}."""
    lib = load_library()
    arr = (_KernelTime * ADT_NKERNELS)()
    _check(lib.adt_timing_read(ctypes.cast(arr, ctypes.c_void_p)))
    return {lib.adt_kernel_name(k).decode(): {
        "launches": int(arr[k].launches), "total_ms": arr[k].total_ms,
        "min_ms": arr[k].min_ms, "max_ms": arr[k].max_ms} for k in range(ADT_NKERNELS)}


class AwpPlan:
    """awp_plan_*: device-resident AWP state; step() is one asynchronous pass
    statistics -> rule -> pack -> unpack (see include/adt.h)."""

    def __init__(self, layer_offsets, T: float, interval: int, n_bits: int = 8,
                 init_bits=None, group_offsets=None):
        self._h = None
        self._lib = load_library()
        off = _host(layer_offsets, np.int64)
        self.n_layers = off.size - 1
        self.n_weights = int(off[-1])
        grp = None if group_offsets is None else _host(group_offsets, np.int32)
        self.n_groups = self.n_layers if grp is None else grp.size - 1
        ib = None if init_bits is None else _host(init_bits, np.int32)
        if ib is not None and ib.shape != (self.n_groups,):
            raise ValueError("init_bits must have one entry per group")
        h = ctypes.c_void_p()
        _check(self._lib.awp_plan_create_grouped(_hptr(off), self.n_layers, _hptr(grp),
                                                 self.n_groups, _hptr(ib), float(T),
                                                 int(interval), int(n_bits), ctypes.byref(h)))
        self._h = h

    def step(self, weights, packed, weights_out=None, stream=None) -> None:
        """awp_adt_step; `packed` must hold at least 4 bytes per weight."""
        import torch
        w = _dev_tensor(weights, torch.float32, "weights")
        p = _dev_tensor(packed, torch.uint8, "packed")
        if w.numel() != self.n_weights:
            raise ValueError("weights size does not match the plan")
        o = None
        if weights_out is not None:
            if not isinstance(weights_out, torch.Tensor) or \
                    weights_out.dtype not in (torch.float32, torch.bfloat16, torch.float16):
                raise TypeError("weights_out must be a float32, bfloat16 or float16 tensor")
            o = _dev_tensor(weights_out, weights_out.dtype, "weights_out")
            if o.numel() != self.n_weights:
                raise ValueError("weights_out size does not match the plan")
        optr = None if o is None else (o.data_ptr() or None)
        if o is not None and o.dtype != torch.float32:
            # awp_adt_step16: truncated weights in a 16-bit format
            code = 1 if o.dtype == torch.bfloat16 else 2
            _check(self._lib.awp_adt_step16(self._h, w.data_ptr() or None, p.data_ptr() or None,
                                            p.numel(), optr, code, _stream(stream)))
        else:
            _check(self._lib.awp_adt_step(self._h, w.data_ptr() or None, p.data_ptr() or None,
                                          p.numel(), optr, _stream(stream)))

    def flush(self) -> None:
        """awp_plan_flush: enqueue what the last step left to the next one (no wait)."""
        _check(self._lib.awp_plan_flush(self._h))

    def read(self) -> dict:
        """awp_plan_read: waits for the enqueued steps, returns the state."""
        L, G = self.n_layers, self.n_groups
        st = np.empty((L, AWP_NSTATS), np.float64)
        bits, cnt = np.empty(G, np.int32), np.empty(G, np.int32)
        rb, size = np.empty(L, np.uint8), np.zeros(1, np.int64)
        _check(self._lib.awp_plan_read(self._h, _hptr(st), _hptr(bits), _hptr(cnt), _hptr(rb),
                                       _hptr(size)))
        return {"stats": st, "bits": bits, "counter": cnt, "bytes": rb,
                "packed_size": int(size[0])}

    def get_state(self) -> dict:
        """awp_plan_get_state: what a checkpoint has to keep."""
        G = self.n_groups
        bits, cnt = np.empty(G, np.int32), np.empty(G, np.int32)
        prev, seen = np.empty(G, np.float64), np.zeros(1, np.int32)
        _check(self._lib.awp_plan_get_state(self._h, _hptr(bits), _hptr(cnt), _hptr(prev),
                                            _hptr(seen)))
        return {"bits": bits, "counter": cnt, "l2_prev": prev, "batches_seen": int(seen[0])}

    def set_state(self, state: dict) -> None:
        """awp_plan_set_state: resume from get_state()'s result."""
        bits = _host(state["bits"], np.int32)
        cnt = _host(state["counter"], np.int32)
        prev = _host(state["l2_prev"], np.float64)
        if not (bits.shape == cnt.shape == prev.shape == (self.n_groups,)):
            raise ValueError("state arrays must have one entry per group")
        _check(self._lib.awp_plan_set_state(self._h, _hptr(bits), _hptr(cnt), _hptr(prev),
                                            int(state["batches_seen"])))

    def close(self) -> None:
        if self._h is not None:
            self._lib.awp_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


ABLATION_NAIVE, ABLATION_VEC_DIRECT, ABLATION_PER_LAYER = 1, 2, 3


def adt_ablation(variant: int, unpack: bool, weights, layer_offsets, bytes_per_layer, packed,
                 stream=None) -> None:
    """adt_ablation: measurement variants of pack (weights -> packed) or, with
    unpack=True, of unpack (packed -> weights)."""
    import torch
    off = _host(layer_offsets, np.int64)
    rb = _host(bytes_per_layer, np.uint8)
    w = _dev_tensor(weights, torch.float32, "weights")
    p = _dev_tensor(packed, torch.uint8, "packed")
    if w.numel() != int(off[-1]) or p.numel() < adt_packed_size(off, rb):
        raise ValueError("buffer sizes do not match the tables")
    _check(load_library().adt_ablation(int(variant), 1 if unpack else 0, w.data_ptr() or None,
                                       _hptr(off), _hptr(rb), off.size - 1,
                                       p.data_ptr() or None, _stream(stream)))


def awp_group_norms(stats, group_offsets) -> np.ndarray:
    """awp_group_norms: per-group l2-norms from per-layer statistics (host)."""
    st = _host(stats, np.float64)
    grp = _host(group_offsets, np.int32)
    out = np.empty(grp.size - 1, np.float64)
    _check(load_library().awp_group_norms(_hptr(st), _hptr(grp), grp.size - 1, _hptr(out)))
    return out


def awp_expand_group_bytes(bytes_group, group_offsets) -> np.ndarray:
    """awp_expand_group_bytes: per-layer byte counts from per-group ones (host)."""
    bg = _host(bytes_group, np.uint8)
    grp = _host(group_offsets, np.int32)
    out = np.empty(int(grp[-1]), np.uint8)
    _check(load_library().awp_expand_group_bytes(_hptr(bg), _hptr(grp), grp.size - 1, _hptr(out)))
    return out
