"""ctypes binding of librgc.so -- argument marshalling only.

Names follow include/rgc.h (and include/rgc_diag.h for the diagnostics).  Tensors are anything with ``data_ptr()`` / ``numel()``
(PyTorch-ROCm tensors on the GPU); streams are raw ``hipStream_t`` values
(``torch.cuda.current_stream().cuda_stream``), ``None`` = the null stream.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

RGC_OK = 0
RGC_EINVAL = -1
RGC_ENOMEM = -2
RGC_EHIP = -3
RGC_EINTERNAL = -4
RGC_NO_MOMENTUM_MASK = 0x1
RGC_NO_HINTS = 0x2
RGC_NESTEROV = 0x4
RGC_OVERWRITE = 0x10
RGC_ADD_TO_DST = 0x20
RGC_VALIDATE = 0x40
RGC_ONE_VALUE = 0x80
RGC_SELECT_LARGEST = 0x100
RGC_SELECT_SMALLEST = 0x200
RGC_THRESHOLD_SEARCH = 0x400
RGC_STATUS_INDEX_RANGE = 0x1
RGC_STATUS_INDEX_ORDER = 0x2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librgc.so")

EXPORTS = ["rgc_create", "rgc_destroy", "rgc_k_for_density", "rgc_compress_layers",
           "rgc_compress_layers_scaled", "rgc_clip_coefficient", "rgc_message_means", "rgc_message_means_noalloc",
           "rgc_compress_layers_threshold",
           "rgc_decompress_accumulate", "rgc_reset_hints", "rgc_poison_hints", "rgc_limit_optional_scratch", "rgc_selftest",
           "rgc_last_paths", "rgc_last_stats", "rgc_last_error", "rgc_decompress_status", "rgc_profile_enable", "rgc_profile_read", "rgc_stream_yardstick", "rgc_strerror"]


class RgcError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("rgc status %d: %s" % (status, text))
        self.status = status


class rgc_layer(ctypes.Structure):
    _fields_ = [("grad", ctypes.c_void_p), ("residual", ctypes.c_void_p), ("momentum", ctypes.c_void_p),
                ("n", ctypes.c_int64), ("k", ctypes.c_int32), ("out_idx", ctypes.c_void_p),
                ("out_val", ctypes.c_void_p), ("out_count", ctypes.c_void_p)]


class rgc_msg(ctypes.Structure):
    _fields_ = [("idx", ctypes.c_void_p), ("val", ctypes.c_void_p), ("count", ctypes.c_int32)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load librgc.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("librgc.so is not built: run `python -m paper_1808_04357_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    # The tensors handed to the library are PyTorch's, so both must talk to ONE HIP runtime: PyTorch's
    # wheel brings its own libamdhip64.so.7, and whichever copy of that soname is mapped first serves the
    # whole process.  Loaded before torch, librgc.so would bind to the system copy and see no device.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    L.rgc_create.restype = ctypes.c_int
    L.rgc_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int64, ctypes.c_int32]
    L.rgc_destroy.restype = ctypes.c_int
    L.rgc_destroy.argtypes = [ctypes.c_void_p]
    L.rgc_k_for_density.restype = ctypes.c_int32
    L.rgc_k_for_density.argtypes = [ctypes.c_int64, ctypes.c_uint32]
    L.rgc_compress_layers.restype = ctypes.c_int
    L.rgc_compress_layers.argtypes = [ctypes.c_void_p, ctypes.POINTER(rgc_layer), ctypes.c_int32,
                                      ctypes.c_float, ctypes.c_uint32, ctypes.c_void_p]
    L.rgc_compress_layers_scaled.restype = ctypes.c_int
    L.rgc_compress_layers_scaled.argtypes = [ctypes.c_void_p, ctypes.POINTER(rgc_layer), ctypes.c_int32,
                                             ctypes.c_float, ctypes.c_void_p, ctypes.c_uint32, ctypes.c_void_p]
    L.rgc_compress_layers_threshold.restype = ctypes.c_int
    L.rgc_compress_layers_threshold.argtypes = [ctypes.c_void_p, ctypes.POINTER(rgc_layer), ctypes.c_int32,
                                                ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_uint32, ctypes.c_void_p]
    L.rgc_message_means.restype = ctypes.c_int
    L.rgc_message_means.argtypes = [ctypes.c_void_p, ctypes.POINTER(rgc_layer), ctypes.c_int32, ctypes.c_void_p,
                                    ctypes.c_void_p]
    L.rgc_message_means_noalloc.restype = ctypes.c_int
    L.rgc_message_means_noalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                                            ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, ctypes.c_void_p,
                                            ctypes.c_void_p]
    L.rgc_clip_coefficient.restype = ctypes.c_int
    L.rgc_clip_coefficient.argtypes = [ctypes.c_void_p, ctypes.POINTER(rgc_layer), ctypes.c_int32, ctypes.c_float,
                                       ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    L.rgc_decompress_accumulate.restype = ctypes.c_int
    L.rgc_decompress_accumulate.argtypes = [ctypes.c_void_p, ctypes.POINTER(rgc_msg), ctypes.c_int32,
                                            ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p),
                                            ctypes.POINTER(ctypes.c_int64), ctypes.c_float,
                                            ctypes.c_uint32, ctypes.c_void_p]
    L.rgc_reset_hints.restype = ctypes.c_int
    L.rgc_reset_hints.argtypes = [ctypes.c_void_p]
    L.rgc_limit_optional_scratch.restype = ctypes.c_int
    L.rgc_limit_optional_scratch.argtypes = [ctypes.c_void_p, ctypes.c_int64]
    L.rgc_poison_hints.restype = ctypes.c_int
    L.rgc_poison_hints.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    L.rgc_selftest.restype = ctypes.c_int
    L.rgc_selftest.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    L.rgc_last_paths.restype = ctypes.c_int
    L.rgc_last_paths.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, ctypes.c_void_p]
    L.rgc_last_error.restype = ctypes.c_int
    L.rgc_last_error.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    L.rgc_last_stats.restype = ctypes.c_int
    L.rgc_last_stats.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.c_int32, ctypes.c_void_p]
    L.rgc_decompress_status.restype = ctypes.c_int
    L.rgc_decompress_status.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint32), ctypes.c_void_p]
    L.rgc_profile_enable.restype = ctypes.c_int
    L.rgc_profile_enable.argtypes = [ctypes.c_void_p, ctypes.c_int]
    L.rgc_profile_read.restype = ctypes.c_int
    L.rgc_profile_read.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    L.rgc_stream_yardstick.restype = ctypes.c_int
    L.rgc_stream_yardstick.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_float,
                                       ctypes.c_int, ctypes.c_void_p]
    L.rgc_strerror.restype = ctypes.c_char_p
    L.rgc_strerror.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _check(status: int) -> None:
    if status != RGC_OK:
        raise RgcError(status, load_library().rgc_strerror(status).decode())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        return ctypes.c_void_p(0)
    return ctypes.c_void_p(int(getattr(stream, "cuda_stream", stream)))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def rgc_k_for_density(n: int, density_ppm: int = 1000) -> int:
    return int(load_library().rgc_k_for_density(int(n), int(density_ppm)))


class Context:
    """Owns an ``rgc_ctx`` (scratch + speed hints) on one device."""

    def __init__(self, max_total_elems: int, max_layers: int, device_id: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p(0)
        _check(self._lib.rgc_create(ctypes.byref(self._h), int(device_id), int(max_total_elems), int(max_layers)))

    @property
    def handle(self) -> ctypes.c_void_p:
        return self._h

    def close(self) -> None:
        if self._h:
            self._lib.rgc_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset_hints(self) -> None:
        _check(self._lib.rgc_reset_hints(self._h))

    def limit_optional_scratch(self, max_bytes: int) -> None:
        _check(self._lib.rgc_limit_optional_scratch(self._h, int(max_bytes)))

    def poison_hints(self, mode: int, stream=None) -> None:
        _check(self._lib.rgc_poison_hints(self._h, int(mode), _stream(stream)))

    def selftest(self, stream=None) -> None:
        _check(self._lib.rgc_selftest(self._h, _stream(stream)))

    def profile_enable(self, enable: bool) -> None:
        _check(self._lib.rgc_profile_enable(self._h, 1 if enable else 0))

    def profile_read(self):
        """-> (ms[4]: accumulate, phases, decompress table, decompress tiles; calls[2])."""
        ms = (ctypes.c_double * 4)()
        calls = (ctypes.c_int64 * 2)()
        _check(self._lib.rgc_profile_read(self._h, ms, calls))
        return list(ms), list(calls)

    def last_stats(self, num_layers: int, stream=None) -> List[List[int]]:
        """-> per layer [path, candidates, exactly ranked candidates, threshold key, hint misses so far]."""
        out = (ctypes.c_int64 * (5 * num_layers))()
        _check(self._lib.rgc_last_stats(self._h, out, int(num_layers), _stream(stream)))
        return [list(out[5 * l:5 * l + 5]) for l in range(num_layers)]

    def decompress_status(self, stream=None) -> int:
        """OR of the RGC_STATUS_* bits found by the RGC_VALIDATE checks so far (waits for the stream; clears the word)."""
        out = ctypes.c_uint32(0)
        _check(self._lib.rgc_decompress_status(self._h, ctypes.byref(out), _stream(stream)))
        return int(out.value)

    def last_error(self, stream=None) -> None:
        """Raises RgcError(RGC_EINTERNAL) if a kernel has reported an internal inconsistency (waits for the stream)."""
        _check(self._lib.rgc_last_error(self._h, _stream(stream)))

    def last_paths(self, num_layers: int, stream=None) -> List[int]:
        out = (ctypes.c_int32 * num_layers)()
        _check(self._lib.rgc_last_paths(self._h, out, int(num_layers), _stream(stream)))
        return list(out)


class LayerList:
    """A host ``rgc_layer[]`` built once from tensors (keeps them alive)."""

    def __init__(self, grads: Sequence, residuals: Sequence, ks: Sequence[int], out_idx: Sequence,
                 out_val: Sequence, out_count, momenta: Optional[Sequence] = None):
        L = len(grads)
        self.num_layers = L
        self._keep = (grads, residuals, ks, out_idx, out_val, out_count, momenta)
        self.array = (rgc_layer * L)()
        base = int(out_count.data_ptr())
        for l in range(L):
            a = self.array[l]
            a.grad = _ptr(grads[l])
            a.residual = _ptr(residuals[l])
            a.momentum = _ptr(momenta[l]) if momenta is not None else None
            a.n = int(grads[l].numel())
            a.k = int(ks[l])
            a.out_idx = _ptr(out_idx[l])
            a.out_val = _ptr(out_val[l])
            a.out_count = base + 4 * l


class MessageList:
    """Host ``rgc_msg[workers][layers]`` plus the dense pointer / size arrays."""

    def __init__(self, idx: Sequence[Sequence], val: Sequence[Sequence], dense: Sequence):
        N = len(idx)
        L = len(dense)
        self.num_workers, self.num_layers = N, L
        self._keep = (idx, val, dense)
        self.msgs = (rgc_msg * max(N * L, 1))()
        for w in range(N):
            for l in range(L):
                m = self.msgs[w * L + l]
                c = int(idx[w][l].numel())
                m.idx = _ptr(idx[w][l]) if c else None
                m.val = _ptr(val[w][l]) if c else None
                m.count = c
        self.dense = (ctypes.c_void_p * L)(*[int(d.data_ptr()) for d in dense])
        self.n = (ctypes.c_int64 * L)(*[int(d.numel()) for d in dense])


def rgc_compress_layers(ctx: Context, layers: LayerList, momentum: float = 0.0, flags: int = 0,
                        stream=None) -> None:
    _check(load_library().rgc_compress_layers(ctx.handle, layers.array, layers.num_layers,
                                              float(momentum), int(flags), _stream(stream)))


def rgc_compress_layers_scaled(ctx: Context, layers: LayerList, momentum: float = 0.0, grad_scale=None,
                               flags: int = 0, stream=None) -> None:
    """grad_scale: a one-element float32 device tensor (or None)."""
    _check(load_library().rgc_compress_layers_scaled(ctx.handle, layers.array, layers.num_layers,
                                                     float(momentum), _ptr(grad_scale), int(flags), _stream(stream)))


def rgc_compress_layers_threshold(ctx: Context, layers: LayerList, momentum: float, thresholds, nnz=None,
                                  flags: int = 0, stream=None, grad_scale=None) -> None:
    """thresholds: float32 device tensor of num_layers elements (written with RGC_THRESHOLD_SEARCH, read
    otherwise); nnz: int32 device tensor of num_layers elements or None; grad_scale: a one-element float32
    device tensor or None.  The layers' out_idx / out_val hold 2 * k entries."""
    _check(load_library().rgc_compress_layers_threshold(ctx.handle, layers.array, layers.num_layers, float(momentum),
                                                        _ptr(grad_scale) if grad_scale is not None else None,
                                                        _ptr(thresholds), _ptr(nnz) if nnz is not None else None,
                                                        int(flags), _stream(stream)))


def rgc_message_means(ctx: Context, layers: LayerList, means, stream=None) -> None:
    """means: a float32 device tensor of num_layers elements that receives each layer's average value."""
    _check(load_library().rgc_message_means(ctx.handle, layers.array, layers.num_layers, _ptr(means), _stream(stream)))


RGC_NOALLOC_MAX_LAYERS = 64


def rgc_message_means_noalloc(values: Sequence, counts, capacity: Sequence[int], means, stream=None) -> None:
    """values: one float32 device tensor per message; counts: an int32 device tensor holding their length
    words, one per message; capacity: how many values each buffer holds; means: float32 device tensor."""
    L = len(values)
    vp = (ctypes.c_void_p * max(L, 1))(*[int(v.data_ptr()) for v in values])
    base = int(counts.data_ptr())
    cp = (ctypes.c_void_p * max(L, 1))(*[base + 4 * l for l in range(L)])
    cap = (ctypes.c_int32 * max(L, 1))(*[int(c) for c in capacity])
    _check(load_library().rgc_message_means_noalloc(vp, cp, cap, L, _ptr(means), _stream(stream)))


def rgc_stream_yardstick(grad, residual, velocity, momentum: float, reverse: bool = False, stream=None) -> None:
    """grad, residual, velocity: float32 device tensors of one length; residual and velocity are updated in place."""
    _check(load_library().rgc_stream_yardstick(_ptr(grad), _ptr(residual), _ptr(velocity), int(grad.numel()),
                                               float(momentum), int(bool(reverse)), _stream(stream)))


def rgc_clip_coefficient(ctx: Context, layers: LayerList, max_norm: float, num_workers: int, coefficient,
                         stream=None) -> None:
    """coefficient: a one-element float32 device tensor that receives the clipping coefficient."""
    _check(load_library().rgc_clip_coefficient(ctx.handle, layers.array, layers.num_layers, float(max_norm),
                                               int(num_workers), _ptr(coefficient), _stream(stream)))


def rgc_decompress_accumulate(ctx: Context, msgs: MessageList, scale: float,
                              flags: int = RGC_OVERWRITE, stream=None) -> None:
    _check(load_library().rgc_decompress_accumulate(ctx.handle, msgs.msgs, msgs.num_workers,
                                                    msgs.num_layers, msgs.dense, msgs.n,
                                                    float(scale), int(flags), _stream(stream)))
