"""ctypes binding of libsbc.so: one Python function per C entry point, same names.

Argument marshalling only: torch tensors are used for device memory and the
current stream; every step of the method runs inside the library's HIP kernels.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch  # imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsbc.so")
_lib = None

SBC_OK = 0
SBC_EINVAL = -1
SBC_ECAPACITY = -2
SBC_EHIP = -3
SBC_ECORRUPT = -4
SBC_ENONFINITE = -5
SBC_EINTERNAL = -6
SBC_OPT_FORCE_EXACT_PATH = 1
SBC_OPT_CARRY_FILTER_KEYS = 2
SBC_OPT_WIDE_MIN_KEPT = 3
SBC_OPT_SAMPLED_THRESHOLD = 4
SBC_OPT_DEFER_DECODE_STATUS = 5
SBC_OPT_FUSED_STEP = 6
SBC_ROUTE_CARRIED_KEYS = 1
SBC_ROUTE_HISTOGRAM = 2
SBC_ROUTE_WIDE = 4
SBC_ROUTE_LOOSE_KEYS = 8
SBC_ROUTE_TAKEN_OVER = 16

EXPORTS = (
    "sbc_create", "sbc_create_compact", "sbc_destroy", "sbc_golomb_bstar", "sbc_num_kept", "sbc_msg_bound", "sbc_msg_bound_sampled",
    "sbc_compress", "sbc_compress_begin", "sbc_compress_end", "sbc_decompress_accumulate", "sbc_last_tensor_stats", "sbc_last_mask",
    "sbc_profile_enable", "sbc_profile_level", "sbc_profile_read", "sbc_copy_baseline", "sbc_set_option",
    "sbc_last_route", "sbc_strerror", "sbc_decode_status", "sbc_decompress_accumulate_noalloc", "sbc_last_candidates",
)


class SbcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, sbc_strerror(code), code))


def load() -> ctypes.CDLL:
    """Loads libsbc.so (built by paper_1805_08768_amd/build.py) and declares the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libsbc.so is missing: run `python -m paper_1805_08768_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    lib.sbc_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, ctypes.c_int]
    lib.sbc_create.restype = ctypes.c_int
    lib.sbc_create_compact.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, ctypes.c_int]
    lib.sbc_create_compact.restype = ctypes.c_int
    lib.sbc_destroy.argtypes = [vp]
    lib.sbc_destroy.restype = None
    lib.sbc_golomb_bstar.argtypes = [ctypes.c_double]
    lib.sbc_golomb_bstar.restype = ctypes.c_int
    lib.sbc_num_kept.argtypes = [i64, ctypes.c_double]
    lib.sbc_num_kept.restype = i64
    lib.sbc_msg_bound.argtypes = [ctypes.POINTER(i64), ctypes.c_int, ctypes.c_double]
    lib.sbc_msg_bound.restype = sz
    lib.sbc_msg_bound_sampled.argtypes = [ctypes.POINTER(i64), ctypes.c_int, ctypes.c_double]
    lib.sbc_msg_bound_sampled.restype = sz
    lib.sbc_compress.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(i64),
                                 ctypes.c_int, ctypes.c_double, vp, sz, ctypes.POINTER(sz)]
    lib.sbc_compress.restype = ctypes.c_int
    lib.sbc_compress_begin.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(i64),
                                       ctypes.c_int, ctypes.c_double, vp, sz]
    lib.sbc_compress_begin.restype = ctypes.c_int
    lib.sbc_compress_end.argtypes = [vp, ctypes.POINTER(sz)]
    lib.sbc_compress_end.restype = ctypes.c_int
    lib.sbc_decompress_accumulate.argtypes = [vp, vp, vp, sz, ctypes.POINTER(i64), ctypes.c_int,
                                              ctypes.c_double, ctypes.c_float, ctypes.POINTER(vp)]
    lib.sbc_decompress_accumulate.restype = ctypes.c_int
    lib.sbc_last_tensor_stats.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int),
                                          ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.sbc_last_tensor_stats.restype = ctypes.c_int
    lib.sbc_last_candidates.argtypes = [vp, ctypes.c_int, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.sbc_last_candidates.restype = ctypes.c_int
    lib.sbc_last_mask.argtypes = [vp, ctypes.c_int, vp, sz]
    lib.sbc_last_mask.restype = ctypes.c_int
    lib.sbc_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.sbc_profile_enable.restype = ctypes.c_int
    lib.sbc_profile_level.argtypes = [vp, ctypes.c_int]
    lib.sbc_profile_level.restype = ctypes.c_int
    lib.sbc_profile_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                     ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    lib.sbc_profile_read.restype = ctypes.c_int
    lib.sbc_copy_baseline.argtypes = [vp, vp, vp, sz]
    lib.sbc_copy_baseline.restype = ctypes.c_int
    lib.sbc_set_option.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    lib.sbc_set_option.restype = ctypes.c_int
    lib.sbc_last_route.argtypes = [vp]
    lib.sbc_last_route.restype = ctypes.c_int
    lib.sbc_decode_status.argtypes = [vp, vp]
    lib.sbc_decode_status.restype = ctypes.c_int
    lib.sbc_decompress_accumulate_noalloc.argtypes = [ctypes.c_int, vp, vp, sz, ctypes.POINTER(i64), ctypes.c_int,
                                                      ctypes.c_double, ctypes.c_float, ctypes.POINTER(vp), vp]
    lib.sbc_decompress_accumulate_noalloc.restype = ctypes.c_int
    lib.sbc_strerror.argtypes = [ctypes.c_int]
    lib.sbc_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check_device(t: torch.Tensor) -> None:
    if not t.is_cuda:
        raise ValueError("libsbc works on device memory: expected a CUDA/HIP tensor")


def _ptr_array(tensors: Sequence[torch.Tensor], dtype: torch.dtype):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        _check_device(t)
        if t.dtype != dtype or not t.is_contiguous():
            raise ValueError("tensor %d must be contiguous %s" % (i, dtype))
        arr[i] = t.data_ptr()
    return arr


def _i64_array(values: Sequence[int]):
    return (ctypes.c_int64 * len(values))(*[int(v) for v in values])


_NUMEL_KEYS: dict = {}


class TensorList:
    """A list of contiguous fp32 device tensors marshalled once into the pointer and size arrays
    the C ABI takes.  Keeps the tensors alive.  Pass it instead of a plain list when the same
    buffers are used call after call (weights, residuals, accumulators): marshalling a few
    hundred tensors in Python costs more than the kernels."""

    def __init__(self, tensors: Sequence[torch.Tensor]):
        self.tensors = list(tensors)
        self.ptrs = _ptr_array(self.tensors, torch.float32)
        self.numel = [t.numel() for t in self.tensors]
        # (lists of the same sizes share one key object, so that comparing two lists is one pointer test)
        key = tuple(self.numel)
        self.numel_key = _NUMEL_KEYS.setdefault(key, key)
        self.numel_arr = _i64_array(self.numel)

    def __len__(self):
        return len(self.tensors)


def _as_list(x) -> "TensorList":
    return x if isinstance(x, TensorList) else TensorList(x)


def _stream_handle(stream) -> Optional[int]:
    """stream: None (torch's current stream), a torch stream, or a raw hipStream_t as an int."""
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class MessageBuffer:
    """A contiguous uint8 device tensor checked and marshalled once, for callers that reuse one
    message buffer call after call.  Keeps the tensor alive."""

    def __init__(self, tensor: torch.Tensor):
        _check_device(tensor)
        if tensor.dtype != torch.uint8 or not tensor.is_contiguous():
            raise ValueError("msg must be a contiguous uint8 tensor")
        self.tensor = tensor
        self.ptr = ctypes.c_void_p(tensor.data_ptr())
        self.capacity = tensor.numel()


def _as_msg(x) -> "MessageBuffer":
    return x if isinstance(x, MessageBuffer) else MessageBuffer(x)


# ------------------------------------------------------------------ scalars

def sbc_strerror(code: int) -> str:
    return load().sbc_strerror(int(code)).decode()


def sbc_golomb_bstar(p: float) -> int:
    return int(load().sbc_golomb_bstar(float(p)))


def sbc_num_kept(numel: int, p: float) -> int:
    return int(load().sbc_num_kept(int(numel), float(p)))


def sbc_msg_bound(numel: Sequence[int], p: float) -> int:
    return int(load().sbc_msg_bound(_i64_array(numel), len(numel), float(p)))


def sbc_msg_bound_sampled(numel: Sequence[int], p: float) -> int:
    return int(load().sbc_msg_bound_sampled(_i64_array(numel), len(numel), float(p)))


# ------------------------------------------------------------------ context

def sbc_create(device: int, max_total_elems: int, max_tensors: int) -> ctypes.c_void_p:
    ctx = ctypes.c_void_p()
    rc = load().sbc_create(ctypes.byref(ctx), int(device), int(max_total_elems), int(max_tensors))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_create")
    return ctx


def sbc_create_compact(device: int, max_total_elems: int, max_tensors: int) -> ctypes.c_void_p:
    """A context with candidate lists of a quarter of each tensor per side (about 5 bytes of scratch per entry)."""
    ctx = ctypes.c_void_p()
    rc = load().sbc_create_compact(ctypes.byref(ctx), int(device), int(max_total_elems), int(max_tensors))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_create_compact")
    return ctx


def sbc_destroy(ctx: ctypes.c_void_p) -> None:
    load().sbc_destroy(ctx)


def sbc_compress(ctx, dW, residual, p: float,
                 msg: torch.Tensor, stream=None) -> int:
    """Runs the client step on the given fp32 device tensors (lists of tensors or TensorList);
    returns the message size in bytes.  `residual` is updated in place, `msg` (uint8 device
    tensor) receives the message."""
    dW, residual, msg = _as_list(dW), _as_list(residual), _as_msg(msg)
    if dW.numel_key is not residual.numel_key and dW.numel_key != residual.numel_key:
        raise ValueError("dW and residual must list tensors of the same sizes")
    out_bytes = ctypes.c_size_t(0)
    rc = load().sbc_compress(ctx, _stream_handle(stream), dW.ptrs, residual.ptrs, dW.numel_arr, len(dW.tensors),
                             p, msg.ptr, msg.capacity, ctypes.byref(out_bytes))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_compress")
    return int(out_bytes.value)


def sbc_compress_begin(ctx, dW, residual, p: float, msg: torch.Tensor, stream=None) -> None:
    """Enqueues the client step without waiting; sbc_compress_end(ctx) completes it.  The tensors
    and `msg` must stay alive and untouched until then."""
    dW, residual, msg = _as_list(dW), _as_list(residual), _as_msg(msg)
    if dW.numel_key is not residual.numel_key and dW.numel_key != residual.numel_key:
        raise ValueError("dW and residual must list tensors of the same sizes")
    rc = load().sbc_compress_begin(ctx, _stream_handle(stream), dW.ptrs, residual.ptrs, dW.numel_arr,
                                   len(dW.tensors), p, msg.ptr, msg.capacity)
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_compress_begin")


def sbc_compress_end(ctx) -> int:
    """Waits for the step enqueued by sbc_compress_begin; returns the message size in bytes."""
    out_bytes = ctypes.c_size_t(0)
    rc = load().sbc_compress_end(ctx, ctypes.byref(out_bytes))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_compress_end")
    return int(out_bytes.value)


def sbc_decompress_accumulate(ctx, msg: torch.Tensor, msg_bytes: int, p: float, scale: float,
                              out, stream=None) -> None:
    """Adds scale * (decoded sparse binary update) of one client message into `out`."""
    msg = _as_msg(msg)
    if msg_bytes > msg.capacity:
        raise ValueError("msg must be a contiguous uint8 tensor holding msg_bytes bytes")
    out = _as_list(out)
    rc = load().sbc_decompress_accumulate(ctx, _stream_handle(stream), msg.ptr, msg_bytes, out.numel_arr,
                                          len(out.tensors), p, scale, out.ptrs)
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_decompress_accumulate")


def sbc_decompress_accumulate_noalloc(msg: torch.Tensor, msg_bytes: int, p: float, scale: float, out,
                                      status: torch.Tensor, stream=None, device: int = 0) -> None:
    """The server step without a context and without any allocation; only enqueues.  `status`
    (one int32 on the device) receives the validation result once the stream has passed the call."""
    msg = _as_msg(msg)
    if msg_bytes > msg.capacity:
        raise ValueError("msg must be a contiguous uint8 tensor holding msg_bytes bytes")
    _check_device(status)
    if status.dtype != torch.int32 or status.numel() < 1:
        raise ValueError("status must be an int32 device tensor")
    out = _as_list(out)
    rc = load().sbc_decompress_accumulate_noalloc(int(device), _stream_handle(stream), msg.ptr, msg_bytes,
                                                  out.numel_arr, len(out.tensors), p, scale, out.ptrs,
                                                  ctypes.c_void_p(status.data_ptr()))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_decompress_accumulate_noalloc")


def sbc_decode_status(ctx, stream=None) -> None:
    """With SBC_OPT_DEFER_DECODE_STATUS: waits for the stream and raises if any deferred
    sbc_decompress_accumulate call since the previous check failed validation."""
    rc = load().sbc_decode_status(ctx, _stream_handle(stream))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_decode_status")


def sbc_last_tensor_stats(ctx, tensor: int) -> Tuple[float, float, int, int, int]:
    """(mu_pos, mu_neg, side, nnz, bit_len) of one tensor of the latest sbc_compress call."""
    mp, mn = ctypes.c_double(), ctypes.c_double()
    side = ctypes.c_int()
    nnz, bl = ctypes.c_int64(), ctypes.c_int64()
    rc = load().sbc_last_tensor_stats(ctx, int(tensor), ctypes.byref(mp), ctypes.byref(mn),
                                      ctypes.byref(side), ctypes.byref(nnz), ctypes.byref(bl))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_last_tensor_stats")
    return mp.value, mn.value, side.value, nnz.value, bl.value


def sbc_last_candidates(ctx, tensor: int) -> Tuple[int, int]:
    """(positive, negative) candidate counts of one tensor of the latest sbc_compress call."""
    cp, cn = ctypes.c_int64(), ctypes.c_int64()
    rc = load().sbc_last_candidates(ctx, int(tensor), ctypes.byref(cp), ctypes.byref(cn))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_last_candidates")
    return cp.value, cn.value


def sbc_last_mask(ctx, tensor: int, numel: int) -> torch.Tensor:
    """Kept-position bitmap of one tensor of the latest sbc_compress call as a host int32
    tensor of ceil(numel/32) words (entry j is bit j%32 of word j//32)."""
    n_words = (int(numel) + 31) // 32
    words = torch.empty(n_words, dtype=torch.int32)
    rc = load().sbc_last_mask(ctx, int(tensor), ctypes.c_void_p(words.data_ptr()), n_words)
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_last_mask")
    return words


def sbc_profile_level(ctx, level: int) -> None:
    rc = load().sbc_profile_level(ctx, int(level))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_profile_level")


def sbc_profile_enable(ctx, level: int) -> None:
    rc = load().sbc_profile_enable(ctx, int(level))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_profile_enable")


def sbc_profile_read(ctx) -> List[Tuple[str, float, int]]:
    """[(kernel name, total ms, bracketed launches)] for every stage of sbc_compress."""
    out = []
    stage = 0
    while True:
        name = ctypes.c_char_p()
        ms = ctypes.c_double()
        calls = ctypes.c_int64()
        rc = load().sbc_profile_read(ctx, stage, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(calls))
        if rc != SBC_OK:
            break
        out.append((name.value.decode(), ms.value, calls.value))
        stage += 1
    return out


def sbc_copy_baseline(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Enqueues the library's plain streaming copy kernel dst <- src (no synchronisation)."""
    _check_device(dst)
    _check_device(src)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    rc = load().sbc_copy_baseline(_stream_handle(stream), ctypes.c_void_p(dst.data_ptr()),
                                  ctypes.c_void_p(src.data_ptr()), nbytes)
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_copy_baseline")


def sbc_set_option(ctx, option: int, value: int) -> None:
    rc = load().sbc_set_option(ctx, int(option), int(value))
    if rc != SBC_OK:
        raise SbcError(rc, "sbc_set_option")


def sbc_last_route(ctx) -> int:
    """Bit set of SBC_ROUTE_CARRIED_KEYS / SBC_ROUTE_HISTOGRAM for the latest sbc_compress call."""
    rc = load().sbc_last_route(ctx)
    if rc < 0:
        raise SbcError(rc, "sbc_last_route")
    return rc
