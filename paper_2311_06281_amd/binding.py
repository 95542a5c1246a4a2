"""ctypes binding of libheinsen: same names as include/heinsen.h, argument marshalling only.

Every step of the computation runs in the HIP kernels of the shared library; nothing here (or
anywhere in this package) falls back to the CPU.  If the library has not been built, importing the
entry points raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libheinsen.so")

HEINSEN_LAYOUT_BND = 0
HEINSEN_LAYOUT_BDN = 1
LAYOUTS = {"BND": HEINSEN_LAYOUT_BND, "BDN": HEINSEN_LAYOUT_BDN}

HEINSEN_LOG_INPUTS = 1 << 0
HEINSEN_LOG_OUTPUT = 1 << 1
HEINSEN_IN_BF16 = 1 << 2
HEINSEN_POSITIVE = 1 << 3
HEINSEN_X0_SCALAR = 1 << 4
HEINSEN_OUT_COMPLEX = 1 << 5
HEINSEN_LINEAR = 1 << 6
FLAGS = {"LOG_INPUTS": HEINSEN_LOG_INPUTS, "LOG_OUTPUT": HEINSEN_LOG_OUTPUT, "IN_BF16": HEINSEN_IN_BF16,
         "POSITIVE": HEINSEN_POSITIVE, "X0_SCALAR": HEINSEN_X0_SCALAR, "OUT_COMPLEX": HEINSEN_OUT_COMPLEX,
         "LINEAR": HEINSEN_LINEAR}

HEINSEN_OK = 0
HEINSEN_ERR_INVALID_ARG = 1
HEINSEN_ERR_UNSUPPORTED = 2
HEINSEN_ERR_ALLOC = 3
HEINSEN_ERR_HIP = 4
HEINSEN_ERR_SCRATCH_LIMIT = 5
HEINSEN_ERR_CARRY_LOST = 6

EXPORTS = ("heinsen_scan", "heinsen_scan_static", "heinsen_status_string", "heinsen_last_hip_error", "heinsen_version",
           "heinsen_release_scratch", "heinsen_kernel_name", "heinsen_tile_shape", "heinsen_sequential", "heinsen_check",
           "heinsen_set_timeline", "heinsen_test_carry", "heinsen_stream_probe")

_lib = None


class HeinsenError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libheinsen: {message} (status {status})")
        self.status = status


def load() -> ctypes.CDLL:
    """Load the shared library built by paper_2311_06281_amd.build (raises if it is missing)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2311_06281_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32
        lib.heinsen_scan.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, u32, vp]
        lib.heinsen_scan.restype = ci
        lib.heinsen_scan_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, u32, vp]
        lib.heinsen_scan_static.restype = ci
        lib.heinsen_status_string.argtypes = [ci]
        lib.heinsen_status_string.restype = ctypes.c_char_p
        lib.heinsen_last_hip_error.argtypes = []
        lib.heinsen_last_hip_error.restype = ci
        lib.heinsen_version.argtypes = []
        lib.heinsen_version.restype = ci
        lib.heinsen_release_scratch.argtypes = []
        lib.heinsen_release_scratch.restype = ci
        lib.heinsen_kernel_name.argtypes = [i64, i64, i64, ci, u32, ctypes.c_char_p, ci]
        lib.heinsen_kernel_name.restype = ci
        lib.heinsen_tile_shape.argtypes = [i64, i64, i64, ci, u32, ctypes.POINTER(ci), ctypes.POINTER(i64)]
        lib.heinsen_tile_shape.restype = ci
        lib.heinsen_check.argtypes = [vp]
        lib.heinsen_check.restype = ci
        lib.heinsen_set_timeline.argtypes = [vp, ctypes.c_uint64]
        lib.heinsen_set_timeline.restype = ci
        lib.heinsen_test_carry.argtypes = [u32, u32, u32, vp]
        lib.heinsen_test_carry.restype = ci
        lib.heinsen_stream_probe.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp]
        lib.heinsen_stream_probe.restype = ci
        lib.heinsen_sequential.argtypes = [vp, vp, vp, vp, i64, vp]
        lib.heinsen_sequential.restype = ci
        _lib = lib
    return _lib


def _addr(x) -> int:
    """Device address of a tensor-like object (anything with data_ptr()) or a plain integer."""
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _stream_handle(stream) -> int:
    if stream is None:
        return 0
    if hasattr(stream, "cuda_stream"):  # torch.cuda.Stream
        return int(stream.cuda_stream)
    return int(stream)


def flags_from_names(names) -> int:
    f = 0
    for nm in names:
        f |= FLAGS[nm]
    return f


def heinsen_status_string(status: int) -> str:
    return load().heinsen_status_string(int(status)).decode()


def heinsen_last_hip_error() -> int:
    return int(load().heinsen_last_hip_error())


def heinsen_version() -> int:
    return int(load().heinsen_version())


def heinsen_release_scratch() -> int:
    return int(load().heinsen_release_scratch())


def heinsen_kernel_name(B: int, D: int, n: int, layout: int, flags: int) -> str:
    buf = ctypes.create_string_buffer(128)
    st = load().heinsen_kernel_name(B, D, n, layout, flags, buf, 128)
    if st != HEINSEN_OK:
        raise HeinsenError(st, heinsen_status_string(st))
    return buf.value.decode()


def heinsen_tile_shape(B: int, D: int, n: int, layout: int, flags: int):
    """(adjacent sequences, consecutive steps) of the tile one workgroup takes; see include/heinsen.h."""
    seqs, steps = ctypes.c_int(0), ctypes.c_int64(0)
    st = load().heinsen_tile_shape(B, D, n, layout, flags, ctypes.byref(seqs), ctypes.byref(steps))
    if st != HEINSEN_OK:
        raise HeinsenError(st, heinsen_status_string(st))
    return seqs.value, steps.value


def heinsen_scan_status(a, b, x0, out, B: int, D: int, n: int, layout: int, flags: int, stream=None) -> int:
    """Raw call: returns the heinsen_status_t instead of raising."""
    return int(load().heinsen_scan(_addr(a), _addr(b), _addr(x0), _addr(out), int(B), int(D), int(n),
                                   int(layout), int(flags), _stream_handle(stream)))


def heinsen_scan(a, b, x0, out, B: int, D: int, n: int, layout: int, flags: int, stream=None) -> None:
    """x_t = a_t x_{t-1} + b_t for B*D sequences; see include/heinsen.h.  Asynchronous on `stream`.

    a, b, x0, out: device tensors (anything with data_ptr()) or integer device addresses."""
    st = heinsen_scan_status(a, b, x0, out, B, D, n, layout, flags, stream)
    if st != HEINSEN_OK:
        msg = heinsen_status_string(st)
        if st in (HEINSEN_ERR_HIP, HEINSEN_ERR_ALLOC):
            msg += f", hipError_t {heinsen_last_hip_error()}"
        raise HeinsenError(st, msg)


def heinsen_scan_static_status(a, b, x0, out, B: int, D: int, n: int, layout: int, flags: int, stream=None) -> int:
    """Raw call of the allocation-free variant: returns the heinsen_status_t instead of raising."""
    return int(load().heinsen_scan_static(_addr(a), _addr(b), _addr(x0), _addr(out), int(B), int(D), int(n),
                                          int(layout), int(flags), _stream_handle(stream)))


def heinsen_scan_static(a, b, x0, out, B: int, D: int, n: int, layout: int, flags: int, stream=None) -> None:
    """heinsen_scan without any device allocation (fixed scratch inside the library); see include/heinsen.h."""
    st = heinsen_scan_static_status(a, b, x0, out, B, D, n, layout, flags, stream)
    if st != HEINSEN_OK:
        msg = heinsen_status_string(st)
        if st == HEINSEN_ERR_HIP:
            msg += f", hipError_t {heinsen_last_hip_error()}"
        raise HeinsenError(st, msg)


def heinsen_check(stream=None) -> int:
    """Synchronises `stream`; HEINSEN_OK, or HEINSEN_ERR_CARRY_LOST if a launch gave up waiting for a carry."""
    return int(load().heinsen_check(_stream_handle(stream)))


def heinsen_set_timeline(stamps, tiles: int) -> None:
    """Per-tile time stamps into the device buffer `stamps` (tiles * 8 uint64); (None, 0) switches them off."""
    st = int(load().heinsen_set_timeline(_addr(stamps), int(tiles)))
    if st != HEINSEN_OK:
        raise HeinsenError(st, heinsen_status_string(st))


def heinsen_test_carry(spin_limit: int = 0, drop_tile: int = 0xFFFFFFFF, epoch: int = 0, stream=None) -> None:
    """Testing aid of the carry chain's error path; see include/heinsen.h."""
    st = int(load().heinsen_test_carry(int(spin_limit), int(drop_tile), int(epoch), _stream_handle(stream)))
    if st != HEINSEN_OK:
        raise HeinsenError(st, heinsen_status_string(st))


def heinsen_stream_probe_status(a, b, out, B: int, n: int, D: int, pattern: int, stream=None) -> int:
    """out = a + b with the access pattern `pattern` of the scan kernels; see include/heinsen.h."""
    return int(load().heinsen_stream_probe(_addr(a), _addr(b), _addr(out), int(B), int(n), int(D), int(pattern),
                                           _stream_handle(stream)))


def heinsen_sequential(a, b, x0, out, n: int, stream=None) -> None:
    """One sequence, one element after the other, on the GPU (the baseline of the paper's Fig. 1)."""
    st = int(load().heinsen_sequential(_addr(a), _addr(b), _addr(x0), _addr(out), int(n), _stream_handle(stream)))
    if st != HEINSEN_OK:
        raise HeinsenError(st, heinsen_status_string(st))
