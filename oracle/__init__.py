"""CPU float64 oracle for x_t = a_t x_{t-1} + b_t.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``heinsen_oracle.c`` (plain C, float64 / complex128).  Only tests, the smoke
check and the CPU leg of the benchmark may import this package; the GPU library never does and the
two share no code.

Functions
---------
sequential(a, b, x0, layout=..., threads=1)   the definition (paper Sec. 3), float32/float64 inputs
sequential_log(log_a, log_b, log_x0, ...)     the same loop in the log domain (positive data)
logspace(a, b, x0)                            the closed form of Sec. 4 with complex logs, one sequence
lcse(z)                                       LCSE of Sec. 4 on a complex vector
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "heinsen_oracle.c")
# HEINSEN_ORACLE_SANITIZE=1: a second build with AddressSanitizer and UndefinedBehaviorSanitizer (CPU only), to
# be run with libasan preloaded, e.g.
#   LD_PRELOAD="$(gcc -print-file-name=libasan.so) $LD_PRELOAD" ASAN_OPTIONS=detect_leaks=0 \
#   HEINSEN_ORACLE_SANITIZE=1 python -m pytest tests/test_oracle_pins.py -q
_SANITIZE = os.environ.get("HEINSEN_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libheinsen_oracle_san.so" if _SANITIZE else "libheinsen_oracle.so")

LAYOUT_BND = 0  # [B, n, D]
LAYOUT_BDN = 1  # [B, D, n]

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if _SANITIZE else []
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-std=gnu11", *extra, "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, dbl, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        p = ctypes.c_void_p
        lib.oracle_seq_f64.argtypes = [p, p, dbl, p, i64]
        lib.oracle_seq_f64.restype = None
        lib.oracle_sequential_f32in.argtypes = [p, p, p, p, i64, i64, i64, ci, ci, ci]
        lib.oracle_sequential_f32in.restype = None
        lib.oracle_sequential_log_f32in.argtypes = [p, p, p, p, i64, i64, i64, ci, ci, ci]
        lib.oracle_sequential_log_f32in.restype = None
        lib.oracle_lcse_c128.argtypes = [p, p, i64]
        lib.oracle_lcse_c128.restype = None
        lib.oracle_logspace_c128.argtypes = [p, p, dbl, p, p, p, i64]
        lib.oracle_logspace_c128.restype = ci
        lib.oracle_max_threads.argtypes = []
        lib.oracle_max_threads.restype = ci
        _lib = lib
    return _lib


def _ptr(arr: np.ndarray):
    return arr.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def seq_f64(a, b, x0: float) -> np.ndarray:
    """One sequence, float64 in, float64 out: out[t-1] = x_t."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    assert a.ndim == 1 and a.shape == b.shape
    out = np.empty_like(a)
    _load().oracle_seq_f64(_ptr(a), _ptr(b), float(x0), _ptr(out), a.shape[0])
    return out


def _batched(fn, a, b, x0, layout, threads):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.ndim == 3 and a.shape == b.shape
    if layout == LAYOUT_BND:
        B, n, D = a.shape
    elif layout == LAYOUT_BDN:
        B, D, n = a.shape
    else:
        raise ValueError("layout")
    x0 = np.ascontiguousarray(x0, dtype=np.float32).reshape(-1)
    scalar = 1 if x0.size == 1 else 0
    assert scalar or x0.size == B * D
    out = np.empty(a.shape, dtype=np.float64)
    fn(_ptr(a), _ptr(b), _ptr(x0), _ptr(out), B, D, n, layout, scalar, int(threads))
    return out


def sequential(a, b, x0, layout: int = LAYOUT_BDN, threads: int = 1) -> np.ndarray:
    """Definition of the recurrence on float32-stored inputs (widened exactly), float64 result.

    a, b: 3-d arrays in ``layout``; x0: B*D values (or one, broadcast). bf16 inputs must be widened to
    float32 by the caller (exact)."""
    return _batched(_load().oracle_sequential_f32in, a, b, x0, layout, threads)


def sequential_log(log_a, log_b, log_x0, layout: int = LAYOUT_BDN, threads: int = 1) -> np.ndarray:
    """Log-domain form of the definition for positive data: returns float64 log x_t."""
    return _batched(_load().oracle_sequential_log_f32in, log_a, log_b, log_x0, layout, threads)


def sequential_clog(a, b, x0, layout: int = LAYOUT_BDN, threads: int = 1) -> np.ndarray:
    """Complex logarithm of the recurrence on signed data (paper Sec. 1, last paragraph: the logarithm of a
    negative number is complex): complex128 with real part log|x_t| and imaginary part pi where x_t < 0,
    0 elsewhere (principal value), x_t from the definition in float64."""
    x = sequential(a, b, x0, layout=layout, threads=threads)
    with np.errstate(divide="ignore"):
        re = np.log(np.abs(x))
    return re + 1j * np.where(np.signbit(x), np.pi, 0.0)


def seq_clog_scaled(a, b, x0: float) -> np.ndarray:
    """Complex logarithm of one sequence whose values may leave the float64 range: the definition
    x_t = a_t x_{t-1} + b_t with x carried as sign * exp(l), i.e. x_t = exp(l_{t-1}) (a_t sign + b_t exp(-l_{t-1})).
    Pure Python, for short sequences.  Returns complex128 (log|x_t|, pi where x_t < 0)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    n = a.shape[0]
    out = np.empty(n, dtype=np.complex128)
    x0 = float(x0)
    l = math.log(abs(x0)) if x0 != 0.0 else -math.inf
    sg = -1.0 if x0 < 0 else 1.0
    for t in range(n):
        if l == -math.inf:
            y = b[t]
            base = 0.0
        else:
            y = a[t] * sg + b[t] * math.exp(-l) if l > -700.0 else (a[t] * sg * math.exp(l) + b[t])
            base = l if l > -700.0 else 0.0
        l = base + math.log(abs(y)) if y != 0.0 else -math.inf
        sg = -1.0 if y < 0 else 1.0
        out[t] = complex(l, math.pi if y < 0 else 0.0)
    return out


def lcse(z) -> np.ndarray:
    """LCSE(z) = log cumsum exp(z) on a complex128 vector (paper Sec. 4)."""
    z = np.ascontiguousarray(z, dtype=np.complex128)
    out = np.empty_like(z)
    _load().oracle_lcse_c128(_ptr(z), _ptr(out), z.shape[0])
    return out


def logspace(a, b, x0: float):
    """Closed form of Sec. 4 for one sequence.  Returns (x, log_x) with log_x complex128."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    n = a.shape[0]
    x = np.empty(n, dtype=np.float64)
    re = np.empty(n, dtype=np.float64)
    im = np.empty(n, dtype=np.float64)
    rc = _load().oracle_logspace_c128(_ptr(a), _ptr(b), float(x0), _ptr(x), _ptr(re), _ptr(im), n)
    if rc != 0:
        raise MemoryError("oracle_logspace_c128")
    return x, re + 1j * im
