"""CPU oracle for the segmented-operation hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never imports it.

``oracle.mmvseg_oracle.c`` holds the sequential definitions (Problem 2.1 of
Sec. 2 for the segmented scan, the "last element of every segment" definition
of the segmented sum, and y = A x for SpMV); this module compiles that file
with gcc and exposes it through ctypes on numpy arrays.  ``oracle.formulations``
holds the paper's other routes to the same results (SCD, SSCR, the
block-recursive algorithm, the REVSPEC lemma) in plain numpy / Python, used
to pin the definitions against each other.

The parallel primitives that Algorithms SCD and SSCR are composed of (SCAN,
COMPRESS, DIFF, REVERT) and CSR SpMV have their plain definitions here too
(pins: tests/test_oracle_primitives.py).

Pins (tests/test_oracle_pins.py, tests/test_formulations.py): the worked
example printed in Sec. 2, closed forms (all-ones values give segment lengths,
arithmetic series), library special cases (numpy.cumsum, numpy.add.reduceat,
reshape-sum, scipy.sparse), invariants, brute force over every flag pattern
for n <= 12 against an O(n^2) definitional form in Python integers, and the
paper's SCD / SSCR / block-recursive formulations for several s.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# MMVSEG_ORACLE_SANITIZE=1 (tests/test_sanitizers.py): both C files are built with the address and undefined-
# behaviour sanitizers into libraries of their own; the process must then have gcc's libasan preloaded.
_SANITIZE = os.environ.get("MMVSEG_ORACLE_SANITIZE") == "1"
_SAN_FLAGS = ("-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g") if _SANITIZE else ()
_SRC = os.path.join(_HERE, "mmvseg_oracle.c")
_LIB = os.path.join(_HERE, "libmmvseg_oracle%s.so" % ("_san" if _SANITIZE else ""))
_lib = None


_HOST_SRC = os.path.join(_HERE, "host_threads.c")
_HOST_LIB = os.path.join(_HERE, "libmmvseg_host_threads%s.so" % ("_san" if _SANITIZE else ""))
_host_lib = None


def _compile(src: str, lib: str, force: bool, extra=()) -> str:
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        tmp = lib + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-fno-fast-math", *_SAN_FLAGS, *extra, "-o", tmp, src])
        os.replace(tmp, lib)
    return lib


def build(force: bool = False) -> str:
    """Compile the C oracle (-O2, no fast-math, single thread) and the threaded host baseline beside it."""
    _compile(_HOST_SRC, _HOST_LIB, force, ("-pthread",))
    return _compile(_SRC, _LIB, force)


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.oracle_segscan_i8.argtypes = [vp, vp, u64, vp]
        lib.oracle_segscan_i8.restype = None
        lib.oracle_segsum_i8.argtypes = [vp, vp, u64, vp]
        lib.oracle_segsum_i8.restype = u64
        lib.oracle_segscan_xor_u8.argtypes = [vp, vp, u64, vp]
        lib.oracle_segscan_xor_u8.restype = None
        lib.oracle_segsum_xor_u8.argtypes = [vp, vp, u64, vp]
        lib.oracle_segsum_xor_u8.restype = u64
        lib.oracle_segscan_f64.argtypes = [vp, vp, u64, vp]
        lib.oracle_segscan_f64.restype = None
        lib.oracle_segscan_f32in.argtypes = [vp, vp, u64, vp]
        lib.oracle_segscan_f32in.restype = None
        lib.oracle_segsum_f64.argtypes = [vp, vp, u64, vp]
        lib.oracle_segsum_f64.restype = u64
        lib.oracle_spmv_coo.argtypes = [u64, u64, u64, vp, vp, vp, vp, vp]
        lib.oracle_spmv_coo.restype = ctypes.c_int
        lib.oracle_scan_i8.argtypes = [vp, u64, vp]
        lib.oracle_scan_i8.restype = None
        lib.oracle_scan_f32in.argtypes = [vp, u64, vp]
        lib.oracle_scan_f32in.restype = None
        lib.oracle_scan_f64.argtypes = [vp, u64, vp]
        lib.oracle_scan_f64.restype = None
        lib.oracle_compress_u32.argtypes = [vp, vp, u64, vp]
        lib.oracle_compress_u32.restype = u64
        lib.oracle_diff_i32.argtypes = [vp, u64, vp]
        lib.oracle_diff_i32.restype = None
        lib.oracle_diff_f32in.argtypes = [vp, u64, vp]
        lib.oracle_diff_f32in.restype = None
        lib.oracle_revert_i32.argtypes = [vp, vp, vp, u64, u64, vp]
        lib.oracle_revert_i32.restype = ctypes.c_int
        lib.oracle_revert_f32in.argtypes = [vp, vp, vp, u64, u64, vp]
        lib.oracle_revert_f32in.restype = ctypes.c_int
        lib.oracle_spmv_csr.argtypes = [u64, u64, vp, vp, vp, vp, vp]
        lib.oracle_spmv_csr.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _flags_u8(f, n: int) -> np.ndarray:
    """Flags as one byte per element (non-zero = segment start)."""
    f = np.asarray(f)
    if f.shape != (n,):
        raise ValueError("flags must have the same length as the values")
    return np.ascontiguousarray(f != 0, dtype=np.uint8)


def segscan(x, f) -> np.ndarray:
    """Segmented inclusive scan (Problem 2.1).

    int8 values -> int32 result with wrap-around; float16/float32/float64
    values -> float64 result accumulated in float64; uint8 values are elements
    of the group of bytes under bit-wise exclusive or -> int32 holding the byte.
    """
    x = np.ascontiguousarray(x)
    n = x.shape[0]
    f = _flags_u8(f, n)
    lib = _load()
    if x.dtype == np.int8:
        z = np.empty(n, dtype=np.int32)
        lib.oracle_segscan_i8(_ptr(x), _ptr(f), n, _ptr(z))
        return z
    if x.dtype == np.uint8:
        z = np.empty(n, dtype=np.int32)
        lib.oracle_segscan_xor_u8(_ptr(x), _ptr(f), n, _ptr(z))
        return z
    if x.dtype == np.float32:
        z = np.empty(n, dtype=np.float64)
        lib.oracle_segscan_f32in(_ptr(x), _ptr(f), n, _ptr(z))
        return z
    if x.dtype in (np.float16, np.float64):
        xd = np.ascontiguousarray(x, dtype=np.float64)  # exact widening
        z = np.empty(n, dtype=np.float64)
        lib.oracle_segscan_f64(_ptr(xd), _ptr(f), n, _ptr(z))
        return z
    raise TypeError("unsupported value dtype %s" % x.dtype)


def segsum(x, f) -> np.ndarray:
    """Segmented sum: one value per segment, in segment order (Sec. 2)."""
    x = np.ascontiguousarray(x)
    n = x.shape[0]
    f = _flags_u8(f, n)
    lib = _load()
    if n == 0:
        return np.empty(0, dtype=np.int32 if x.dtype in (np.int8, np.uint8) else np.float64)
    # room for the worst case (every element its own segment); the C loop tests
    # i == n-1 before it looks at f[i+1], so nothing past the end is read.
    if x.dtype == np.int8:
        out = np.empty(n, dtype=np.int32)
        k = lib.oracle_segsum_i8(_ptr(x), _ptr(f), n, _ptr(out))
        return out[:k].copy()
    if x.dtype == np.uint8:
        out = np.empty(n, dtype=np.int32)
        k = lib.oracle_segsum_xor_u8(_ptr(x), _ptr(f), n, _ptr(out))
        return out[:k].copy()
    if x.dtype in (np.float16, np.float32, np.float64):
        xd = np.ascontiguousarray(x, dtype=np.float64)
        out = np.empty(n, dtype=np.float64)
        k = lib.oracle_segsum_f64(_ptr(xd), _ptr(f), n, _ptr(out))
        return out[:k].copy()
    raise TypeError("unsupported value dtype %s" % x.dtype)


def spmv_coo(n_rows: int, n_cols: int, row, col, val, x) -> np.ndarray:
    """y = A x in float64 from (row, col, val) triples in any order."""
    row = np.ascontiguousarray(row, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    if not (row.shape == col.shape == val.shape) or x.shape != (n_cols,):
        raise ValueError("shape mismatch")
    y = np.empty(n_rows, dtype=np.float64)
    bad = _load().oracle_spmv_coo(n_rows, n_cols, row.shape[0], _ptr(row), _ptr(col), _ptr(val),
                                  _ptr(x), _ptr(y))
    if bad:
        raise ValueError("row or column index out of range")
    return y


# ---- the parallel primitives of Algorithms SCD and SSCR (Sec. 4.1) -----------------------------

def scan(x) -> np.ndarray:
    """Unsegmented inclusive scan z(i) = x(0) + ... + x(i) (Sec. 1.1; Algorithm Scan computes it).

    int8 -> int32 with wrap-around; float16/float32/float64 -> float64 accumulated in float64.
    """
    x = np.ascontiguousarray(x)
    n = x.shape[0]
    lib = _load()
    if x.dtype == np.int8:
        z = np.empty(n, dtype=np.int32)
        lib.oracle_scan_i8(_ptr(x), n, _ptr(z))
        return z
    if x.dtype == np.uint8:      # bytes under exclusive or: the segmented scan with no flag set
        z = np.empty(n, dtype=np.int32)
        none = np.zeros(n, dtype=np.uint8)
        lib.oracle_segscan_xor_u8(_ptr(x), _ptr(none), n, _ptr(z))
        return z
    if x.dtype == np.float32:
        z = np.empty(n, dtype=np.float64)
        lib.oracle_scan_f32in(_ptr(x), n, _ptr(z))
        return z
    if x.dtype in (np.float16, np.float64):
        xd = np.ascontiguousarray(x, dtype=np.float64)
        z = np.empty(n, dtype=np.float64)
        lib.oracle_scan_f64(_ptr(xd), n, _ptr(z))
        return z
    raise TypeError("unsupported value dtype %s" % x.dtype)


def compress(x, mask) -> np.ndarray:
    """COMPRESS (Sec. 2): the entries of x (any 32-bit type) whose mask entry is non-zero, in order."""
    x = np.ascontiguousarray(x)
    if x.dtype.itemsize != 4:
        raise TypeError("compress works on 32-bit elements")
    n = x.shape[0]
    m = _flags_u8(mask, n)
    out = np.empty(n, dtype=x.dtype)
    k = _load().oracle_compress_u32(_ptr(x), _ptr(m), n, _ptr(out))
    return out[:k].copy()


def diff(x) -> np.ndarray:
    """DIFF (Sec. 4.1): z(i) = x(i) - x(i-1), x(-1) = 0.  int32 wraps; float32 -> float64."""
    x = np.ascontiguousarray(x)
    n = x.shape[0]
    lib = _load()
    if x.dtype == np.int32:
        z = np.empty(n, dtype=np.int32)
        lib.oracle_diff_i32(_ptr(x), n, _ptr(z))
        return z
    if x.dtype == np.float32:
        z = np.empty(n, dtype=np.float64)
        lib.oracle_diff_f32in(_ptr(x), n, _ptr(z))
        return z
    raise TypeError("unsupported value dtype %s" % x.dtype)


def revert(xhat, fhat, w) -> np.ndarray:
    """REVERT (Sec. 4.1): xhat(i) - w(fhat(i) - 2) where the inclusive segment count fhat(i) >= 2."""
    xhat = np.ascontiguousarray(xhat)
    fhat = np.ascontiguousarray(fhat, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=xhat.dtype)
    n = xhat.shape[0]
    if fhat.shape != (n,):
        raise ValueError("shape mismatch")
    lib = _load()
    if xhat.dtype == np.int32:
        z = np.empty(n, dtype=np.int32)
        bad = lib.oracle_revert_i32(_ptr(xhat), _ptr(fhat), _ptr(w), n, w.shape[0], _ptr(z))
    elif xhat.dtype == np.float32:
        z = np.empty(n, dtype=np.float64)
        bad = lib.oracle_revert_f32in(_ptr(xhat), _ptr(fhat), _ptr(w), n, w.shape[0], _ptr(z))
    else:
        raise TypeError("unsupported value dtype %s" % xhat.dtype)
    if bad:
        raise ValueError("a segment count points outside w")
    return z


def spmv_csr(n_rows: int, n_cols: int, rowptr, col, val, x) -> np.ndarray:
    """y = A x in float64 for a CSR matrix (Algorithm "MMV-RAM CSR SpMV", Sec. 4.3)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    if rowptr.shape != (n_rows + 1,) or col.shape != val.shape or x.shape != (n_cols,):
        raise ValueError("shape mismatch")
    if n_rows and (rowptr[0] != 0 or rowptr[-1] != val.shape[0]):
        raise ValueError("rowptr must start at 0 and end at nnz")
    y = np.empty(n_rows, dtype=np.float64)
    bad = _load().oracle_spmv_csr(n_rows, n_cols, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(x), _ptr(y))
    if bad:
        raise ValueError("row pointers not monotone or column index out of range")
    return y


def host_threads_segscan(x, f, threads: int) -> np.ndarray:
    """NOT the oracle: the chunked segmented scan on `threads` host threads (host_threads.c), int8 -> int32,
    the all-cores baseline of the benchmark.  Checked against `segscan` in tests/test_host_threads.py."""
    global _host_lib
    x = np.ascontiguousarray(x)
    if x.dtype != np.int8:
        raise TypeError("the threaded host baseline takes int8 values")
    n = x.shape[0]
    f = _flags_u8(f, n)
    if _host_lib is None:
        build()
        lib = ctypes.CDLL(_HOST_LIB)
        lib.host_threads_segscan_i8.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
                                                ctypes.c_int]
        lib.host_threads_segscan_i8.restype = ctypes.c_int
        _host_lib = lib
    z = np.empty(n, dtype=np.int32)
    used = _host_lib.host_threads_segscan_i8(_ptr(x), _ptr(f), n, _ptr(z), int(threads))
    if used < 0:
        raise RuntimeError("host_threads_segscan_i8 failed (threads=%r)" % (threads,))
    return z
