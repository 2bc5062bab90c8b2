"""ctypes binding of libmmvseg.so: argument marshalling only.

Every function here has the name of the C entry point it calls
(include/mmvseg.h) and takes torch tensors that live on the GPU; torch only
provides the device memory and the HIP stream.  No step of the computation
runs in Python or in torch, and there is no fallback: if the library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmmvseg.so")

MMV_OK = 0
MMV_F32_F32, MMV_F16_F32, MMV_BF16_F32, MMV_I8_I32, MMV_U8_XOR = 0, 1, 2, 3, 4
MMV_FLAGS_U8, MMV_FLAGS_PACKED32 = 0, 1
MMV_VARIANT_MFMA, MMV_VARIANT_SHUFFLE = 0, 1
MMV_OP_SEGSCAN, MMV_OP_SEGSUM, MMV_OP_SPMV_COO = 0, 1, 2
MMV_OP_SCAN, MMV_OP_COMPRESS, MMV_OP_SEGSUM_SCD, MMV_OP_SEGSCAN_SSCR, MMV_OP_SPMV_CSR = 3, 4, 5, 6, 7
MMV_ELEM_I32, MMV_ELEM_F32 = 0, 1

EXPORTS = [
    "mmv_workspace_bytes", "mmv_segscan", "mmv_segsum", "mmv_spmv_coo", "mmv_workspace_status",
    "mmv_stream_copy", "mmv_gather_reference", "mmv_status_string", "mmv_tile_elems", "mmv_set_kernel_events",
    "mmv_spmv_csr_workspace_bytes", "mmv_spmv_csr", "mmv_scan", "mmv_compress", "mmv_diff", "mmv_revert",
    "mmv_segsum_scd", "mmv_segscan_sscr", "mmv_segscan_static",
    "mmv_spmv_coo_prepare", "mmv_spmv_coo_run", "mmv_spmv_csr_prepare", "mmv_spmv_csr_run",
]
STATIC_SCRATCH_BYTES = 1 << 20   # MMV_STATIC_SCRATCH_BYTES

_DTYPES = {torch.float32: MMV_F32_F32, torch.float16: MMV_F16_F32, torch.bfloat16: MMV_BF16_F32,
           torch.int8: MMV_I8_I32, torch.uint8: MMV_U8_XOR}   # uint8 values: bytes under bit-wise exclusive or
_OUT_DTYPE = {MMV_F32_F32: torch.float32, MMV_F16_F32: torch.float32, MMV_BF16_F32: torch.float32,
              MMV_I8_I32: torch.int32, MMV_U8_XOR: torch.int32}
_VARIANTS = {"mfma": MMV_VARIANT_MFMA, "shuffle": MMV_VARIANT_SHUFFLE}

_lib = None


class MmvError(RuntimeError):
    pass


def load() -> ctypes.CDLL:
    """Loads libmmvseg.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MmvError("libmmvseg.so is not built: run `python -m paper_2506_23906_amd.build` "
                       "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, u64, sz, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int
    lib.mmv_workspace_bytes.argtypes = [i32, i32, i32, u64]
    lib.mmv_workspace_bytes.restype = sz
    lib.mmv_segscan.argtypes = [vp, vp, u64, vp, i32, i32, i32, vp, sz, vp]
    lib.mmv_segscan.restype = i32
    lib.mmv_segscan_static.argtypes = [vp, vp, u64, vp, i32, i32, i32, vp]
    lib.mmv_segscan_static.restype = i32
    lib.mmv_segsum.argtypes = [vp, vp, u64, vp, u64, vp, i32, i32, i32, vp, sz, vp]
    lib.mmv_segsum.restype = i32
    lib.mmv_spmv_coo.argtypes = [u64, u64, u64, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.mmv_spmv_coo.restype = i32
    lib.mmv_workspace_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint32)]
    lib.mmv_workspace_status.restype = i32
    lib.mmv_stream_copy.argtypes = [vp, sz, vp, sz, vp]
    lib.mmv_stream_copy.restype = i32
    lib.mmv_gather_reference.argtypes = [u64, vp, vp, u64, vp, vp, vp]
    lib.mmv_gather_reference.restype = i32
    lib.mmv_status_string.argtypes = [i32]
    lib.mmv_status_string.restype = ctypes.c_char_p
    lib.mmv_set_kernel_events.argtypes = [vp, vp]
    lib.mmv_set_kernel_events.restype = i32
    lib.mmv_tile_elems.argtypes = [i32, i32, u64]
    lib.mmv_tile_elems.restype = ctypes.c_uint32
    lib.mmv_spmv_csr_workspace_bytes.argtypes = [u64, u64]
    lib.mmv_spmv_csr_workspace_bytes.restype = sz
    lib.mmv_spmv_csr.argtypes = [u64, u64, u64, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.mmv_spmv_csr.restype = i32
    for name in ("mmv_spmv_coo_prepare", "mmv_spmv_csr_prepare"):
        getattr(lib, name).argtypes = [u64, u64, u64, vp, vp, vp, sz, vp]
        getattr(lib, name).restype = i32
    for name in ("mmv_spmv_coo_run", "mmv_spmv_csr_run"):
        getattr(lib, name).argtypes = [u64, u64, u64, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        getattr(lib, name).restype = i32
    lib.mmv_scan.argtypes = [vp, u64, vp, i32, i32, vp, sz, vp]
    lib.mmv_scan.restype = i32
    lib.mmv_compress.argtypes = [vp, vp, u64, vp, u64, vp, i32, vp, sz, vp]
    lib.mmv_compress.restype = i32
    lib.mmv_diff.argtypes = [vp, u64, vp, i32, vp]
    lib.mmv_diff.restype = i32
    lib.mmv_revert.argtypes = [vp, vp, vp, u64, u64, vp, i32, vp]
    lib.mmv_revert.restype = i32
    lib.mmv_segsum_scd.argtypes = [vp, vp, u64, vp, u64, vp, i32, i32, i32, vp, sz, vp]
    lib.mmv_segsum_scd.restype = i32
    lib.mmv_segscan_sscr.argtypes = [vp, vp, u64, vp, i32, i32, i32, vp, sz, vp]
    lib.mmv_segscan_sscr.restype = i32
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != MMV_OK:
        raise MmvError("%s failed: %s (status %d)" % (what, load().mmv_status_string(status).decode(), status))


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda or not t.is_contiguous():
        raise MmvError("%s must be a contiguous tensor in GPU memory" % name)
    return t.data_ptr()


def _flag_fmt(flags: torch.Tensor) -> int:
    if flags.dtype == torch.uint8:
        return MMV_FLAGS_U8
    if flags.dtype == torch.int32:
        return MMV_FLAGS_PACKED32
    raise MmvError("flags must be uint8 (one byte per element) or int32 (bit-packed words)")


def mmv_tile_elems(op: int = MMV_OP_SEGSCAN, dt: int = MMV_I8_I32, n: int = 1 << 40) -> int:
    """Elements per workgroup tile; the default arguments give the largest tile there is."""
    return int(load().mmv_tile_elems(op, dt, n))


def mmv_workspace_bytes(op: int, dt: int, ff: int, n: int) -> int:
    return int(load().mmv_workspace_bytes(op, dt, ff, n))


def workspace(nbytes: int, device=None) -> torch.Tensor:
    """Scratch of at least `nbytes` bytes (torch allocations are 256-byte aligned)."""
    return torch.empty(max(256, nbytes), dtype=torch.uint8, device=device or "cuda")


def new_workspace(op: int, dt: int, ff: int, n: int, device=None) -> torch.Tensor:
    return workspace(mmv_workspace_bytes(op, dt, ff, n), device)


def mmv_segscan(x: torch.Tensor, flags: torch.Tensor, n: int | None = None, z: torch.Tensor | None = None,
                variant: str = "mfma", ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """Segmented inclusive scan of x under segment-start flags; returns z (fp32 or int32)."""
    lib = load()
    n = x.numel() if n is None else n
    dt, ff = _DTYPES[x.dtype], _flag_fmt(flags)
    if z is None:
        z = torch.empty(n, dtype=_OUT_DTYPE[dt], device=x.device)
    if ws is None:
        ws = new_workspace(MMV_OP_SEGSCAN, dt, ff, n, x.device)
    st = lib.mmv_segscan(_dev(x, "x"), _dev(flags, "flags"), n, _dev(z, "z"), dt, ff, _VARIANTS[variant],
                         _dev(ws, "ws"), ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_segscan")
    return z


def mmv_segscan_static(x: torch.Tensor, flags: torch.Tensor, z: torch.Tensor, n: int | None = None,
                       variant: str = "mfma", stream=None) -> torch.Tensor:
    """mmv_segscan on the library's built-in scratch array: the caller passes inputs and the output, nothing
    is allocated (neither here nor in the library)."""
    n = x.numel() if n is None else n
    st = load().mmv_segscan_static(_dev(x, "x"), _dev(flags, "flags"), n, _dev(z, "z"), _DTYPES[x.dtype],
                                   _flag_fmt(flags), _VARIANTS[variant], _stream_ptr(stream))
    _check(st, "mmv_segscan_static")
    return z


def mmv_segsum(x: torch.Tensor, flags: torch.Tensor, n: int | None = None, out: torch.Tensor | None = None,
               nseg: torch.Tensor | None = None, variant: str = "mfma", ws: torch.Tensor | None = None,
               stream=None):
    """Segmented sum; returns (out, nseg) where nseg is a one-element int64 device tensor."""
    lib = load()
    n = x.numel() if n is None else n
    dt, ff = _DTYPES[x.dtype], _flag_fmt(flags)
    if out is None:
        out = torch.empty(max(n, 1), dtype=_OUT_DTYPE[dt], device=x.device)
    if nseg is None:
        nseg = torch.empty(1, dtype=torch.int64, device=x.device)
    if ws is None:
        ws = new_workspace(MMV_OP_SEGSUM, dt, ff, n, x.device)
    st = lib.mmv_segsum(_dev(x, "x"), _dev(flags, "flags"), n, _dev(out, "out"), out.numel(), _dev(nseg, "nseg"),
                        dt, ff, _VARIANTS[variant], _dev(ws, "ws"), ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_segsum")
    return out, nseg


def mmv_spmv_coo(n_rows: int, n_cols: int, row: torch.Tensor, col: torch.Tensor, val: torch.Tensor,
                 x: torch.Tensor, y: torch.Tensor | None = None, variant: str = "mfma",
                 ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """y = A x for a row-sorted COO matrix (int32 indices, fp32 values)."""
    lib = load()
    nnz = val.numel()
    if y is None:
        y = torch.empty(n_rows, dtype=torch.float32, device=val.device)
    if ws is None:
        ws = new_workspace(MMV_OP_SPMV_COO, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz, val.device)
    st = lib.mmv_spmv_coo(n_rows, n_cols, nnz, _dev(row, "row"), _dev(col, "col"), _dev(val, "val"), _dev(x, "x"),
                          _dev(y, "y"), _VARIANTS[variant], _dev(ws, "ws"), ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_spmv_coo")
    return y


def mmv_spmv_coo_prepare(n_rows: int, n_cols: int, row: torch.Tensor, col: torch.Tensor,
                         ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """First step of the two-step COO SpMV: returns the workspace that holds the plan for this matrix."""
    nnz = row.numel()
    if ws is None:
        ws = new_workspace(MMV_OP_SPMV_COO, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz, row.device)
    st = load().mmv_spmv_coo_prepare(n_rows, n_cols, nnz, _dev(row, "row"), _dev(col, "col"), _dev(ws, "ws"), ws.numel(),
                                     _stream_ptr(stream))
    _check(st, "mmv_spmv_coo_prepare")
    return ws


def mmv_spmv_coo_run(n_rows: int, n_cols: int, row: torch.Tensor, col: torch.Tensor, val: torch.Tensor,
                     x: torch.Tensor, ws: torch.Tensor, y: torch.Tensor | None = None, variant: str = "mfma",
                     stream=None) -> torch.Tensor:
    """Second step: y = A x with the plan that mmv_spmv_coo_prepare left in ws."""
    if y is None:
        y = torch.empty(n_rows, dtype=torch.float32, device=val.device)
    st = load().mmv_spmv_coo_run(n_rows, n_cols, val.numel(), _dev(row, "row"), _dev(col, "col"), _dev(val, "val"),
                                 _dev(x, "x"), _dev(y, "y"), _VARIANTS[variant], _dev(ws, "ws"), ws.numel(),
                                 _stream_ptr(stream))
    _check(st, "mmv_spmv_coo_run")
    return y


def mmv_spmv_csr_prepare(n_rows: int, n_cols: int, rowptr: torch.Tensor, col: torch.Tensor,
                         ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """First step of the two-step CSR SpMV: returns the workspace that holds the plan for this matrix."""
    nnz = col.numel()
    if ws is None:
        ws = workspace(mmv_spmv_csr_workspace_bytes(n_rows, nnz), col.device)
    st = load().mmv_spmv_csr_prepare(n_rows, n_cols, nnz, _dev(rowptr, "rowptr"), _dev(col, "col"), _dev(ws, "ws"),
                                     ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_spmv_csr_prepare")
    return ws


def mmv_spmv_csr_run(n_rows: int, n_cols: int, rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor,
                     x: torch.Tensor, ws: torch.Tensor, y: torch.Tensor | None = None, variant: str = "mfma",
                     stream=None) -> torch.Tensor:
    """Second step: y = A x with the plan that mmv_spmv_csr_prepare left in ws."""
    if y is None:
        y = torch.empty(n_rows, dtype=torch.float32, device=val.device)
    st = load().mmv_spmv_csr_run(n_rows, n_cols, val.numel(), _dev(rowptr, "rowptr"), _dev(col, "col"), _dev(val, "val"),
                                 _dev(x, "x"), _dev(y, "y"), _VARIANTS[variant], _dev(ws, "ws"), ws.numel(),
                                 _stream_ptr(stream))
    _check(st, "mmv_spmv_csr_run")
    return y


def mmv_workspace_status(ws: torch.Tensor, stream=None) -> int:
    h = ctypes.c_uint32(0)
    _check(load().mmv_workspace_status(_dev(ws, "ws"), _stream_ptr(stream), ctypes.byref(h)), "mmv_workspace_status")
    return int(h.value)


def mmv_stream_copy(src: torch.Tensor, dst: torch.Tensor, in_bytes: int | None = None,
                    out_bytes: int | None = None, stream=None) -> None:
    ib = src.numel() * src.element_size() if in_bytes is None else in_bytes
    ob = dst.numel() * dst.element_size() if out_bytes is None else out_bytes
    _check(load().mmv_stream_copy(_dev(src, "src"), ib, _dev(dst, "dst"), ob, _stream_ptr(stream)),
           "mmv_stream_copy")


GATHER_REFERENCE_PARTIALS = 8192 * 256


def mmv_gather_reference(val: torch.Tensor, col: torch.Tensor, x: torch.Tensor, partial: torch.Tensor,
                         nnz: int | None = None, stream=None) -> None:
    if partial.numel() < GATHER_REFERENCE_PARTIALS:
        raise MmvError("mmv_gather_reference: partial needs %d floats" % GATHER_REFERENCE_PARTIALS)
    _check(load().mmv_gather_reference(val.numel() if nnz is None else nnz, _dev(val, "val"), _dev(col, "col"),
                                       x.numel(), _dev(x, "x"), _dev(partial, "partial"), _stream_ptr(stream)),
           "mmv_gather_reference")


def mmv_set_kernel_events(ev_start: int | None, ev_stop: int | None) -> None:
    """ev_start / ev_stop are hipEvent_t handles as integers (or None to switch off)."""
    _check(load().mmv_set_kernel_events(ev_start, ev_stop), "mmv_set_kernel_events")


# ---- CSR SpMV, the stand-alone primitives of Sec. 4.1 and the un-fused compositions ------------------------

_ELEMS = {torch.int32: MMV_ELEM_I32, torch.float32: MMV_ELEM_F32}


def mmv_spmv_csr_workspace_bytes(n_rows: int, nnz: int) -> int:
    return int(load().mmv_spmv_csr_workspace_bytes(n_rows, nnz))


def mmv_spmv_csr(n_rows: int, n_cols: int, rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor,
                 x: torch.Tensor, y: torch.Tensor | None = None, variant: str = "mfma",
                 ws: torch.Tensor | None = None, stream=None, nnz: int | None = None) -> torch.Tensor:
    """y = A x for a CSR matrix (int32 row pointers and column indices, fp32 values)."""
    lib = load()
    nnz = val.numel() if nnz is None else nnz
    if y is None:
        y = torch.empty(n_rows, dtype=torch.float32, device=val.device)
    if ws is None:
        ws = workspace(mmv_spmv_csr_workspace_bytes(n_rows, nnz), val.device)
    st = lib.mmv_spmv_csr(n_rows, n_cols, nnz, _dev(rowptr, "rowptr"), _dev(col, "col"), _dev(val, "val"),
                          _dev(x, "x"), _dev(y, "y"), _VARIANTS[variant], _dev(ws, "ws"), ws.numel(),
                          _stream_ptr(stream))
    _check(st, "mmv_spmv_csr")
    return y


def mmv_scan(x: torch.Tensor, n: int | None = None, z: torch.Tensor | None = None, variant: str = "mfma",
             ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """Unsegmented inclusive scan; returns z (fp32 or int32)."""
    lib = load()
    n = x.numel() if n is None else n
    dt = _DTYPES[x.dtype]
    if z is None:
        z = torch.empty(n, dtype=_OUT_DTYPE[dt], device=x.device)
    if ws is None:
        ws = new_workspace(MMV_OP_SCAN, dt, MMV_FLAGS_PACKED32, n, x.device)
    st = lib.mmv_scan(_dev(x, "x"), n, _dev(z, "z"), dt, _VARIANTS[variant], _dev(ws, "ws"), ws.numel(),
                      _stream_ptr(stream))
    _check(st, "mmv_scan")
    return z


def mmv_compress(x: torch.Tensor | None, mask: torch.Tensor, n: int, out: torch.Tensor | None = None,
                 count: torch.Tensor | None = None, ws: torch.Tensor | None = None, stream=None):
    """COMPRESS of a 32-bit vector (or of the positions, x=None); returns (out, count)."""
    lib = load()
    ff = _flag_fmt(mask)
    if x is not None and x.element_size() != 4:
        raise MmvError("mmv_compress works on 32-bit elements")
    if out is None:
        out = torch.empty(max(n, 1), dtype=torch.int32 if x is None else x.dtype, device=mask.device)
    if count is None:
        count = torch.empty(1, dtype=torch.int64, device=mask.device)
    if ws is None:
        ws = new_workspace(MMV_OP_COMPRESS, MMV_I8_I32, ff, n, mask.device)
    st = lib.mmv_compress(None if x is None else _dev(x, "x"), _dev(mask, "mask"), n, _dev(out, "out"), out.numel(),
                          _dev(count, "count"), ff, _dev(ws, "ws"), ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_compress")
    return out, count


def mmv_diff(x: torch.Tensor, n: int | None = None, z: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """DIFF of an int32 or fp32 vector."""
    n = x.numel() if n is None else n
    if z is None:
        z = torch.empty(max(n, 1), dtype=x.dtype, device=x.device)
    _check(load().mmv_diff(_dev(x, "x"), n, _dev(z, "z"), _ELEMS[x.dtype], _stream_ptr(stream)), "mmv_diff")
    return z


def mmv_revert(xhat: torch.Tensor, fhat: torch.Tensor, w: torch.Tensor, n: int | None = None,
               nw: int | None = None, z: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """REVERT: xhat(i) - w(fhat(i) - 2) where fhat(i) >= 2; int32 or fp32, fhat int32."""
    n = xhat.numel() if n is None else n
    nw = w.numel() if nw is None else nw
    if fhat.dtype != torch.int32 or w.dtype != xhat.dtype:
        raise MmvError("fhat must be int32 and w must have the type of xhat")
    if z is None:
        z = torch.empty(max(n, 1), dtype=xhat.dtype, device=xhat.device)
    _check(load().mmv_revert(_dev(xhat, "xhat"), _dev(fhat, "fhat"), _dev(w, "w"), n, nw, _dev(z, "z"),
                             _ELEMS[xhat.dtype], _stream_ptr(stream)), "mmv_revert")
    return z


def mmv_segsum_scd(x: torch.Tensor, flags: torch.Tensor, n: int | None = None, out: torch.Tensor | None = None,
                   nseg: torch.Tensor | None = None, variant: str = "mfma", ws: torch.Tensor | None = None,
                   stream=None):
    """Segmented sum through the un-fused Algorithm SCD; returns (out, nseg) like mmv_segsum."""
    lib = load()
    n = x.numel() if n is None else n
    dt, ff = _DTYPES[x.dtype], _flag_fmt(flags)
    if out is None:
        out = torch.empty(max(n, 1), dtype=_OUT_DTYPE[dt], device=x.device)
    if nseg is None:
        nseg = torch.empty(1, dtype=torch.int64, device=x.device)
    if ws is None:
        ws = new_workspace(MMV_OP_SEGSUM_SCD, dt, ff, n, x.device)
    st = lib.mmv_segsum_scd(_dev(x, "x"), _dev(flags, "flags"), n, _dev(out, "out"), out.numel(), _dev(nseg, "nseg"),
                            dt, ff, _VARIANTS[variant], _dev(ws, "ws"), ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_segsum_scd")
    return out, nseg


def mmv_segscan_sscr(x: torch.Tensor, flags: torch.Tensor, n: int | None = None, z: torch.Tensor | None = None,
                     variant: str = "mfma", ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """Segmented scan through the un-fused Algorithm SSCR; returns z like mmv_segscan."""
    lib = load()
    n = x.numel() if n is None else n
    dt, ff = _DTYPES[x.dtype], _flag_fmt(flags)
    if z is None:
        z = torch.empty(n, dtype=_OUT_DTYPE[dt], device=x.device)
    if ws is None:
        ws = new_workspace(MMV_OP_SEGSCAN_SSCR, dt, ff, n, x.device)
    st = lib.mmv_segscan_sscr(_dev(x, "x"), _dev(flags, "flags"), n, _dev(z, "z"), dt, ff, _VARIANTS[variant],
                              _dev(ws, "ws"), ws.numel(), _stream_ptr(stream))
    _check(st, "mmv_segscan_sscr")
    return z
