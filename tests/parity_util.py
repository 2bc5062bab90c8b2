"""Helpers for the GPU parity tests: move inputs to the GPU, call the C-ABI
through the binding, and compare with the CPU oracle.

Comparison rules
* integers (int8 -> int32, and bytes under exclusive or): bit-exact on every element and on the segment count.
* floating point: |got - ref| <= tol * max(A_i, 1) for every element, where ref
  is the fp64-accumulated oracle, A_i the segmented inclusive scan of |x| in
  fp64 (A_i >= |ref_i|; the classical summation bound is relative to it) and 1
  is the value scale of the workloads (U(-1,1), N(0,1)).  tol = 1e-4 for fp32
  inputs, 2e-3 for fp16 inputs, 1e-2 for bf16 inputs, fp32 accumulation.
  On a long segment A_i outgrows the result itself (a segment of 2^28 values from U(-1,1) reaches A_i = 1.3e8
  while |ref| stays near 1e4), so that gate alone could be passed there by a wrong answer.  Two more
  assertions stand beside it:
  - margin: the worst |got - ref| / max(A_i, 1) over the vector stays below MARGIN = 2e-5, ten times the
    worst ever measured (the revert subtracts two row prefixes of at most 32 terms, 2 * 32 * 2^-24 = 4e-6
    of the row's sum of |x|; carries add one rounding per level);
  - per segment: max |got - ref| over the segment <= tol * max(max |ref| over the segment, 1), a bound
    relative to the result's own size, which an all-zero or shifted output cannot meet on any segment whose
    values exceed the floor.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W

TOL = {np.dtype(np.float32): 1e-4, np.dtype(np.float16): 2e-3, "bf16": 1e-2}


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def packed_dev(f_u8: np.ndarray) -> torch.Tensor:
    words = W.pack_flags(f_u8)
    if words.shape[0] == 0:
        words = np.zeros(1, dtype="<u4")
    return torch.from_numpy(words.view(np.int32).copy()).cuda()


def flags_dev(f_u8: np.ndarray, packed: bool) -> torch.Tensor:
    return packed_dev(f_u8) if packed else dev(f_u8.astype(np.uint8))


def run_segscan(x: np.ndarray, f: np.ndarray, variant="mfma", packed=True, xt: torch.Tensor | None = None):
    xt = dev(x) if xt is None else xt
    ft = flags_dev(f, packed)
    n = x.shape[0]
    dt = B._DTYPES[xt.dtype]
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, dt, B._flag_fmt(ft), n)
    z = B.mmv_segscan(xt, ft, n=n, variant=variant, ws=ws)
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 0
    return z.cpu().numpy()


def run_segsum(x: np.ndarray, f: np.ndarray, variant="mfma", packed=True, xt: torch.Tensor | None = None,
               out_capacity: int | None = None):
    xt = dev(x) if xt is None else xt
    ft = flags_dev(f, packed)
    n = x.shape[0]
    dt = B._DTYPES[xt.dtype]
    ws = B.new_workspace(B.MMV_OP_SEGSUM, dt, B._flag_fmt(ft), n)
    cap = max(n, 1) if out_capacity is None else out_capacity
    out = torch.full((max(cap, 1),), -77, dtype=B._OUT_DTYPE[dt], device="cuda")
    nseg = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    B.mmv_segsum(xt, ft, n=n, out=out, nseg=nseg, variant=variant, ws=ws)
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 0
    return out.cpu().numpy(), int(nseg.item())


def abs_scan(x: np.ndarray, f: np.ndarray) -> np.ndarray:
    """A_i: segmented inclusive scan of |x| in fp64 (through the oracle)."""
    return oracle.segscan(np.abs(x.astype(np.float64)), f)


MARGIN = 2e-5


def segment_starts(f: np.ndarray) -> np.ndarray:
    """Positions that open a segment (position 0 always does)."""
    st = np.flatnonzero(np.asarray(f) != 0)
    return st if len(st) and st[0] == 0 else np.concatenate([[0], st])


def check_scan(got: np.ndarray, x: np.ndarray, f: np.ndarray, tol=None, chunk: int = 1 << 24, margin: float = MARGIN):
    ref = oracle.segscan(x, f)
    if x.dtype in (np.int8, np.uint8):      # int8 sums and bytes under xor: exact
        assert got.dtype == np.int32
        assert np.array_equal(got, ref), _first_diff(got, ref)
        return 0.0
    tol = TOL[x.dtype] if tol is None else tol
    A = abs_scan(x, f)
    worst = 0.0
    err = np.empty(len(ref), dtype=np.float64)
    for a in range(0, len(ref), chunk):
        b = min(len(ref), a + chunk)
        err[a:b] = np.abs(got[a:b].astype(np.float64) - ref[a:b])
        bound = tol * np.maximum(A[a:b], 1.0)
        bad = ~(err[a:b] <= bound)              # (a NaN is bad)
        assert not bad.any(), "element %d: got %r ref %r A %r" % (
            a + int(np.argmax(bad)), got[a + int(np.argmax(bad))], ref[a + int(np.argmax(bad))],
            A[a + int(np.argmax(bad))])
        worst = max(worst, float((err[a:b] / np.maximum(A[a:b], 1.0)).max()))
    assert worst <= margin, "worst |err| / max(A, 1) = %.3g exceeds the measured margin %.3g" % (worst, margin)
    del A
    if len(ref):
        st = segment_starts(f)
        seg_err = np.maximum.reduceat(err, st)
        np.abs(ref, out=ref)
        seg_ref = np.maximum.reduceat(ref, st)
        bad = ~(seg_err <= tol * np.maximum(seg_ref, 1.0))
        assert not bad.any(), "segment %d (starts at %d): max |err| %r, max |ref| %r" % (
            int(np.argmax(bad)), int(st[int(np.argmax(bad))]), seg_err[int(np.argmax(bad))], seg_ref[int(np.argmax(bad))])
    return worst


def check_sum(got: np.ndarray, nseg: int, x: np.ndarray, f: np.ndarray, tol=None, margin: float | None = None):
    margin = MARGIN if margin is None else margin
    ref = oracle.segsum(x, f)
    assert nseg == len(ref), (nseg, len(ref))
    got = got[:nseg]
    if x.dtype in (np.int8, np.uint8):
        assert np.array_equal(got, ref), _first_diff(got, ref)
        return 0.0
    tol = TOL[x.dtype] if tol is None else tol
    A = oracle.segsum(np.abs(x.astype(np.float64)), f)
    err = np.abs(got.astype(np.float64) - ref)
    bad = ~(err <= tol * np.maximum(A, 1.0))
    assert not bad.any(), "segment %d: got %r ref %r A %r" % (int(np.argmax(bad)), got[int(np.argmax(bad))],
                                                              ref[int(np.argmax(bad))], A[int(np.argmax(bad))])
    worst = float((err / np.maximum(A, 1.0)).max()) if len(ref) else 0.0
    assert worst <= margin, "worst |err| / max(A, 1) = %.3g exceeds the measured margin %.3g" % (worst, margin)
    if len(ref):
        # relative to the size the running sum reaches inside the segment (the sum itself may cancel to zero)
        seg_ref = np.maximum.reduceat(np.abs(oracle.segscan(x, f)), segment_starts(f))
        bad = ~(err <= tol * np.maximum(seg_ref, 1.0))
        assert not bad.any(), "segment %d: |err| %r, max |running sum| %r" % (
            int(np.argmax(bad)), err[int(np.argmax(bad))], seg_ref[int(np.argmax(bad))])
    return worst


def _first_diff(got, ref):
    d = np.flatnonzero(got != ref)
    if len(d) == 0:
        return "shapes %r %r" % (got.shape, ref.shape)
    i = int(d[0])
    return "first difference at %d of %d (%d differ): got %r ref %r" % (i, len(ref), len(d), got[i - 2:i + 3],
                                                                       ref[i - 2:i + 3])


def random_values(rng, n: int, dtype) -> np.ndarray:
    if dtype == np.int8:
        return rng.integers(-128, 128, size=n, dtype=np.int8)
    if dtype == np.uint8:
        return rng.integers(0, 256, size=n, dtype=np.uint8)
    if dtype == np.float16:
        return rng.standard_normal(n).astype(np.float16)
    return (rng.random(n, dtype=np.float32) * 2 - 1).astype(np.float32)
