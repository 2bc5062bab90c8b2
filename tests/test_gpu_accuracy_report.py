"""What speculation costs numerically: besides the gate of the parity tests (|err| <= tol * max(A_i, 1)), the
strict relative error |err| / A_i (A_i the segmented scan of |x|, so a segment that starts with tiny values
after large ones in the same row of 32 shows the cancellation of the revert), the number of elements whose
strict error exceeds the tolerance, and the normwise error max|err| / max|ref| -- for both variants (matrix
cores / shuffles only), and how many segment starts do not hold their own value bit for bit (with 16-bit inputs a
start inside a row is x-bar(j) - x-bar(j-1); with fp32 inputs the kernel stores the input itself there); printed as a
table (run with -s).  The gate, the normwise error and, for fp32 inputs, "every start holds its input" are asserted."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import workloads as W
from parity_util import TOL, abs_scan, run_segscan, run_segsum

pytestmark = pytest.mark.gpu


def _cases():
    x, f = W.scan_sum_f32_bernoulli()
    yield "workload 1  fp32 U(-1,1) n=2^16 Bernoulli(1/64)", x, f
    x, f = W.segsum_f16_geometric(1 << 20)
    yield "workload 2  fp16 N(0,1) n=2^20 Geometric(1/32)", x, f
    x, f = W.stress_f32_three_regimes(1 << 22)
    yield "workload 5  fp32 U(-1,1) n=2^22 three regimes", x, f
    x8, f = W.segscan_i8_uniform_len(1 << 22)
    rng = np.random.default_rng(2390660)
    yield "fp32 N(0,1) n=2^22 lengths U{1..4096}", rng.standard_normal(len(f), dtype=np.float32), f
    f = W.uniform_density_flags(1 << 20, 0.01, 2390661)
    # values of mixed magnitude: short segments of small values right after large ones
    x = (rng.standard_normal(1 << 20) * 10.0 ** rng.integers(-4, 1, size=1 << 20)).astype(np.float32)
    yield "fp32 N(0,1) * 10^U{-4..0} n=2^20 density 1 %", x, f


def test_error_report_scan_and_sum():
    rows = []
    for name, x, f in _cases():
        tol = TOL[x.dtype]
        ref = oracle.segscan(x, f)
        A = abs_scan(x, f)
        ends = np.flatnonzero(np.append(f[1:] != 0, True))
        for variant in ("mfma", "shuffle"):
            z = run_segscan(x, f, variant).astype(np.float64)
            err = np.abs(z - ref)
            gate = float((err / np.maximum(A, 1.0)).max())
            strict = np.where(A > 0, err / np.where(A > 0, A, 1.0), 0.0)
            normwise = float(err.max() / np.abs(ref).max())
            out, nseg = run_segsum(x, f, variant)
            serr = np.abs(out[:nseg].astype(np.float64) - ref[ends])
            sgate = float((serr / np.maximum(A[ends], 1.0)).max())
            starts = np.flatnonzero(f != 0)
            inexact = int((z[starts] != x[starts].astype(np.float64)).sum())   # a start is x-bar(j) - x-bar(j-1), not x(j)
            rows.append((name, variant, gate, float(strict.max()), int((strict > tol).sum()), normwise, sgate,
                         "%d of %d" % (inexact, len(starts))))
            assert gate <= tol and sgate <= tol and normwise <= tol, rows[-1]
            if x.dtype == np.float32:
                assert inexact == 0, rows[-1]
    print()
    print("%-52s %-8s %10s %10s %9s %10s %10s  %s" % ("scan inputs", "variant", "gate", "strict", "> tol", "normwise",
                                                       "sum gate", "starts not bit-equal to x"))
    for r in rows:
        print("%-52s %-8s %10.3g %10.3g %9d %10.3g %10.3g  %s" % r)
