"""GPU parity of the COO SpMV path against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import dev

pytestmark = pytest.mark.gpu
TILE = 65536          # largest workgroup tile (int8); other types and short inputs use smaller ones


def run_spmv(n_rows, n_cols, row, col, val, x, variant="mfma"):
    nnz = len(val)
    pad = lambda a: a if len(a) else np.zeros(1, dtype=a.dtype)
    ws = B.new_workspace(B.MMV_OP_SPMV_COO, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, nnz)
    y = torch.full((max(n_rows, 1),), 123.0, dtype=torch.float32, device="cuda")
    rt, ct, vt = dev(pad(row)), dev(pad(col)), dev(pad(val))
    lib = B.load()
    st = lib.mmv_spmv_coo(n_rows, n_cols, nnz, rt.data_ptr(), ct.data_ptr(), vt.data_ptr(), dev(x).data_ptr(),
                          y.data_ptr(), B._VARIANTS[variant], ws.data_ptr(), ws.numel(), B._stream_ptr(None))
    assert st == 0
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 0
    return y.cpu().numpy()[:n_rows]


def check_spmv(y, n_rows, n_cols, row, col, val, x, tol=1e-4):
    ref = oracle.spmv_coo(n_rows, n_cols, row, col, val, x)
    A = oracle.spmv_coo(n_rows, n_cols, row, col, np.abs(val), np.abs(x))     # sum |val * x| per row
    err = np.abs(y.astype(np.float64) - ref)
    bad = err > tol * np.maximum(A, 1.0)
    assert not bad.any(), "row %d: got %r ref %r" % (int(np.argmax(bad)), y[int(np.argmax(bad))],
                                                     ref[int(np.argmax(bad))])
    counts = np.bincount(row, minlength=n_rows)
    assert (y[counts == 0] == 0.0).all()                # rows without entries are exactly zero
    return float((err / np.maximum(A, 1.0)).max())


@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
def test_spmv_small_shapes(variant):
    for n_rows, n_cols, nnz, cap, seed in [(1, 1, 1, 1, 1), (5, 7, 20, 7, 2), (300, 257, 1500, 64, 21),
                                           (1000, 999, 40_000, 512, 3), (4096, 4096, 3 * TILE + 11, 4096, 4)]:
        row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, nnz, cap=cap, seed=seed)
        if len(val) == 0:
            continue
        print("spmv", variant, n_rows, n_cols, len(val), flush=True)
        check_spmv(run_spmv(n_rows, n_cols, row, col, val, x, variant), n_rows, n_cols, row, col, val, x)


def test_spmv_one_row_spanning_many_tiles_and_trailing_empty_rows():
    rng = np.random.default_rng(5)
    nnz = 9 * TILE + 17
    row = np.full(nnz, 3, dtype=np.int32)
    row[:10] = 1
    row[-5:] = 6
    col = rng.integers(0, 50, size=nnz, dtype=np.int32)
    val = rng.standard_normal(nnz, dtype=np.float32)
    x = rng.standard_normal(50, dtype=np.float32)
    check_spmv(run_spmv(10, 50, row, col, val, x), 10, 50, row, col, val, x)


def test_spmv_integer_valued_is_exact_and_duplicates_add():
    rng = np.random.default_rng(6)
    nnz = 30_000
    row = np.sort(rng.integers(0, 2000, size=nnz)).astype(np.int32)
    col = rng.integers(0, 8, size=nnz).astype(np.int32)          # many duplicate (row, col) pairs
    val = rng.integers(-9, 10, size=nnz).astype(np.float32)
    x = rng.integers(-9, 10, size=8).astype(np.float32)
    y = run_spmv(2000, 8, row, col, val, x)
    assert np.array_equal(y.astype(np.float64), oracle.spmv_coo(2000, 8, row, col, val, x))


def test_spmv_no_entries():
    y = run_spmv(100, 10, np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                 np.ones(10, np.float32))
    assert (y == 0).all()


@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
@pytest.mark.parametrize("log2rows", [14, 20])
def test_workload4_spmv_zipf(log2rows, variant):
    n = 1 << log2rows
    row, col, val, x = W.spmv_coo_zipf(n, n, 32 * n)
    y = run_spmv(n, n, row, col, val, x, variant)
    worst = check_spmv(y, n, n, row, col, val, x)
    print("workload 4 rows=2^%d nnz=%d %s: worst |err|/max(A,1) = %.3g" % (log2rows, len(val), variant, worst))
