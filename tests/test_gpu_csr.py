"""GPU parity of the CSR SpMV entry point against the fp64 oracle (y = A x over the entries of
each row), on Zipf row lengths with empty rows and on the blocked sparse-attention matrices."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import dev

pytestmark = pytest.mark.gpu
TILE = 16384          # workgroup tile of the SpMV kernel


def run_csr(n_rows, n_cols, rowptr, col, val, x, variant="mfma"):
    pad = lambda a: a if len(a) else np.zeros(1, dtype=a.dtype)
    y = torch.full((max(n_rows, 1),), 123.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(256, B.mmv_spmv_csr_workspace_bytes(n_rows, len(val))), dtype=torch.uint8, device="cuda")
    B.mmv_spmv_csr(n_rows, n_cols, dev(rowptr), dev(pad(col)), dev(pad(val)), dev(x), y=y, variant=variant, ws=ws,
                   nnz=len(val))
    torch.cuda.synchronize()
    if len(val):
        assert B.mmv_workspace_status(ws) == 0
    return y.cpu().numpy()[:n_rows]


def check_csr(y, n_rows, n_cols, rowptr, col, val, x, tol=1e-4):
    ref = oracle.spmv_csr(n_rows, n_cols, rowptr, col, val, x)
    A = oracle.spmv_csr(n_rows, n_cols, rowptr, col, np.abs(val), np.abs(x))
    err = np.abs(y.astype(np.float64) - ref)
    bad = err > tol * np.maximum(A, 1.0)
    assert not bad.any(), "row %d: got %r ref %r" % (int(np.argmax(bad)), y[int(np.argmax(bad))], ref[int(np.argmax(bad))])
    assert (y[np.diff(rowptr) == 0] == 0.0).all()       # rows without entries are exactly zero
    return float((err / np.maximum(A, 1.0)).max())


@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
def test_csr_small_shapes(variant):
    for n_rows, n_cols, nnz, cap, seed in [(1, 1, 1, 1, 1), (5, 7, 20, 7, 2), (300, 257, 1500, 64, 21),
                                           (1000, 999, 40_000, 512, 3), (4096, 4096, 3 * TILE + 11, 4096, 4),
                                           (70_000, 50_000, 20 * TILE + 5, 3000, 5)]:
        row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, nnz, cap=cap, seed=seed)
        rowptr = W.csr_rowptr(row, n_rows)
        y = run_csr(n_rows, n_cols, rowptr, col, val, x, variant)
        check_csr(y, n_rows, n_cols, rowptr, col, val, x)


def test_csr_leading_trailing_empty_rows_and_one_long_row():
    n_rows, n_cols = 1000, 64
    nnz = 5 * TILE + 123
    rng = np.random.default_rng(71)
    rowptr = np.zeros(n_rows + 1, dtype=np.int32)
    rowptr[501:] = nnz                                    # rows 0..499 empty, row 500 holds everything
    col = rng.integers(0, n_cols, size=nnz, dtype=np.int32)
    val = rng.standard_normal(nnz, dtype=np.float32)
    x = rng.standard_normal(n_cols, dtype=np.float32)
    y = run_csr(n_rows, n_cols, rowptr, col, val, x)
    check_csr(y, n_rows, n_cols, rowptr, col, val, x)
    assert y[500] != 0 and (np.delete(y, 500) == 0).all()


def test_csr_integer_valued_is_exact_and_equals_coo():
    n_rows = n_cols = 3000
    row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, 200_000, cap=900, seed=72)
    rng = np.random.default_rng(73)
    val = rng.integers(-4, 5, size=len(val)).astype(np.float32)
    x = rng.integers(-4, 5, size=n_cols).astype(np.float32)
    rowptr = W.csr_rowptr(row, n_rows)
    y = run_csr(n_rows, n_cols, rowptr, col, val, x)
    assert np.array_equal(y.astype(np.float64), oracle.spmv_csr(n_rows, n_cols, rowptr, col, val, x))
    yc = B.mmv_spmv_coo(n_rows, n_cols, dev(row), dev(col), dev(val), dev(x)).cpu().numpy()
    assert np.array_equal(y, yc)


def test_csr_no_entries():
    y = run_csr(17, 5, np.zeros(18, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32),
                np.ones(5, dtype=np.float32))
    assert (y == 0).all()


@pytest.mark.parametrize("block,n_random", [(2, 2), (4, 8), (16, 4), (64, 2)])
def test_csr_blocked_sparse_attention(block, n_random):
    n = 1 << 13 if block < 16 else 1 << 14
    rowptr, col, val, x = W.blocked_sparse_attention(n, block=block, n_random=n_random)
    y = run_csr(n, n, rowptr, col, val, x)
    worst = check_csr(y, n, n, rowptr, col, val, x)
    print("sparse attention n=%d b-%d_r-%d nnz=%d: worst |err|/max(A,1) = %.3g" % (n, block, n_random, len(val), worst))


def test_csr_blocked_sparse_attention_full_size():
    """The paper's size, 65,536 x 65,536, standard block size 64 with 2 random blocks (37.6 M non-zeros)."""
    n = 1 << 16
    rowptr, col, val, x = W.blocked_sparse_attention(n, block=64, n_random=2)
    y = run_csr(n, n, rowptr, col, val, x)
    check_csr(y, n, n, rowptr, col, val, x)


def test_csr_one_workspace_for_matrices_with_and_without_empty_rows():
    """A matrix none of whose rows is empty takes a path of its own (segment k is row k, no row map);
    the same workspace serves both kinds in turn, so the mark of the earlier call must not survive."""
    n = 5000
    rng = np.random.default_rng(74)
    lengths = rng.integers(1, 40, size=n)
    dense = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)          # every row has entries
    holes = lengths.copy()
    holes[rng.random(n) < 0.3] = 0
    holes[0] = holes[-1] = 0
    sparse = np.concatenate([[0], np.cumsum(holes)]).astype(np.int32)           # 30 % of the rows empty
    x = rng.integers(-4, 5, size=n).astype(np.float32)
    mats = []
    for rowptr in (dense, sparse):
        nnz = int(rowptr[-1])
        mats.append((rowptr, rng.integers(0, n, size=nnz, dtype=np.int32), rng.integers(-4, 5, size=nnz).astype(np.float32)))
    ws = torch.empty(max(B.mmv_spmv_csr_workspace_bytes(n, len(m[2])) for m in mats), dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    for which in (0, 1, 0, 0, 1, 1, 0):
        rowptr, col, val = mats[which]
        y.fill_(77.0)
        B.mmv_spmv_csr(n, n, dev(rowptr), dev(col), dev(val), dev(x), y=y, ws=ws)
        torch.cuda.synchronize()
        assert B.mmv_workspace_status(ws) == 0
        assert np.array_equal(y.cpu().numpy().astype(np.float64), oracle.spmv_csr(n, n, rowptr, col, val, x)), which


def test_gather_reference_sums_the_product_vector():
    """The random-access reference of the benchmark report: its partial sums add up to sum(val * x[col])
    (integer-valued data, so the check is exact); the entries past the last multiple of four are left out."""
    rng = np.random.default_rng(2390611)
    nnz, n_cols = 100003, 4099
    val = rng.integers(-3, 4, size=nnz).astype(np.float32)
    col = rng.integers(0, n_cols, size=nnz, dtype=np.int32)
    x = rng.integers(-3, 4, size=n_cols).astype(np.float32)
    part = torch.empty(B.GATHER_REFERENCE_PARTIALS, dtype=torch.float32, device="cuda")
    B.mmv_gather_reference(dev(val), dev(col), dev(x), part)
    torch.cuda.synchronize()
    used = nnz - nnz % 4
    want = float(np.dot(val[:used].astype(np.float64), x[col[:used]].astype(np.float64)))
    assert float(part.double().sum().item()) == want
