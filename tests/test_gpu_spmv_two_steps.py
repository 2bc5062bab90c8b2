"""GPU tests of SpMV in two steps (mmv_spmv_coo_prepare / _run, mmv_spmv_csr_prepare / _run): the plan made once
from the index arrays, then several products with it.  Results must agree with the fp64 oracle and, to the last
bits (the order in which the carries of rows that cross tile borders are added may differ from run to run), with
the one-step calls; on integer-valued inputs, where every sum is exact, they must be bit-identical."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import dev
from test_gpu_csr import check_csr
from test_gpu_spmv import check_spmv

pytestmark = pytest.mark.gpu
TILE = 16384

SHAPES = [(1, 1, 1, 1, 1), (5, 7, 20, 7, 2), (300, 257, 1500, 64, 21), (1000, 999, 40_000, 512, 3),
          (4096, 4096, 3 * TILE + 11, 4096, 4), (70_000, 50_000, 20 * TILE + 5, 3000, 5),
          (1 << 18, 1 << 18, 2200 * TILE + 77, 100_000, 6)]      # the last one: more than 2048 tiles, tickets, count prefix


@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
def test_coo_two_steps_equal_one_step_and_the_oracle(variant):
    rng = np.random.default_rng(81)
    for n_rows, n_cols, nnz, cap, seed in SHAPES:
        row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, nnz, cap=cap, seed=seed)
        if len(val) == 0:
            continue
        print("coo two steps", variant, n_rows, n_cols, len(val), flush=True)
        rt, ct, vt = dev(row), dev(col), dev(val)
        ws = B.mmv_spmv_coo_prepare(n_rows, n_cols, rt, ct)
        one = B.mmv_spmv_coo(n_rows, n_cols, rt, ct, vt, dev(x), variant=variant)
        for rep in range(3):                      # the plan serves several products, with new x (and new values)
            xr = x if rep == 0 else rng.standard_normal(n_cols).astype(np.float32)
            vr = val if rep < 2 else rng.standard_normal(len(val)).astype(np.float32)
            y = torch.full((n_rows,), 123.0, dtype=torch.float32, device="cuda")
            B.mmv_spmv_coo_run(n_rows, n_cols, rt, ct, dev(vr), dev(xr), ws, y=y, variant=variant)
            torch.cuda.synchronize()
            assert B.mmv_workspace_status(ws) == 0
            got = y.cpu().numpy()
            if rep == 0:
                assert np.allclose(got, one.cpu().numpy(), rtol=1e-5, atol=1e-5)
            check_spmv(got, n_rows, n_cols, row, col, vr, xr)


@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
def test_csr_two_steps_equal_one_step_and_the_oracle(variant):
    rng = np.random.default_rng(82)
    for n_rows, n_cols, nnz, cap, seed in SHAPES:
        row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, nnz, cap=cap, seed=seed)
        if len(val) == 0:
            continue
        rowptr = W.csr_rowptr(row, n_rows)
        print("csr two steps", variant, n_rows, n_cols, len(val), flush=True)
        rpt, ct, vt = dev(rowptr), dev(col), dev(val)
        ws = B.mmv_spmv_csr_prepare(n_rows, n_cols, rpt, ct)
        one = B.mmv_spmv_csr(n_rows, n_cols, rpt, ct, vt, dev(x), variant=variant)
        for rep in range(3):
            xr = x if rep == 0 else rng.standard_normal(n_cols).astype(np.float32)
            vr = val if rep < 2 else rng.standard_normal(len(val)).astype(np.float32)
            y = torch.full((n_rows,), 123.0, dtype=torch.float32, device="cuda")
            B.mmv_spmv_csr_run(n_rows, n_cols, rpt, ct, dev(vr), dev(xr), ws, y=y, variant=variant)
            torch.cuda.synchronize()
            assert B.mmv_workspace_status(ws) == 0
            got = y.cpu().numpy()
            if rep == 0:
                assert np.allclose(got, one.cpu().numpy(), rtol=1e-5, atol=1e-5)
            check_csr(got, n_rows, n_cols, rowptr, col, vr, xr)


def test_two_steps_on_integer_valued_inputs_are_bit_identical_to_one_step():
    n_rows, n_cols = 1 << 18, 1 << 18
    row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, 2200 * TILE + 77, cap=100_000, seed=6)
    rng = np.random.default_rng(83)
    val = rng.integers(-4, 5, size=len(val)).astype(np.float32)
    x = rng.integers(-4, 5, size=n_cols).astype(np.float32)
    rowptr = W.csr_rowptr(row, n_rows)
    rt, rpt, ct, vt, xt = dev(row), dev(rowptr), dev(col), dev(val), dev(x)
    ref = oracle.spmv_coo(n_rows, n_cols, row, col, val, x).astype(np.float32)
    ws = B.mmv_spmv_coo_prepare(n_rows, n_cols, rt, ct)
    wc = B.mmv_spmv_csr_prepare(n_rows, n_cols, rpt, ct)
    for rep in range(2):
        assert np.array_equal(B.mmv_spmv_coo_run(n_rows, n_cols, rt, ct, vt, xt, ws).cpu().numpy(), ref)
        assert np.array_equal(B.mmv_spmv_csr_run(n_rows, n_cols, rpt, ct, vt, xt, wc).cpu().numpy(), ref)
    assert np.array_equal(B.mmv_spmv_coo(n_rows, n_cols, rt, ct, vt, xt).cpu().numpy(), ref)
    assert np.array_equal(B.mmv_spmv_csr(n_rows, n_cols, rpt, ct, vt, xt).cpu().numpy(), ref)


def test_csr_two_steps_on_a_blocked_matrix_without_empty_rows():
    n = 1 << 14
    rowptr, col, val, x = W.blocked_sparse_attention(n, block=64, n_random=4)
    rpt, ct = dev(rowptr), dev(col)
    ws = B.mmv_spmv_csr_prepare(n, n, rpt, ct)
    for rep in range(2):
        y = B.mmv_spmv_csr_run(n, n, rpt, ct, dev(val), dev(x), ws)
        torch.cuda.synchronize()
        assert B.mmv_workspace_status(ws) == 0
        check_csr(y.cpu().numpy(), n, n, rowptr, col, val, x)


def test_run_on_a_workspace_that_was_not_prepared_gives_zeros_and_a_status():
    """A workspace full of ones (no plan, flag words and row map that point anywhere), one prepared for another
    shape, and one whose plan another call has overwritten: y comes back as zeros, the status word says 2, and
    nothing is read or written out of bounds (the product kernel leaves at once)."""
    n_rows, n_cols = 5000, 4000
    row, col, val, x = W.spmv_coo_zipf(n_rows, n_cols, 5 * TILE + 3, cap=900, seed=9)
    rowptr = W.csr_rowptr(row, n_rows)
    rt, rpt, ct, vt, xt = dev(row), dev(rowptr), dev(col), dev(val), dev(x)
    nnz = len(val)
    for kind in ("coo", "csr"):
        nbytes = (B.mmv_workspace_bytes(B.MMV_OP_SPMV_COO, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, nnz) if kind == "coo"
                  else B.mmv_spmv_csr_workspace_bytes(n_rows, nnz))
        garbage = torch.full((nbytes,), 1, dtype=torch.uint8, device="cuda")
        rpt1 = dev(np.concatenate([rowptr, rowptr[-1:]]))                             # one more row, without entries
        other = (B.mmv_spmv_coo_prepare(n_rows + 1, n_cols, rt, ct) if kind == "coo"
                 else B.mmv_spmv_csr_prepare(n_rows + 1, n_cols, rpt1, ct))          # a plan for another shape
        for ws in (garbage, other):
            if ws.numel() < nbytes:
                continue
            y = torch.full((n_rows,), 123.0, dtype=torch.float32, device="cuda")
            if kind == "coo":
                B.mmv_spmv_coo_run(n_rows, n_cols, rt, ct, vt, xt, ws, y=y)
            else:
                B.mmv_spmv_csr_run(n_rows, n_cols, rpt, ct, vt, xt, ws, y=y)
            torch.cuda.synchronize()
            assert B.mmv_workspace_status(ws) == 2
            assert (y.cpu().numpy() == 0).all()
    # a good plan still works afterwards, and the one-step call on the same workspace replaces it
    ws = B.mmv_spmv_coo_prepare(n_rows, n_cols, rt, ct)
    y = B.mmv_spmv_coo_run(n_rows, n_cols, rt, ct, vt, xt, ws)
    check_spmv(y.cpu().numpy(), n_rows, n_cols, row, col, val, x)
    B.mmv_segscan(torch.zeros(1 << 16, dtype=torch.int8, device="cuda"), torch.zeros(1 << 11, dtype=torch.int32, device="cuda"),
                  n=1 << 16, ws=ws)                                                   # another call takes the workspace
    y = torch.full((n_rows,), 123.0, dtype=torch.float32, device="cuda")
    B.mmv_spmv_coo_run(n_rows, n_cols, rt, ct, vt, xt, ws, y=y)
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 2 and (y.cpu().numpy() == 0).all()


def test_two_steps_no_entries_and_no_rows():
    e32, ef = torch.zeros(4, dtype=torch.int32, device="cuda"), torch.zeros(4, dtype=torch.float32, device="cuda")
    lib = B.load()
    ws = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    y = torch.full((17,), 5.0, dtype=torch.float32, device="cuda")
    assert lib.mmv_spmv_coo_prepare(17, 5, 0, None, None, None, 0, None) == 0
    assert lib.mmv_spmv_coo_run(17, 5, 0, None, None, None, None, y.data_ptr(), 0, None, 0, None) == 0
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == 0).all()
    y.fill_(5.0)
    assert lib.mmv_spmv_csr_prepare(17, 5, 0, None, None, None, 0, None) == 0
    assert lib.mmv_spmv_csr_run(17, 5, 0, None, None, None, None, y.data_ptr(), 0, None, 0, None) == 0
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == 0).all()
    assert lib.mmv_spmv_coo_run(0, 5, 0, None, None, None, None, None, 0, None, 0, None) == 0
