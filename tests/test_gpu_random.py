"""Randomised differential test: a few hundred seeded cases with random length, element type, flag
density and format, variant and entry point, each compared with the CPU oracle under the usual
rule (integers bit-exact, floats within tol * max(A, 1)); plus HIP-graph replays of the entry points
that enqueue several kernels."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import check_scan, check_sum, dev, flags_dev, packed_dev, random_values, run_segscan, run_segsum

pytestmark = pytest.mark.gpu


def _random_flags(rng, n):
    kind = rng.integers(0, 5)
    if kind == 0:
        f = np.zeros(n, dtype=np.uint8)                                   # one segment
    elif kind == 1:
        f = np.ones(n, dtype=np.uint8)                                    # every element its own segment
    elif kind == 2:
        f = (rng.random(n) < 10.0 ** rng.uniform(-4, 0)).astype(np.uint8)  # uniform density 0.01 % .. 100 %
    elif kind == 3:
        lengths = W.draw_lengths_until(rng, max(n, 1), lambda r, k: r.geometric(1.0 / r.integers(2, 5000), size=k))
        f = W.flags_from_lengths(lengths, n)
    else:                                                                 # dense start, one long run, dense end
        f = np.zeros(n, dtype=np.uint8)
        a, b = sorted(rng.integers(0, n + 1, size=2))
        f[:a] = rng.random(a) < 0.5
        f[b:] = rng.random(n - b) < 0.5
    if n and rng.random() < 0.5:
        f[0] = 0                                                          # position 0 opens a segment anyway
    return f


def test_random_cases_against_the_oracle():
    rng = np.random.default_rng(20260623)
    dtypes = [np.int8, np.int8, np.float16, np.float32]
    for case in range(240):
        n = int(rng.choice([rng.integers(1, 200), rng.integers(200, 40_000), rng.integers(40_000, 600_000)]))
        dtype = dtypes[rng.integers(0, len(dtypes))]
        variant = ["mfma", "shuffle"][rng.integers(0, 2)]
        packed = bool(rng.integers(0, 2))
        x = random_values(rng, n, dtype)
        f = _random_flags(rng, n)
        what = int(rng.integers(0, 5))
        tag = (case, n, np.dtype(dtype).name, variant, packed, what)
        if what == 0:
            check_scan(run_segscan(x, f, variant, packed), x, f)
        elif what == 1:
            out, nseg = run_segsum(x, f, variant, packed)
            check_sum(out, nseg, x, f)
        elif what == 2:
            z = B.mmv_scan(dev(x), n=n, variant=variant)
            torch.cuda.synchronize()
            check_scan(z.cpu().numpy(), x, np.zeros(n, dtype=np.uint8))
        elif what == 3 and dtype == np.int8:
            z = B.mmv_segscan_sscr(dev(x), flags_dev(f, packed), n=n, variant=variant)
            torch.cuda.synchronize()
            assert np.array_equal(z.cpu().numpy(), oracle.segscan(x, f)), tag
            ref = oracle.segsum(x, f)
            out, nseg = B.mmv_segsum_scd(dev(x), flags_dev(f, packed), n=n, variant=variant)
            torch.cuda.synchronize()
            assert int(nseg.item()) == len(ref) and np.array_equal(out.cpu().numpy()[:len(ref)], ref), tag
        else:
            m = _random_flags(rng, n)
            v = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
            out, count = B.mmv_compress(dev(v), flags_dev(m, packed), n)
            torch.cuda.synchronize()
            ref = oracle.compress(v, m)
            assert int(count.item()) == len(ref) and np.array_equal(out.cpu().numpy()[:len(ref)], ref), tag


def test_random_cases_longer_than_one_round_of_workgroups():
    """Vectors that need more tiles than the device holds workgroups at once take their tiles by atomic
    ticket and end in short tiles; shorter ones (all cases above) take tile = workgroup index."""
    rng = np.random.default_rng(20260625)
    one_round = {np.int8: 512 * 65536, np.float16: 512 * 32768, np.float32: 512 * 16384}
    for case in range(12):
        dtype = [np.int8, np.float16, np.float32][case % 3]
        dt = B._DTYPES[torch.from_numpy(np.zeros(1, dtype)).dtype]
        assert one_round[dtype] == 512 * B.mmv_tile_elems(B.MMV_OP_SEGSCAN, dt, 1 << 40)
        what = (case // 3) % 3
        # the scan without a flag vector has tiles of its own length (longer for 16-bit inputs)
        fits = 512 * B.mmv_tile_elems(B.MMV_OP_SCAN, dt, 1 << 40) if what == 2 else one_round[dtype]
        n = fits + int(rng.integers(1, 3_000_000))
        variant = ["mfma", "shuffle"][rng.integers(0, 2)]
        x = random_values(rng, n, dtype)
        f = _random_flags(rng, n)
        if what == 0:
            check_scan(run_segscan(x, f, variant, True), x, f)
        elif what == 1:
            out, nseg = run_segsum(x, f, variant, True)
            check_sum(out, nseg, x, f)
        else:
            z = B.mmv_scan(dev(x), n=n, variant=variant)
            torch.cuda.synchronize()
            check_scan(z.cpu().numpy(), x, np.zeros(n, dtype=np.uint8))


def test_random_csr_matrices():
    rng = np.random.default_rng(20260624)
    for case in range(30):
        n_rows, n_cols = int(rng.integers(1, 5000)), int(rng.integers(1, 5000))
        lengths = np.where(rng.random(n_rows) < rng.uniform(0.05, 1.0),
                           rng.geometric(1.0 / rng.integers(1, 200), size=n_rows), 0)
        lengths = np.minimum(lengths, 100_000 // max(n_rows, 1) + 50)
        rowptr = np.zeros(n_rows + 1, dtype=np.int32)
        np.cumsum(lengths, out=rowptr[1:])
        nnz = int(rowptr[-1])
        col = rng.integers(0, n_cols, size=nnz, dtype=np.int32)
        val = rng.standard_normal(nnz).astype(np.float32)
        x = rng.standard_normal(n_cols).astype(np.float32)
        pad = lambda a: a if len(a) else np.zeros(1, dtype=a.dtype)
        y = B.mmv_spmv_csr(n_rows, n_cols, dev(rowptr), dev(pad(col)), dev(pad(val)), dev(x), nnz=nnz)
        torch.cuda.synchronize()
        ref = oracle.spmv_csr(n_rows, n_cols, rowptr, col, val, x)
        A = oracle.spmv_csr(n_rows, n_cols, rowptr, col, np.abs(val), np.abs(x))
        assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * np.maximum(A, 1.0)).all(), case
        assert (y.cpu().numpy()[lengths == 0] == 0).all(), case


def test_hip_graph_replay_of_the_multi_kernel_entry_points():
    """segsum (count kernel + main kernel), CSR SpMV (six kernels) and SSCR (nine) enqueue only kernels;
    every replay of a captured call must give the eager result."""
    n = (1 << 21) + 77
    x, f = W.segscan_i8_uniform_len(n, max_len=300, seed=43)
    xt, ft = dev(x), packed_dev(f)
    sref, zref = oracle.segsum(x, f), oracle.segscan(x, f)
    out = torch.zeros(len(sref) + 8, dtype=torch.int32, device="cuda")
    nseg = torch.zeros(1, dtype=torch.int64, device="cuda")
    z = torch.zeros(n, dtype=torch.int32, device="cuda")
    ws1 = B.new_workspace(B.MMV_OP_SEGSUM, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    ws2 = B.new_workspace(B.MMV_OP_SEGSCAN_SSCR, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    row, col, val, xv = W.spmv_coo_zipf(20_000, 20_000, 400_000, cap=2000, seed=44)
    rowptr = W.csr_rowptr(row, 20_000)
    rpt, ct, vt, xvt = dev(rowptr), dev(col), dev(val), dev(xv)
    y = torch.zeros(20_000, dtype=torch.float32, device="cuda")
    ws3 = torch.empty(B.mmv_spmv_csr_workspace_bytes(20_000, len(val)), dtype=torch.uint8, device="cuda")

    def calls():
        B.mmv_segsum(xt, ft, n=n, out=out, nseg=nseg, ws=ws1)
        B.mmv_segscan_sscr(xt, ft, n=n, z=z, ws=ws2)
        B.mmv_spmv_csr(20_000, 20_000, rpt, ct, vt, xvt, y=y, ws=ws3)

    calls()                                                # eager
    torch.cuda.synchronize()
    yref = y.cpu().numpy().copy()
    assert np.array_equal(z.cpu().numpy(), zref) and np.array_equal(out.cpu().numpy()[:len(sref)], sref)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls()
    for rep in range(4):
        out.zero_(), z.zero_(), y.fill_(7.0), nseg.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(nseg.item()) == len(sref) and np.array_equal(out.cpu().numpy()[:len(sref)], sref), rep
        assert np.array_equal(z.cpu().numpy(), zref), rep
        got = y.cpu().numpy()
        assert (got[np.diff(rowptr) == 0] == 0).all() and np.allclose(got, yref, rtol=1e-5, atol=1e-5), rep
