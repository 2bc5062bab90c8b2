"""Pins for the oracle's parallel primitives (SCAN, COMPRESS, DIFF, REVERT of Sec. 4.1) and CSR SpMV.

As in test_oracle_pins.py, every test ties an oracle function to something that is not the
oracle: the paper's printed example, closed forms, numpy / scipy routines, algebraic
identities between the primitives, brute force on Python integers, and the paper's own
compositions (SCD, SSCR) against the sequential segmented definitions.
"""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from oracle import formulations as F
from paper_2506_23906_amd import workloads as W


def wrap32(a):
    return (np.asarray(a, dtype=np.int64) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)


# ---- SCAN ----------------------------------------------------------------------------------------

def test_scan_closed_forms():
    n = 5000
    assert (oracle.scan(np.ones(n, dtype=np.int8)) == np.arange(1, n + 1)).all()
    i = np.arange(n, dtype=np.float64)
    assert (oracle.scan(i) == i * (i + 1) / 2).all()                 # exact in fp64 at this size
    assert (oracle.scan(np.full(n, -3, dtype=np.int8)) == -3 * np.arange(1, n + 1)).all()


def test_scan_is_numpy_cumsum():
    rng = np.random.default_rng(41)
    x = rng.integers(-128, 128, size=100_000, dtype=np.int8)
    assert (oracle.scan(x) == wrap32(np.cumsum(x.astype(np.int64)))).all()
    xf = rng.standard_normal(50_000).astype(np.float32)
    assert (oracle.scan(xf) == np.cumsum(xf.astype(np.float64))).all()
    xh = rng.standard_normal(50_000).astype(np.float16)
    assert (oracle.scan(xh) == np.cumsum(xh.astype(np.float64))).all()


def test_scan_wraps_like_two_complement():
    x = np.full(20_000_000, 127, dtype=np.int8)          # 2.54e9 > 2^31
    z = oracle.scan(x)
    assert z[-1] == wrap32([127 * 20_000_000])[0] and z[-1] < 0
    assert z[16_909_320 - 1] == 2147483640               # last value before the wrap


def test_scan_brute_force_python_ints():
    rng = np.random.default_rng(42)
    for n in range(0, 40):
        x = rng.integers(-8, 9, size=n, dtype=np.int8)
        ref = [sum(int(v) for v in x[:i + 1]) for i in range(n)]
        assert oracle.scan(x).tolist() == ref


@pytest.mark.parametrize("s", [2, 3, 4, 16, 32])
def test_scan_equals_algorithm_scan(s):
    """Algorithm "Scan in MMV-RAM" (block scans with U_s, recursion, carry add with B_s)."""
    rng = np.random.default_rng(43 + s)
    for n in [1, s - 1, s, s + 1, s * s, s * s + 1, 777]:
        x = rng.integers(-8, 9, size=n, dtype=np.int8)
        assert oracle.scan(x).tolist() == F.scan_alg(x, s).tolist()


def test_scan_is_segscan_with_one_segment():
    rng = np.random.default_rng(44)
    x = rng.integers(-8, 9, size=3000, dtype=np.int8)
    f = np.zeros(3000, dtype=np.uint8)
    assert (oracle.scan(x) == oracle.segscan(x, f)).all()


# ---- COMPRESS ---------------------------------------------------------------------------------

def test_compress_worked_example(golden_sec2):
    g = golden_sec2
    assert oracle.compress(np.array(g["x"], dtype=np.int32), g["f"]).tolist() == g["compress"]


def test_compress_is_boolean_indexing():
    rng = np.random.default_rng(45)
    for density in (0.0, 0.001, 0.3, 1.0):
        x = rng.integers(-2**31, 2**31, size=50_000, dtype=np.int64).astype(np.int32)
        m = (rng.random(50_000) < density).astype(np.uint8)
        assert (oracle.compress(x, m) == x[m != 0]).all()
    xf = rng.standard_normal(1000).astype(np.float32)
    m = rng.random(1000) < 0.5
    assert (oracle.compress(xf, m) == xf[m]).all()
    assert oracle.compress(np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint8)).shape == (0,)


def test_compress_of_positions_gives_mask_positions():
    m = np.zeros(1000, dtype=np.uint8)
    pos = [0, 1, 31, 32, 63, 64, 500, 999]
    m[pos] = 1
    assert oracle.compress(np.arange(1000, dtype=np.int32), m).tolist() == pos


# ---- DIFF ---------------------------------------------------------------------------------------

def test_diff_is_numpy_diff():
    rng = np.random.default_rng(46)
    x = rng.integers(-2**31, 2**31, size=10_000, dtype=np.int64).astype(np.int32)
    ref = wrap32(np.diff(x.astype(np.int64), prepend=0))
    assert (oracle.diff(x) == ref).all()
    xf = rng.standard_normal(10_000).astype(np.float32)
    assert (oracle.diff(xf) == np.diff(xf.astype(np.float64), prepend=0.0)).all()


def test_diff_inverts_scan():
    rng = np.random.default_rng(47)
    x = rng.integers(-128, 128, size=20_000, dtype=np.int8)
    assert (oracle.diff(oracle.scan(x)) == x).all()
    x = np.full(20_000_000, 127, dtype=np.int8)          # through the wrap-around
    assert (oracle.diff(oracle.scan(x)) == 127).all()


@pytest.mark.parametrize("s", [2, 4, 16])
def test_diff_equals_matrix_form(s):
    """DIFF as the product with D_s on s-blocks plus the boundary fix (Sec. 4.1)."""
    rng = np.random.default_rng(48)
    x = rng.integers(-1000, 1000, size=257, dtype=np.int64).astype(np.int32)
    assert oracle.diff(x).tolist() == F.diff_matmul(x, s).tolist()


# ---- REVERT, and the compositions SCD / SSCR out of the oracle's own primitives -----------------------

def _end_markers(f):
    return np.concatenate([f[1:], [1]]).astype(np.uint8)


def _count_scan(f):
    """SCAN(f) with position 0 counted as a start; flags go through the int8 scan."""
    g = (np.asarray(f) != 0).astype(np.int8)
    g[0] = 1
    return oracle.scan(g)


def test_sscr_on_the_worked_example(golden_sec2):
    g = golden_sec2
    x = np.array(g["x"], dtype=np.int8)
    f = np.array(g["f"], dtype=np.uint8)
    xhat, fhat = oracle.scan(x), _count_scan(f)
    assert xhat.tolist() == [2, 4, 7, 10, 11, 14, 15, 17]
    assert fhat.tolist() == [1, 1, 2, 2, 2, 3, 3, 3]
    w = oracle.compress(xhat, _end_markers(f))
    assert w.tolist() == [4, 11, 17]
    assert oracle.revert(xhat, fhat, w).tolist() == g["segscan"]
    assert oracle.diff(w).tolist() == g["segsum"]          # SCD: DIFF(COMPRESS(SCAN x, f^-))


def test_revert_by_hand():
    xhat = np.array([5, 7, 8, 20, 21], dtype=np.int32)
    fhat = np.array([1, 1, 2, 3, 3], dtype=np.int32)
    w = np.array([7, 8, 21], dtype=np.int32)
    assert oracle.revert(xhat, fhat, w).tolist() == [5, 7, 1, 12, 13]
    with pytest.raises(ValueError):
        oracle.revert(xhat, np.array([1, 1, 2, 3, 9], dtype=np.int32), w)


def test_revert_matches_paper_form_with_shifted_index():
    rng = np.random.default_rng(49)
    x = rng.integers(-8, 9, size=300, dtype=np.int8)
    f = W.uniform_density_flags(300, 0.1, 3)
    xhat, fhat = oracle.scan(x), _count_scan(f)
    w = oracle.compress(xhat, _end_markers(f))
    assert oracle.revert(xhat, fhat, w).tolist() == F.revert(xhat, fhat, w).tolist()


@pytest.mark.parametrize("density", [0.0, 0.01, 0.2, 1.0])
def test_scd_and_sscr_compositions_equal_the_sequential_definitions(density):
    rng = np.random.default_rng(50)
    n = 20_000
    x = rng.integers(-128, 128, size=n, dtype=np.int8)
    f = W.uniform_density_flags(n, density, 4)
    xhat, fhat = oracle.scan(x), _count_scan(f)
    w = oracle.compress(xhat, _end_markers(f))
    assert (oracle.revert(xhat, fhat, w) == oracle.segscan(x, f)).all()
    assert (oracle.diff(w) == oracle.segsum(x, f)).all()


def test_compositions_brute_force_all_flag_patterns():
    x = np.array([3, -1, 4, 1, -5, 9, 2, -6, 5], dtype=np.int8)
    for n in range(1, 10):
        for bits in itertools.product([0, 1], repeat=n):
            f = np.array(bits, dtype=np.uint8)
            xhat, fhat = oracle.scan(x[:n]), _count_scan(f)
            w = oracle.compress(xhat, _end_markers(f))
            assert oracle.revert(xhat, fhat, w).tolist() == F.definitional_segscan(x[:n], f)
            assert oracle.diff(w).tolist() == F.definitional_segsum(x[:n], f)


def test_compositions_survive_wrap_around():
    n = 18_000_000
    x = np.full(n, 127, dtype=np.int8)
    f = np.zeros(n, dtype=np.uint8)
    f[[0, 17_000_000, 17_500_000]] = 1                    # the speculative scan wraps before these
    xhat, fhat = oracle.scan(x), _count_scan(f)
    w = oracle.compress(xhat, _end_markers(f))
    assert (oracle.diff(w) == oracle.segsum(x, f)).all()
    z = oracle.revert(xhat, fhat, w)
    assert z[17_000_000] == 127 and z[-1] == 127 * 500_000 and z[16_999_999] == wrap32([127 * 17_000_000])[0]


# ---- REVERT on floats ---------------------------------------------------------------------------
#
# The float form of REVERT widens to double and subtracts there.  Pins that are not its own formula: the
# worked example of Sec. 2 carried in fp32, integer-valued fp32 inputs (every intermediate is exact, so
# the composition REVERT(SCAN, SCAN, COMPRESS) must equal the sequential definition), a hand case with
# non-integers whose differences are exact binary fractions, the numpy formulation, and the int32 form
# of the same function on the same integers.

def test_revert_fp32_on_the_worked_example(golden_sec2):
    g = golden_sec2
    xhat = np.array([2, 4, 7, 10, 11, 14, 15, 17], dtype=np.float32)   # SCAN(x) of the example
    fhat = np.array([1, 1, 2, 2, 2, 3, 3, 3], dtype=np.int32)           # SCAN(f)
    w = np.array([4, 11, 17], dtype=np.float32)                         # COMPRESS(SCAN(x), f^-)
    z = oracle.revert(xhat, fhat, w)
    assert z.dtype == np.float64
    assert z.tolist() == [float(v) for v in g["segscan"]]


def test_revert_fp32_by_hand_with_binary_fractions():
    xhat = np.array([0.5, 0.75, 1.0, 3.5, 3.625], dtype=np.float32)
    fhat = np.array([1, 1, 2, 3, 3], dtype=np.int32)
    w = np.array([0.75, 1.0, 3.625], dtype=np.float32)
    assert oracle.revert(xhat, fhat, w).tolist() == [0.5, 0.75, 0.25, 2.5, 2.625]
    # the first segment is left alone, the third subtracts w(1), not w(0) or w(2)
    assert oracle.revert(xhat, np.array([1, 1, 1, 1, 1], dtype=np.int32), w).tolist() == xhat.astype(np.float64).tolist()
    with pytest.raises(ValueError):
        oracle.revert(xhat, np.array([1, 1, 2, 3, 6], dtype=np.int32), w)


@pytest.mark.parametrize("density", [0.0, 0.02, 0.3, 1.0])
def test_revert_fp32_integer_valued_composition_equals_definition(density):
    rng = np.random.default_rng(51)
    n = 5_000
    xi = rng.integers(-100, 101, size=n)                      # |prefix| < 2^24: exact in fp32
    x = xi.astype(np.float32)
    f = W.uniform_density_flags(n, density, 6)
    xhat = oracle.scan(x).astype(np.float32)                  # exact
    fhat = _count_scan(f)
    w = oracle.compress(xhat, _end_markers(f))
    z = oracle.revert(xhat, fhat, w)
    assert z.tolist() == [float(v) for v in F.definitional_segscan(xi, f)]
    assert z.tolist() == F.revert(xhat.astype(np.float64), fhat, w.astype(np.float64)).tolist()
    # the int32 form of REVERT on the same integers
    zi = oracle.revert(xhat.astype(np.int32), fhat, w.astype(np.int32))
    assert z.tolist() == [float(v) for v in zi.tolist()]


def test_revert_fp32_brute_force_all_flag_patterns():
    xi = np.array([3, -1, 4, 1, -5, 9, 2, -6], dtype=np.int64)
    x = (xi * 0.25).astype(np.float32)                        # quarter steps: exact sums
    for n in range(1, 9):
        for bits in itertools.product([0, 1], repeat=n):
            f = np.array(bits, dtype=np.uint8)
            xhat = oracle.scan(x[:n]).astype(np.float32)
            w = oracle.compress(xhat, _end_markers(f))
            z = oracle.revert(xhat, _count_scan(f), w)
            assert (z * 4).tolist() == [float(v) for v in F.definitional_segscan(xi[:n], f)]


def test_revert_fp32_subtracts_in_double():
    # 2^24 + 1 is not an fp32 number, so the inputs are 2^24 + 2 and 1: the difference 2^24 + 1 must come
    # out exactly (a subtraction carried out in fp32 would round it)
    xhat = np.array([1.0, 16777218.0], dtype=np.float32)
    z = oracle.revert(xhat, np.array([1, 2], dtype=np.int32), np.array([1.0, 16777218.0], dtype=np.float32))
    assert z.tolist() == [1.0, 16777217.0]


# ---- CSR SpMV ---------------------------------------------------------------------------------------

def test_spmv_csr_is_scipy_csr():
    row, col, val, x = W.spmv_coo_zipf(3000, 2500, 90_000, cap=700, seed=51)
    rowptr = W.csr_rowptr(row, 3000)
    A = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(3000, 2500))
    ref = A.dot(x.astype(np.float64))
    got = oracle.spmv_csr(3000, 2500, rowptr, col, val, x)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)
    assert (got[np.diff(rowptr) == 0] == 0.0).all()        # rows without entries are exactly 0
    assert np.array_equal(got, oracle.spmv_coo(3000, 2500, row, col, val, x))


def test_spmv_csr_dense_tiny():
    rng = np.random.default_rng(52)
    A = (rng.random((7, 5)) < 0.4) * rng.standard_normal((7, 5)).astype(np.float32)
    A[3, :] = 0
    A = A.astype(np.float32)
    x = rng.standard_normal(5).astype(np.float32)
    r, c = np.nonzero(A)
    rowptr = W.csr_rowptr(r, 7)
    got = oracle.spmv_csr(7, 5, rowptr, c, A[r, c], x)
    assert np.allclose(got, A.astype(np.float64) @ x.astype(np.float64), rtol=1e-14, atol=1e-15)


def test_spmv_csr_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.spmv_csr(2, 2, [0, 2, 1], [0, 1], [1.0, 1.0], [1.0, 1.0])
    with pytest.raises(ValueError):
        oracle.spmv_csr(1, 2, [0, 1], [5], [1.0], [1.0, 1.0])


# ---- the blocked sparse-attention generator (structure only: it holds no arithmetic) -----------------

def test_blocked_sparse_attention_structure():
    n, b, r = 512, 4, 2
    rowptr, col, val, x = W.blocked_sparse_attention(n, block=b, n_random=r, seed=53)
    nb = n // b
    A = sp.csr_matrix((np.ones_like(val), col, rowptr), shape=(n, n)).toarray()
    assert (A[:2 * b, :] == 1).all()                                   # global rows are full
    assert (A[:, :2 * b] == 1).all()                                   # global columns
    blocks = A.reshape(nb, b, nb, b).transpose(0, 2, 1, 3)
    present = blocks.reshape(nb, nb, -1)
    assert ((present.min(axis=2) == present.max(axis=2))).all()        # blocks are full or empty
    P = present.max(axis=2)
    for i in range(2, nb):
        assert P[i, max(i - 1, 0):min(i + 2, nb)].all()                # three window blocks
        assert 2 + 2 <= P[i].sum() <= 2 + 3 + r
    assert (np.diff(col.astype(np.int64))[np.setdiff1d(np.arange(len(col) - 1), rowptr[1:-1] - 1)] > 0).all()
