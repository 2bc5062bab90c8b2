"""Pins for the sequential CPU oracle (oracle/mmvseg_oracle.c).

Each test ties the oracle to something that is not the oracle: values printed
in the paper, closed forms, library routines on special cases, invariants, and
brute force against the unrolled definition on Python integers.
"""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from oracle import formulations as F
from paper_2506_23906_amd import workloads as W


# ---- P1: the worked example of Sec. 2 -------------------------------------------

@pytest.mark.parametrize("dtype", [np.int8, np.float16, np.float32])
def test_worked_example(golden_sec2, dtype):
    g = golden_sec2
    x = np.array(g["x"], dtype=dtype)
    f = np.array(g["f"], dtype=np.uint8)
    assert oracle.segscan(x, f).tolist() == g["segscan"]
    assert oracle.segsum(x, f).tolist() == g["segsum"]
    assert F.compress(g["x"], g["f"]).tolist() == g["compress"]


def test_flag_at_position_zero_is_ignored(golden_sec2):
    g = golden_sec2
    x = np.array(g["x"], dtype=np.int8)
    f = np.array(g["f"], dtype=np.uint8)
    f0 = f.copy()
    f0[0] = 0
    assert oracle.segscan(x, f0).tolist() == g["segscan"]
    assert oracle.segsum(x, f0).tolist() == g["segsum"]


# ---- P2: closed forms ----------------------------------------------------------------

def test_all_ones_values_give_segment_lengths():
    rng = np.random.default_rng(11)
    lengths = rng.integers(1, 100, size=500)
    n = int(lengths.sum())
    f = W.flags_from_lengths(lengths, n)
    x = np.ones(n, dtype=np.int8)
    assert oracle.segsum(x, f).tolist() == lengths.tolist()
    starts = np.repeat(np.cumsum(lengths) - lengths, lengths)
    assert (oracle.segscan(x, f) == np.arange(n) - starts + 1).all()
    assert (oracle.segsum(x.astype(np.float32), f) == lengths).all()


def test_arithmetic_series_per_segment():
    rng = np.random.default_rng(12)
    lengths = rng.integers(1, 300, size=200)
    n = int(lengths.sum())
    f = W.flags_from_lengths(lengths, n)
    x = np.arange(n, dtype=np.float64)          # exact in fp64
    a = np.cumsum(lengths) - lengths            # first index of each segment
    b = a + lengths - 1                         # last index
    expect = (a + b) * lengths / 2
    assert (oracle.segsum(x, f) == expect).all()
    i = np.arange(n)
    st = np.repeat(a, lengths)
    assert (oracle.segscan(x, f) == (st + i) * (i - st + 1) / 2).all()


def test_constant_values():
    f = W.uniform_density_flags(5000, 0.03, 5)
    x = np.full(5000, -3, dtype=np.int8)
    idx = np.flatnonzero(f)
    lengths = np.diff(np.append(idx, 5000))
    assert oracle.segsum(x, f).tolist() == (-3 * lengths).tolist()


# ---- P3: special cases that are library routines -------------------------------------------

def test_single_segment_is_cumsum():
    rng = np.random.default_rng(13)
    x = rng.integers(-128, 128, size=10000, dtype=np.int8)
    f = np.zeros(10000, dtype=np.uint8)
    assert (oracle.segscan(x, f) == np.cumsum(x, dtype=np.int32)).all()
    assert oracle.segsum(x, f).tolist() == [int(x.astype(np.int64).sum())]
    xf = rng.standard_normal(10000).astype(np.float32)
    assert np.array_equal(oracle.segscan(xf, f), np.cumsum(xf.astype(np.float64)))


def test_every_flag_set_is_identity():
    rng = np.random.default_rng(14)
    x = rng.integers(-128, 128, size=777, dtype=np.int8)
    f = np.ones(777, dtype=np.uint8)
    assert (oracle.segscan(x, f) == x).all()
    assert (oracle.segsum(x, f) == x).all()
    xh = rng.standard_normal(777).astype(np.float16)
    assert np.array_equal(oracle.segscan(xh, f), xh.astype(np.float64))


@pytest.mark.parametrize("dtype", [np.int8, np.float32])
def test_segsum_is_reduceat(dtype):
    rng = np.random.default_rng(15)
    n = 20000
    f = W.uniform_density_flags(n, 0.02, 6)
    if dtype == np.int8:
        x = rng.integers(-128, 128, size=n, dtype=np.int8)
        ref = np.add.reduceat(x.astype(np.int64), np.flatnonzero(f))
        assert oracle.segsum(x, f).tolist() == ref.tolist()
    else:
        # integers stored as fp32 so that every summation order is exact
        x = rng.integers(-1000, 1000, size=n).astype(np.float32)
        ref = np.add.reduceat(x.astype(np.float64), np.flatnonzero(f))
        assert np.array_equal(oracle.segsum(x, f), ref)


def test_equal_length_segments_are_a_reshape_sum():
    rng = np.random.default_rng(16)
    L, m = 37, 211
    x = rng.integers(-100, 100, size=L * m).astype(np.float32)
    f = np.zeros(L * m, dtype=np.uint8)
    f[::L] = 1
    assert np.array_equal(oracle.segsum(x, f), x.astype(np.float64).reshape(m, L).sum(1))
    assert np.array_equal(oracle.segscan(x, f), np.cumsum(x.astype(np.float64).reshape(m, L), 1).ravel())


def test_spmv_against_scipy_and_dense():
    row, col, val, x = W.spmv_coo_zipf(300, 257, 1500, cap=64, seed=21)
    y = oracle.spmv_coo(300, 257, row, col, val, x)
    A = sp.coo_matrix((val.astype(np.float64), (row, col)), shape=(300, 257))
    ref = A.tocsr().dot(x.astype(np.float64))
    assert np.allclose(y, ref, rtol=1e-13, atol=1e-13)
    dense = np.zeros((300, 257))
    np.add.at(dense, (row, col), val.astype(np.float64))
    assert np.allclose(y, dense @ x.astype(np.float64), rtol=1e-12, atol=1e-12)
    counts = np.bincount(row, minlength=300)
    assert (counts == 0).any()                  # the generator produced empty rows
    assert (y[counts == 0] == 0.0).all()        # and they stay exactly zero


def test_spmv_order_independent_and_integer_exact():
    rng = np.random.default_rng(22)
    nnz = 5000
    row = np.sort(rng.integers(0, 100, size=nnz)).astype(np.int32)
    col = rng.integers(0, 80, size=nnz).astype(np.int32)
    val = rng.integers(-9, 10, size=nnz).astype(np.float32)
    x = rng.integers(-9, 10, size=80).astype(np.float32)
    y = oracle.spmv_coo(100, 80, row, col, val, x)
    perm = rng.permutation(nnz)
    assert np.array_equal(y, oracle.spmv_coo(100, 80, row[perm], col[perm], val[perm], x))
    ref = np.zeros(100, dtype=np.int64)
    np.add.at(ref, row, val.astype(np.int64) * x.astype(np.int64)[col])
    assert np.array_equal(y, ref.astype(np.float64))
    with pytest.raises(ValueError):
        oracle.spmv_coo(100, 80, row, col + 80, val, x)


# ---- P4: invariants -------------------------------------------------------------------------

def test_invariants_int():
    rng = np.random.default_rng(17)
    n = 50000
    x = rng.integers(-128, 128, size=n, dtype=np.int8)
    f = W.uniform_density_flags(n, 0.01, 7)
    z = oracle.segscan(x, f)
    s = oracle.segsum(x, f)
    ends = np.append(f[1:], 1).astype(bool)
    assert (z[ends] == s).all()                          # last scan value of a segment = its sum
    assert (z[f.astype(bool)] == x[f.astype(bool)]).all()  # restart at every flag
    inner = ~f.astype(bool)
    inner[0] = False
    assert ((z[1:] - z[:-1])[inner[1:]] == x[1:][inner[1:]]).all()
    assert len(s) == 1 + int(f[1:].sum())


def test_concatenation_and_shift_invariance():
    rng = np.random.default_rng(18)
    x1 = rng.integers(-128, 128, size=3000, dtype=np.int8)
    x2 = rng.integers(-128, 128, size=4111, dtype=np.int8)
    f1 = W.uniform_density_flags(3000, 0.01, 8)
    f2 = W.uniform_density_flags(4111, 0.02, 9)       # f2[0] = 1
    whole = oracle.segscan(np.concatenate([x1, x2]), np.concatenate([f1, f2]))
    assert (whole == np.concatenate([oracle.segscan(x1, f1), oracle.segscan(x2, f2)])).all()
    for k in (1, 2, 31, 33, 64):
        xs = np.concatenate([np.full(k, 5, dtype=np.int8), x2])
        fs = np.concatenate([np.ones(k, dtype=np.uint8), f2])
        assert (oracle.segscan(xs, fs)[k:] == oracle.segscan(x2, f2)).all()


def test_linearity_mod_2_32():
    rng = np.random.default_rng(19)
    n = 20000
    a = rng.integers(-60, 60, size=n, dtype=np.int8)
    b = rng.integers(-60, 60, size=n, dtype=np.int8)
    f = W.uniform_density_flags(n, 0.005, 10)
    za, zb, zab = oracle.segscan(a, f), oracle.segscan(b, f), oracle.segscan((a + b).astype(np.int8), f)
    assert (zab == za + zb).all()


def test_int32_wraps_like_the_integers_mod_2_32():
    n = 17_500_000                                   # 127 * n > 2^31
    x = np.full(n, 127, dtype=np.int8)
    f = np.zeros(n, dtype=np.uint8)
    z = oracle.segscan(x, f)
    for i in (0, 1, 16_909_320, 16_909_321, n - 1):
        want = (127 * (i + 1) + 2 ** 31) % 2 ** 32 - 2 ** 31
        assert int(z[i]) == want
    assert (z < 0).any()
    x[:] = -128
    s = oracle.segsum(x, f)
    assert int(s[0]) == (-128 * n + 2 ** 31) % 2 ** 32 - 2 ** 31


def test_empty_and_single():
    e8 = np.zeros(0, dtype=np.int8)
    ef = np.zeros(0, dtype=np.uint8)
    assert oracle.segscan(e8, ef).shape == (0,)
    assert oracle.segsum(e8, ef).shape == (0,)
    assert oracle.segscan(np.array([7], dtype=np.int8), np.array([0])).tolist() == [7]
    assert oracle.segsum(np.array([7], dtype=np.int8), np.array([0])).tolist() == [7]


# ---- P5: brute force over every flag pattern, n <= 12 ---------------------------------------

@pytest.mark.parametrize("n", list(range(1, 13)))
def test_brute_force_all_flag_patterns(n):
    rng = np.random.default_rng(100 + n)
    vectors = [rng.integers(-128, 128, size=n, dtype=np.int8),
               np.arange(1, n + 1, dtype=np.int8),
               np.full(n, -128, dtype=np.int8)]
    for bits in itertools.product((0, 1), repeat=n):
        f = np.array(bits, dtype=np.uint8)
        for x in vectors[: (3 if n <= 10 else 1)]:
            want = F.definitional_segscan(x, f)
            assert oracle.segscan(x, f).tolist() == want
            assert oracle.segsum(x, f).tolist() == F.definitional_segsum(x, f)
            assert oracle.segscan(x.astype(np.float32), f).tolist() == want
