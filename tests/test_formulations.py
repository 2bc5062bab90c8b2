"""The paper's own algorithms, written out in numpy, against the sequential oracle.

Exact on integers: SCD (Sec. 4.1), SSCR (Sec. 4.1), the block-recursive
algorithm and the REVSPEC lemma (appendix), for several block sizes s.
"""
import itertools

import numpy as np
import pytest

import oracle
from oracle import formulations as F
from paper_2506_23906_amd import workloads as W

S_VALUES = [2, 3, 4, 16, 32]


def _rand(n, density, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(-128, 128, size=n, dtype=np.int8), W.uniform_density_flags(n, density, seed + 1)


@pytest.mark.parametrize("s", S_VALUES)
@pytest.mark.parametrize("n", [1, 2, 15, 16, 17, 100, 1000])
def test_scan_algorithm_is_cumsum(s, n):
    x, _ = _rand(n, 0.1, 3 * n + s)
    assert F.scan_alg(x, s).tolist() == np.cumsum(x.astype(np.int64)).tolist()


def test_scan_alg_matrix_shapes():
    assert F.U(3).tolist() == [[1, 1, 1], [0, 1, 1], [0, 0, 1]]
    assert F.D(3).tolist() == [[1, -1, 0], [0, 1, -1], [0, 0, 1]]
    # MATMUL(x, U_s) prefix-sums every s-block on its own and zero-pads the tail
    assert F.matmul_op([1, 2, 3, 4, 5], F.U(3)).tolist() == [1, 3, 6, 4, 9, 9]
    z = np.arange(23) ** 2
    assert F.diff_matmul(z, 4).tolist() == F.diff(z).tolist()


@pytest.mark.parametrize("s", S_VALUES)
@pytest.mark.parametrize("n,density", [(1, 1.0), (7, 0.5), (64, 0.2), (500, 0.05), (2000, 0.01), (333, 1.0),
                                       (333, 0.0)])
def test_scd_sscr_block_recursive(s, n, density):
    x, f = _rand(n, density, 17 * n + s)
    zref = oracle.segscan(x, f)
    sref = oracle.segsum(x, f)
    assert F.scd(x, f, s).tolist() == sref.tolist()
    assert F.sscr(x, f, s).tolist() == zref.tolist()
    assert F.block_recursive_segscan(x, f, s).tolist() == zref.tolist()


@pytest.mark.parametrize("s", [2, 3, 4])
def test_formulations_brute_force_small(s):
    for n in range(1, 10):
        x = np.arange(1, n + 1, dtype=np.int8) * 3 - 7
        for bits in itertools.product((0, 1), repeat=n):
            f = np.array(bits, dtype=np.uint8)
            want = oracle.segscan(x, f).tolist()
            assert F.block_recursive_segscan(x, f, s).tolist() == want
            assert F.sscr(x, f, s).tolist() == want
            assert F.scd(x, f, s).tolist() == oracle.segsum(x, f).tolist()


@pytest.mark.parametrize("s", [4, 8, 16, 32])
def test_revspec_lemma_per_block(s):
    """REVSPEC on one block equals the segmented scan of that block alone, and its
    filter matrix selects at most one earlier position per element."""
    rng = np.random.default_rng(40 + s)
    for trial in range(200):
        x = rng.integers(-128, 128, size=s, dtype=np.int8)
        f = (rng.random(s) < rng.choice([0.0, 0.1, 0.5, 1.0])).astype(np.uint8)
        xbar = np.cumsum(x.astype(np.int64))
        fbar = np.cumsum(f.astype(np.int64))
        # inside one block a segment that was open at the block start keeps its running value
        want = oracle.segscan(x, f)
        assert F.revspec_lemma(xbar, fbar).tolist() == want.tolist()
        assert max(F._count_selected(xbar, fbar)) <= 1
    # shortcut cases of the simple revert: no flag / only flag at 0 -> unchanged; all flags -> z = x
    x = rng.integers(-128, 128, size=3 * s, dtype=np.int8)
    f = np.zeros(3 * s, dtype=np.uint8)
    f[s] = 1
    f[2 * s:] = 1
    z = F.revert_spec_simple(x, f, s)
    assert z[:s].tolist() == np.cumsum(x[:s].astype(np.int64)).tolist()
    assert z[s:2 * s].tolist() == np.cumsum(x[s:2 * s].astype(np.int64)).tolist()
    assert z[2 * s:].tolist() == x[2 * s:].tolist()


@pytest.mark.parametrize("s", [4, 16, 32])
def test_revert_simple_equals_lemma_blockwise(s):
    x, f = _rand(40 * s + 5, 0.15, 77 + s)
    a = F.revert_spec_simple(x, f, s)
    b = F.revspec(F.matmul_op(x, F.U(s)), F.matmul_op(f, F.U(s)), s)[:len(x)]
    assert a.tolist() == b.tolist()
    # and both are the segmented scan restarted at every block boundary
    f2 = f.copy()
    f2[::s] = 1
    assert a.tolist() == oracle.segscan(x, f2).tolist()
