"""Pins of the oracle's second group, bytes under bit-wise exclusive or (Sec. 2 states segmented scan for any
group): closed forms, numpy's own xor accumulate / reduceat, the group laws (self-inverse: the scan of the scan's
differences, concatenation, involution), brute force over every flag pattern against the unrolled definition, and
the paper's block-recursive algorithm and SCD route carried out with xor as the group operation."""
import itertools
from functools import reduce

import numpy as np

import oracle


def _definition(x, f):
    """z(i) = x(start(i)) ^ ... ^ x(i), start(i) the last segment start at or before i, on Python integers."""
    z = []
    for i in range(len(x)):
        s = max([k for k in range(i + 1) if k == 0 or f[k]])
        z.append(reduce(lambda a, b: a ^ b, [int(v) for v in x[s:i + 1]]))
    return z


def test_small_example_by_hand():
    x = np.array([2, 2, 3, 3, 1, 3, 1, 2], dtype=np.uint8)        # the values and flags of the worked example of Sec. 2
    f = np.array([1, 0, 1, 0, 0, 1, 0, 0], dtype=np.uint8)
    assert oracle.segscan(x, f).tolist() == [2, 0, 3, 0, 1, 3, 2, 0]
    assert oracle.segsum(x, f).tolist() == [0, 1, 0]


def test_every_flag_pattern_against_the_definition():
    rng = np.random.default_rng(2390680)
    for n in range(1, 10):
        for _ in range(3):
            x = rng.integers(0, 256, size=n, dtype=np.uint8)
            for bits in itertools.product((0, 1), repeat=n):
                f = np.array(bits, dtype=np.uint8)
                want = _definition(x, bits)
                assert oracle.segscan(x, f).tolist() == want
                ends = [i for i in range(n) if i == n - 1 or bits[i + 1]]
                assert oracle.segsum(x, f).tolist() == [want[i] for i in ends]


def test_library_special_cases():
    rng = np.random.default_rng(2390681)
    x = rng.integers(0, 256, size=10_001, dtype=np.uint8)
    f = (rng.random(len(x)) < 0.03).astype(np.uint8)
    none = np.zeros(len(x), dtype=np.uint8)
    assert np.array_equal(oracle.segscan(x, none), np.bitwise_xor.accumulate(x).astype(np.int32))
    assert np.array_equal(oracle.scan(x), np.bitwise_xor.accumulate(x).astype(np.int32))
    assert np.array_equal(oracle.segscan(x, np.ones(len(x), dtype=np.uint8)), x.astype(np.int32))
    starts = np.flatnonzero(np.concatenate([[1], f[1:]]))
    assert np.array_equal(oracle.segsum(x, f), np.bitwise_xor.reduceat(x, starts).astype(np.int32))
    L = 37
    y = x[:L * 270]
    g = np.zeros(len(y), dtype=np.uint8)
    g[::L] = 1
    assert np.array_equal(oracle.segsum(y, g), np.bitwise_xor.reduce(y.reshape(-1, L), axis=1).astype(np.int32))


def test_closed_forms_and_group_laws():
    rng = np.random.default_rng(2390682)
    n = 5000
    f = (rng.random(n) < 0.01).astype(np.uint8)
    f[0] = 1
    pos = np.arange(n) - np.maximum.accumulate(np.where(f != 0, np.arange(n), 0))     # offset inside the segment
    c = 0xA7
    z = oracle.segscan(np.full(n, c, dtype=np.uint8), f)
    assert np.array_equal(z, np.where(pos % 2 == 0, c, 0))                          # c, 0, c, 0, ... in every segment
    x = rng.integers(0, 256, size=n, dtype=np.uint8)
    z = oracle.segscan(x, f)
    assert (z[f != 0] == x[f != 0]).all()                                          # restart at every flag
    inner = f == 0
    inner[0] = False
    assert np.array_equal((z[1:] ^ z[:-1])[inner[1:]], x[1:][inner[1:]])            # x is the xor-difference of z
    y = rng.integers(0, 256, size=n, dtype=np.uint8)
    assert np.array_equal(oracle.segscan(x ^ y, f), z ^ oracle.segscan(y, f))       # homomorphism
    assert (oracle.segscan(x, f) >> 8 == 0).all()                                  # the byte, nothing above it
    g = (rng.random(n) < 0.02).astype(np.uint8)
    g[0] = 1
    both = oracle.segscan(np.concatenate([x, y]), np.concatenate([f, g]))
    assert np.array_equal(both, np.concatenate([z, oracle.segscan(y, g)]))          # concatenation


def test_block_recursive_algorithm_with_xor():
    """Speculative row scans ignoring the flags, revert with the group inverse (xor again), aggregates, recursion,
    carry into the open first segments: the steps of the block-recursive algorithm (Sec. 4.2), s = 4 and 32."""
    rng = np.random.default_rng(2390683)

    def block_recursive(x, f, s):
        n = len(x)
        if n == 0:
            return []
        if n <= s:
            return _definition(x, f)
        rows = [(a, min(n, a + s)) for a in range(0, n, s)]
        z = [0] * n
        agg, any_flag = [], []
        for a, b in rows:
            spec = list(itertools.accumulate([int(v) for v in x[a:b]], lambda p, q: p ^ q))     # x-bar: flags ignored
            for j in range(a, b):
                st = max([k for k in range(a, j + 1) if f[k]], default=None)
                z[j] = spec[j - a] ^ (spec[st - 1 - a] if st is not None and st > a else 0)       # REVSPEC
            agg.append(z[b - 1])
            any_flag.append(1 if any(f[a:b]) else 0)
        up = block_recursive(agg, any_flag, s)                                                    # recursion
        for r, (a, b) in enumerate(rows[1:], start=1):
            for j in range(a, b):                                                                # UpdateFirstSegment
                if any(f[a:j + 1]):
                    break
                z[j] ^= up[r - 1]
        return z

    for n, s in [(70, 4), (300, 4), (2000, 32), (1025, 32)]:
        x = rng.integers(0, 256, size=n, dtype=np.uint8)
        f = (rng.random(n) < 0.05).astype(np.uint8)
        f[0] = 1
        assert block_recursive(x, f, s) == oracle.segscan(x, f).tolist(), (n, s)
