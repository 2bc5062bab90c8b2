"""GPU parity of the second group, bytes under bit-wise exclusive or (uint8 values): segmented scan, segmented
sum and the unsegmented scan against the oracle, bit for bit, both variants (the matrix-core one takes the
running xor as the parity of integer sums of bit planes)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import check_scan, check_sum, dev, packed_dev, run_segscan, run_segsum

pytestmark = pytest.mark.gpu
VARIANTS = ["mfma", "shuffle"]
TILE = 65536


@pytest.mark.parametrize("variant", VARIANTS)
def test_sizes_and_densities(variant):
    rng = np.random.default_rng(2390690)
    for n in (1, 2, 31, 32, 33, 2047, 2048, 2049, 16384, TILE - 1, TILE, TILE + 1, 3 * TILE + 4321, 40 * TILE + 77):
        for density in (0.0, 0.0005, 0.03, 0.5, 1.0):
            x = rng.integers(0, 256, size=n, dtype=np.uint8)
            f = (rng.random(n) < density).astype(np.uint8)
            check_scan(run_segscan(x, f, variant, packed=bool(n % 2)), x, f)
            out, nseg = run_segsum(x, f, variant)
            check_sum(out, nseg, x, f)


@pytest.mark.parametrize("variant", VARIANTS)
def test_every_flag_pattern_n10(variant):
    x = np.array([0x80, 0xFF, 0x01, 0x7E, 0x55, 0xAA, 0x0F, 0xF0, 0x33, 0xC4], dtype=np.uint8)
    pats = np.array(list(itertools.product((0, 1), repeat=10)), dtype=np.uint8)
    xs = np.tile(x, len(pats))
    # all 1024 patterns side by side, each opened by a flag so that they do not run into each other
    fs = pats.copy()
    fs[:, 0] = 1
    z = run_segscan(xs, fs.reshape(-1), variant)
    assert np.array_equal(z, oracle.segscan(xs, fs.reshape(-1)))


@pytest.mark.parametrize("variant", VARIANTS)
def test_long_segments_and_unsegmented_scan(variant):
    rng = np.random.default_rng(2390691)
    n = 600 * TILE + 12345               # more tiles than one round of workgroups: tickets and look-back
    x = rng.integers(0, 256, size=n, dtype=np.uint8)
    f = np.zeros(n, dtype=np.uint8)
    f[[0, 5, 7 * TILE + 3, 300 * TILE, 300 * TILE + 1, n - 1]] = 1
    check_scan(run_segscan(x, f, variant), x, f)
    out, nseg = run_segsum(x, f, variant)
    check_sum(out, nseg, x, f)
    z = B.mmv_scan(dev(x), n=n, variant=variant)
    torch.cuda.synchronize()
    assert z.dtype == torch.int32
    assert np.array_equal(z.cpu().numpy(), np.bitwise_xor.accumulate(x).astype(np.int32))


def test_workload_shape_of_the_headline():
    """The int8 headline's segment lengths (U{1..4096}) on 2^24 bytes; every bit plane is used."""
    n = 1 << 24
    _, f = W.segscan_i8_uniform_len(n)
    x = np.random.default_rng(2390692).integers(0, 256, size=n, dtype=np.uint8)
    for variant in VARIANTS:
        z = run_segscan(x, f, variant)
        check_scan(z, x, f)
        assert int(np.bitwise_or.reduce(z)) == 0xFF


def test_compositions_and_spmv_do_not_take_the_xor_type():
    n = 4096
    x = dev(np.zeros(n, dtype=np.uint8))
    f = packed_dev(np.zeros(n, dtype=np.uint8))
    with pytest.raises(RuntimeError, match="not implemented|unsupported|UNSUPPORTED"):
        B.mmv_segscan_sscr(x, f, n=n)
    with pytest.raises(RuntimeError, match="not implemented|unsupported|UNSUPPORTED"):
        B.mmv_segsum_scd(x, f, n=n)
