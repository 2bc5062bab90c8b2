"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import (check_scan, check_sum, dev, packed_dev, random_values, run_segscan, run_segsum)

pytestmark = pytest.mark.gpu

DTYPES = [np.int8, np.float16, np.float32]
VARIANTS = ["mfma", "shuffle"]
TILE = 65536          # largest workgroup tile (int8); other types and short inputs use smaller ones
SIZES = [1, 2, 31, 32, 33, 63, 64, 65, 1023, 1024, 1025, 2047, 2048, 2049, TILE - 1, TILE, TILE + 1,
         3 * TILE + 77, 16 * TILE + 5]


def test_worked_example_on_gpu(golden_sec2):
    g = golden_sec2
    f = np.array(g["f"], dtype=np.uint8)
    for dtype in DTYPES:
        x = np.array(g["x"], dtype=dtype)
        for variant in VARIANTS:
            assert run_segscan(x, f, variant).tolist() == g["segscan"]
            out, nseg = run_segsum(x, f, variant)
            assert nseg == 3 and out[:3].tolist() == g["segsum"]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dtype", DTYPES)
def test_sizes_and_densities(dtype, variant):
    rng = np.random.default_rng(1234)
    for n in SIZES:
        for density in (0.0, 0.002, 0.05, 0.5, 1.0):
            x = random_values(rng, n, dtype)
            f = W.uniform_density_flags(n, density, seed=n + int(density * 1000))
            print("segscan/segsum", dtype.__name__, variant, "n=%d density=%g" % (n, density), flush=True)
            check_scan(run_segscan(x, f, variant), x, f)
            out, nseg = run_segsum(x, f, variant)
            check_sum(out, nseg, x, f)


@pytest.mark.parametrize("variant", VARIANTS)
def test_every_flag_pattern_n10(variant):
    """All 2^n flag patterns, n <= 10, laid end to end (each pattern starts a segment)."""
    for n in (3, 7, 10):
        pats = np.array(list(itertools.product((0, 1), repeat=n)), dtype=np.uint8)
        pats[:, 0] = 1
        f = pats.reshape(-1)
        x = np.tile(np.arange(1, n + 1, dtype=np.int8) * 5 - 17, len(pats))
        print("patterns", variant, n, flush=True)
        check_scan(run_segscan(x, f, variant), x, f)
        out, nseg = run_segsum(x, f, variant)
        check_sum(out, nseg, x, f)
        xf = x.astype(np.float32)
        assert np.array_equal(run_segscan(xf, f, variant), oracle.segscan(xf, f).astype(np.float32))


@pytest.mark.parametrize("dtype", DTYPES)
def test_shift_invariance(dtype):
    """Prepending k single-element segments moves every row and tile border."""
    rng = np.random.default_rng(99)
    n = 2 * TILE + 100
    x = random_values(rng, n, dtype)
    f = W.uniform_density_flags(n, 0.01, seed=5)
    for k in (1, 3, 31, 32, 33, 64, 2047, 2049):
        xs = np.concatenate([random_values(rng, k, dtype), x])
        fs = np.concatenate([np.ones(k, dtype=np.uint8), f])
        print("shift", dtype.__name__, k, flush=True)
        check_scan(run_segscan(xs, fs), xs, fs)


@pytest.mark.parametrize("dtype", DTYPES)
def test_u8_flags_equal_packed_flags(dtype):
    rng = np.random.default_rng(7)
    for n in (1, 37, 5000, 3 * TILE + 19):
        x = random_values(rng, n, dtype)
        f = W.uniform_density_flags(n, 0.03, seed=n)
        f[f != 0] = rng.integers(1, 256, size=int(f.sum()))      # any non-zero byte is a flag
        a = run_segscan(x, f, packed=True)
        b = run_segscan(x, f, packed=False)
        assert np.array_equal(a, b)
        check_scan(b, x, f)
        out, nseg = run_segsum(x, f, packed=False)
        check_sum(out, nseg, x, f)


def test_flag_zero_is_ignored_and_bits_beyond_n_too():
    x = np.arange(1, 41, dtype=np.int8)
    f = np.zeros(40, dtype=np.uint8)
    f[[5, 17]] = 1
    want = oracle.segscan(x, f)
    words = W.pack_flags(f).copy()
    words[1] |= 0xFFFFFF00                       # garbage beyond n = 40
    ft = torch.from_numpy(words.view(np.int32).copy()).cuda()
    z = B.mmv_segscan(dev(x), ft, n=40)
    assert np.array_equal(z.cpu().numpy(), want)
    out, nseg = B.mmv_segsum(dev(x), ft, n=40)
    assert int(nseg.item()) == 3
    assert np.array_equal(out.cpu().numpy()[:3], oracle.segsum(x, f))


def test_int32_wraps():
    n = 17_500_000
    x = np.full(n, 127, dtype=np.int8)
    f = np.zeros(n, dtype=np.uint8)
    z = run_segscan(x, f)
    check_scan(z, x, f)
    assert (z < 0).any()
    out, nseg = run_segsum(x, f)
    check_sum(out, nseg, x, f)


def test_long_segments_across_many_tiles():
    rng = np.random.default_rng(3)
    n = 70 * TILE + 123
    for dtype in DTYPES:
        x = random_values(rng, n, dtype)
        f = np.zeros(n, dtype=np.uint8)
        f[[0, 5, 40 * TILE + 7, 40 * TILE + 8, 69 * TILE]] = 1
        check_scan(run_segscan(x, f), x, f)
        out, nseg = run_segsum(x, f)
        check_sum(out, nseg, x, f)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dtype", DTYPES)
def test_vectors_longer_than_one_round_of_workgroups(dtype, variant):
    """Just beyond what the resident workgroups cover with full tiles: the vector starts with tiles of growing length,
    continues with full ones and ends with short ones; the first round of workgroups takes tiles by index, the rest by
    ticket.  Sparse flags, so that carries cross every kind of tile border."""
    rng = np.random.default_rng(77)
    full = B.mmv_tile_elems(B.MMV_OP_SEGSCAN, B._DTYPES[torch.from_numpy(np.zeros(1, dtype=dtype)).dtype], 1 << 40)
    for n in (512 * full + 1, 515 * full + 4321):
        x = random_values(rng, n, dtype)
        f = W.uniform_density_flags(n, 2e-5, seed=n % 1000)
        print("long vector", dtype.__name__, variant, n, flush=True)
        check_scan(run_segscan(x, f, variant), x, f)
        out, nseg = run_segsum(x, f, variant)
        check_sum(out, nseg, x, f)


def test_repeated_runs_are_bit_identical_on_integers():
    x, f = W.segscan_i8_uniform_len(1 << 22, seed=4)
    xt, ft = dev(x), packed_dev(f)
    ref = oracle.segscan(x, f)
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, len(x))
    for rep in range(20):
        z = B.mmv_segscan(xt, ft, ws=ws)
        assert np.array_equal(z.cpu().numpy(), ref), rep
        assert B.mmv_workspace_status(ws) == 0


def test_fp16_subnormal_single_element_segments():
    """What the matrix cores do with fp16 subnormal inputs (the paper is silent)."""
    n = 4096
    x = (np.arange(n) % 1023 + 1).astype(np.uint16).view(np.float16)     # every positive subnormal
    f = np.ones(n, dtype=np.uint8)
    for variant in VARIANTS:
        z = run_segscan(x, f, variant)
        check_scan(z, x, f)                                              # gate: |err| <= 2e-3
        kept = np.array_equal(z, x.astype(np.float32))
        print("fp16 subnormals kept exactly (%s): %s" % (variant, kept))


def test_in_place_fp32():
    x, f = W.scan_sum_f32_bernoulli(3 * TILE + 5, seed=8)
    xt = dev(x)
    z = B.mmv_segscan(xt, packed_dev(f), z=xt)
    check_scan(z.cpu().numpy(), x, f)


@pytest.mark.parametrize("variant", VARIANTS)
def test_fp32_chunks_with_every_flag_set(variant):
    """Blocks of 2048 positions that all start segments (stored straight from the loaded registers by the
    matrix-core variant) between ordinary ones, at aligned and unaligned places, with a ragged end, and in place:
    in a whole chunk of set flags the result is the input bit for bit."""
    rng = np.random.default_rng(2390670)
    n = 37 * 16384 + 2048 * 3 + 777
    x = rng.standard_normal(n, dtype=np.float32)
    f = (rng.random(n) < 0.02).astype(np.uint8)
    dense = np.zeros(n, dtype=bool)
    for a, b in [(0, 2048), (4096, 4096 + 3 * 2048), (16384 * 5 - 2048, 16384 * 5 + 2048), (100_000, 109_999),
                 (16384 * 20, 16384 * 23), (n - 2048 - 777, n - 777), (n - 700, n)]:
        dense[a:b] = True
    f[dense] = 1
    z = run_segscan(x, f, variant)
    check_scan(z, x, f)
    if variant == "mfma":
        whole = np.flatnonzero(f[:n - n % 2048].reshape(-1, 2048).all(axis=1))      # chunks of 2048 with every flag set
        assert len(whole) >= 12
        for c in whole:
            assert np.array_equal(z[2048 * c:2048 * c + 2048].view(np.uint32), x[2048 * c:2048 * c + 2048].view(np.uint32)), c
    xt = dev(x)
    B.mmv_segscan(xt, packed_dev(f), n=n, z=xt, variant=variant)      # in place
    torch.cuda.synchronize()
    check_scan(xt.cpu().numpy(), x, f)


@pytest.mark.parametrize("variant", VARIANTS)
def test_fp32_segment_starts_hold_their_input_and_non_finite_values_stay_in_their_row(variant):
    """Floats are not a group: the method subtracts two speculative prefixes of a row of 32.  What that means next
    to a huge value and next to an infinity, pinned: (1) every position that starts a segment holds its input bit for
    bit, also right behind such a value; (2) an infinity makes the rest of its own segment infinite (as in the
    definition) and may turn later positions of the same row of 32 into NaN (the definition keeps those segments
    finite: the difference of two infinite prefixes is not a number), but nothing outside that row: its carry stops
    at the next flag; (3) the error behind a huge value is bounded by the rounding of that row's prefix."""
    rng = np.random.default_rng(606)
    n = 3 * 16384 + 1000
    x = (rng.random(n, dtype=np.float32) * 2 - 1).astype(np.float32)
    f = (rng.random(n) < 0.1).astype(np.uint8)
    f[0] = 1
    huge_at, inf_at = 5 * 32 + 7, 700 * 32 + 11
    for p in (huge_at, inf_at):
        f[p - 3:p + 12] = 0
        f[[p - 3, p + 1, p + 6]] = 1            # the value sits in a segment of four; two segments start right behind it
        f[(p // 32) * 32 + 32] = 1               # and the next row starts a segment
    x[huge_at] = np.float32(3.0e30)
    x[inf_at] = np.float32(np.inf)
    z = run_segscan(x, f, variant)
    starts = np.flatnonzero(f)
    assert np.array_equal(z[starts].view(np.uint32), x[starts].view(np.uint32))                     # (1)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.segscan(x, f)
    assert np.isinf(z[inf_at:inf_at + 1]).all() and np.isinf(ref[inf_at])                           # (2)
    row = slice((inf_at // 32) * 32, (inf_at // 32) * 32 + 32)
    not_finite = np.flatnonzero(~np.isfinite(z))
    assert len(not_finite) and (not_finite >= row.start).all() and (not_finite < row.stop).all(), not_finite
    assert np.isfinite(ref[inf_at + 1:row.stop]).all()          # the definition keeps the segments behind it finite
    print("positions of the infinity's row that are not finite (%s): %s; by the definition only %s" % (
        variant, (not_finite - row.start).tolist(), (np.flatnonzero(~np.isfinite(ref[row])).tolist())))
    ok = np.ones(n, dtype=bool)
    ok[row] = False
    A = oracle.segscan(np.abs(np.where(np.isfinite(x), x, 0).astype(np.float64)), f)
    err = np.abs(z.astype(np.float64) - ref)
    hrow = slice((huge_at // 32) * 32, (huge_at // 32) * 32 + 32)
    ok[hrow] = False
    assert (err[ok] <= 1e-4 * np.maximum(A[ok], 1.0)).all()
    # (3) in the row of the huge value the row prefix reaches 3e30: one rounding of it bounds the error
    assert (err[hrow] <= 2.0 ** -22 * 3.0e30).all()
    assert np.array_equal(z[huge_at + 1:huge_at + 2], x[huge_at + 1:huge_at + 2])               # a start right behind it: exact


def test_out_capacity_smaller_than_segment_count():
    x, f = W.segscan_i8_uniform_len(50_000, max_len=16, seed=9)
    ref = oracle.segsum(x, f)
    out, nseg = run_segsum(x, f, out_capacity=100)
    assert nseg == len(ref)
    assert np.array_equal(out[:100], ref[:100])
    assert out.shape[0] == 100


def test_empty_input():
    e = torch.empty(0, dtype=torch.int8, device="cuda")
    fl = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert B.mmv_segscan(e, fl, n=0).numel() == 0
    _, nseg = B.mmv_segsum(e, fl, n=0)
    assert int(nseg.item()) == 0


def _bf16_values(rng, n):
    xt = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(torch.bfloat16)
    return xt.cuda(), xt.float().numpy()                              # the bf16 values, exactly, as fp32


def test_bf16_inputs():
    rng = np.random.default_rng(21)
    n = 2 * TILE + 321
    xt, x32 = _bf16_values(rng, n)
    f = W.uniform_density_flags(n, 0.02, seed=2)
    for variant in VARIANTS:
        z = run_segscan(x32, f, variant, xt=xt)
        check_scan(z, x32, f, tol=1e-2)
        out, nseg = run_segsum(x32, f, variant, xt=xt)
        check_sum(out, nseg, x32, f, tol=1e-2)


@pytest.mark.parametrize("variant", VARIANTS)
def test_bf16_sizes_and_densities(variant):
    rng = np.random.default_rng(22)
    for n in SIZES:
        for density in (0.0, 0.002, 0.05, 1.0):
            xt, x32 = _bf16_values(rng, n)
            f = W.uniform_density_flags(n, density, seed=n + int(density * 1000))
            print("segscan/segsum bf16", variant, "n=%d density=%g" % (n, density), flush=True)
            check_scan(run_segscan(x32, f, variant, xt=xt), x32, f, tol=1e-2)
            out, nseg = run_segsum(x32, f, variant, xt=xt)
            check_sum(out, nseg, x32, f, tol=1e-2)


@pytest.mark.parametrize("variant", VARIANTS)
def test_bf16_2p24_uniform_len(variant):
    rng = np.random.default_rng(23)
    n = 1 << 24
    xt, x32 = _bf16_values(rng, n)
    _, f = W.segscan_i8_uniform_len(n, seed=24)
    check_scan(run_segscan(x32, f, variant, xt=xt), x32, f, tol=1e-2)
    out, nseg = run_segsum(x32, f, variant, xt=xt)
    check_sum(out, nseg, x32, f, tol=1e-2)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("density", [2e-5, 1e-3, 0.05])
def test_bf16_sums_longer_than_one_round_of_workgroups(density, variant):
    """The kernel that streams through long spans, bf16 instantiation (see test_sums_longer_than_one_round_of_workgroups
    for the margin: speculation over chunks of 2048 values; bf16 inputs carry 8 significant bits, their sums are
    rounded like those of any other fp32 values)."""
    rng = np.random.default_rng(25)
    full = B.mmv_tile_elems(B.MMV_OP_SEGSUM, B.MMV_BF16_F32, 1 << 40)
    n = 513 * full + 4321
    xt, x32 = _bf16_values(rng, n)
    f = W.uniform_density_flags(n, density, seed=n % 1000)
    print("long bf16 sum", density, n, flush=True)
    out, nseg = run_segsum(x32, f, variant, xt=xt)
    check_sum(out, nseg, x32, f, tol=1e-2, margin=1e-4)


# ---- the benchmark workloads: scaled twins, then full size ------------------------------------------

@pytest.mark.parametrize("variant", VARIANTS)
def test_workload1_f32_bernoulli_full(variant):
    x, f = W.scan_sum_f32_bernoulli()
    check_scan(run_segscan(x, f, variant), x, f)
    out, nseg = run_segsum(x, f, variant)
    check_sum(out, nseg, x, f)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("log2n", [20, 24])
def test_workload2_f16_geometric(log2n, variant):
    x, f = W.segsum_f16_geometric(1 << log2n)
    out, nseg = run_segsum(x, f, variant)
    worst = check_sum(out, nseg, x, f)
    print("workload 2 n=2^%d %s: segments %d, worst |err|/max(A,1) = %.3g" % (log2n, variant, nseg, worst))
    if log2n == 20:
        check_scan(run_segscan(x, f, variant), x, f)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("density", [0.0, 1e-7, 2e-5, 1e-3, 0.05])
@pytest.mark.parametrize("dtype", [np.int8, np.float16])
def test_sums_longer_than_one_round_of_workgroups(dtype, density, variant):
    """The segmented sum of 8- and 16-bit inputs has a kernel and tiles of its own on vectors longer than one round of
    workgroups (longer tiles: a wave streams through its span), with short tiles at both ends and full ones between
    them; in the ablation variant the same kernel scans its 32x32 tiles with vector instructions.  Densities from no flag at all (one segment: every tile hands on a plain sum, the one output waits for the
    carry of all tiles) over a handful of flags (most tiles without one) to a flag in every row."""
    rng = np.random.default_rng(78)
    full = B.mmv_tile_elems(B.MMV_OP_SEGSUM, B._DTYPES[torch.from_numpy(np.zeros(1, dtype=dtype)).dtype], 1 << 40)
    # beyond 768 tiles a small kernel turns the per-tile counts of segment starts into prefix sums first
    sizes = (512 * full + 1, 517 * full + 54321) + ((1100 * full + 77,) if density in (2e-5, 0.05) and dtype == np.int8 else ())
    for n in sizes:
        x = random_values(rng, n, dtype)
        f = W.uniform_density_flags(n, density, seed=n % 1000)
        print("long sum", dtype.__name__, density, variant, n, int(f.sum()), flush=True)
        out, nseg = run_segsum(x, f, variant)
        # This kernel speculates over whole chunks of 2048 values, not rows of 32: a sum is the difference of two
        # prefixes of its chunk, each rounded to fp32 at the size the prefix has there.  Over 2048 values from N(0,1)
        # a prefix stays below 512 (11 sigma), where one rounding is 2^-15 = 3e-5: the margin against max(A, 1) is
        # three such roundings instead of the 2e-5 that hold for speculation over rows.
        check_sum(out, nseg, x, f, margin=1e-4 if dtype == np.float16 else None)


def test_fp32_sums_without_matrix_cores_longer_than_one_round_of_workgroups():
    """The segmented sum of fp32 values in the variant without the matrix cores takes two chunks per wave (tiles twice
    as long as those of the other fp32 kernels), so its vectors need twice the length to go beyond one round of
    workgroups, to tiles taken by ticket and to tiles of growing and shrinking length."""
    rng = np.random.default_rng(79)
    full = 2 * B.mmv_tile_elems(B.MMV_OP_SEGSUM, B.MMV_F32_F32, 1 << 40)
    for n, density in ((512 * full + 1, 2e-5), (517 * full + 54321, 1e-3), (800 * full + 77, 0.05)):
        x = random_values(rng, n, np.float32)
        f = W.uniform_density_flags(n, density, seed=n % 1000)
        print("long fp32 sum", n, density, flush=True)
        out, nseg = run_segsum(x, f, "shuffle")
        check_sum(out, nseg, x, f)


def test_long_sum_with_an_output_array_that_is_too_short():
    """The streaming sum kernel writes its outputs as it goes, and the one per wave that waits for a carry at the end of
    the tile: none of them may land beyond the capacity the caller gave, and the count is the true one."""
    rng = np.random.default_rng(79)
    n = 520 * B.mmv_tile_elems(B.MMV_OP_SEGSUM, B.MMV_I8_I32, 1 << 40) + 77
    x = random_values(rng, n, np.int8)
    f = W.uniform_density_flags(n, 1e-4, seed=5)
    want = oracle.segsum(x, f)
    cap, guard = len(want) // 2, 4096
    whole = torch.full((cap + guard,), -77, dtype=torch.int32, device="cuda")
    nseg = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SEGSUM, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    B.mmv_segsum(dev(x), packed_dev(f), n=n, out=whole[:cap], nseg=nseg, variant="mfma", ws=ws)
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 0
    got = whole.cpu().numpy()
    assert int(nseg.item()) == len(want)
    assert np.array_equal(got[:cap], want[:cap])
    assert np.all(got[cap:] == -77), "an output beyond the capacity was written"


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("log2n", [22, 28])
def test_workload3_i8_uniform_len(log2n, variant):
    x, f = W.segscan_i8_uniform_len(1 << log2n)
    z = run_segscan(x, f, variant)
    check_scan(z, x, f)
    if log2n == 22:
        out, nseg = run_segsum(x, f, variant)
        check_sum(out, nseg, x, f)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("log2n", [22, 30])
def test_workload5_stress_three_regimes(log2n, variant):
    x, f = W.stress_f32_three_regimes(1 << log2n)
    xt = dev(x)
    z = run_segscan(x, f, variant, xt=xt)
    del xt
    worst = check_scan(z, x, f)      # gate, margin and the per-segment bound (the long segment: err <= 1e-4 max|ref|)
    # normwise error of the whole vector
    ref = oracle.segscan(x, f)
    peak = float(np.abs(ref).max())
    nerr = 0.0
    for a in range(0, len(ref), 1 << 26):
        nerr = max(nerr, float(np.abs(z[a:a + (1 << 26)].astype(np.float64) - ref[a:a + (1 << 26)]).max()))
    print("workload 5 n=2^%d %s: worst |err|/max(A,1) = %.3g, normwise %.3g" % (log2n, variant, worst, nerr / peak))
    assert nerr <= 1e-5 * peak, (nerr, peak)


def test_more_than_2_32_elements():
    """64-bit indexing: n just above 2^32 (int8 in, int32 out: 4 GiB + 16 GiB on the GPU)."""
    n = (1 << 32) + 70_001
    rng = np.random.default_rng(77)
    x = np.empty(n, dtype=np.int8)
    step = 1 << 28
    for a in range(0, n, step):
        x[a:min(n, a + step)] = rng.integers(-8, 9, size=min(n, a + step) - a, dtype=np.int8)
    f = np.zeros(n, dtype=np.uint8)
    f[rng.integers(0, n, size=n // 3000)] = 1
    f[[0, (1 << 32) - 1, (1 << 32), (1 << 32) + 1]] = 1
    xt, ft = dev(x), packed_dev(f)
    z = B.mmv_segscan(xt, ft, n=n)
    torch.cuda.synchronize()
    ref = oracle.segscan(x, f)
    got = z.cpu().numpy()
    del z
    for a in range(0, n, step):
        assert np.array_equal(got[a:a + step], ref[a:a + step]), a
    out, nseg = B.mmv_segsum(xt, ft, n=n, out=torch.empty(int(f.sum()) + 8, dtype=torch.int32, device="cuda"))
    sref = oracle.segsum(x, f)
    assert int(nseg.item()) == len(sref)
    assert np.array_equal(out.cpu().numpy()[:len(sref)], sref)


def test_two_streams_at_once_do_not_block_each_other():
    """Two calls in flight on different streams, each with its own workspace.  Both grids fit the device, so
    their workgroups take the tile of their own index (no ticket) and may start in pieces while the other
    call holds part of the chip; the status words tell whether any tile gave up waiting for a predecessor."""
    x1, f1 = W.segscan_i8_uniform_len(1 << 24, seed=31)
    x2, f2 = W.scan_sum_f32_bernoulli(1 << 23, p=1e-4, seed=32)
    a = (dev(x1), packed_dev(f1), torch.empty(len(x1), dtype=torch.int32, device="cuda"),
         B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, len(x1)))
    b = (dev(x2), packed_dev(f2), torch.empty(len(x2), dtype=torch.float32, device="cuda"),
         B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, len(x2)))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(5):
        B.mmv_segscan(a[0], a[1], z=a[2], ws=a[3], stream=s1)
        B.mmv_segscan(b[0], b[1], z=b[2], ws=b[3], stream=s2)
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(a[3]) == 0 and B.mmv_workspace_status(b[3]) == 0
    check_scan(a[2].cpu().numpy(), x1, f1)
    check_scan(b[2].cpu().numpy(), x2, f2)


def test_hip_graph_replay():
    """The calls enqueue only kernels (the workspace reset is a fill kernel), so they can be
    captured; every replay must give the eager result."""
    x, f = W.segscan_i8_uniform_len(1 << 22, seed=41)
    xt, ft = dev(x), packed_dev(f)
    n = len(x)
    z = torch.zeros(n, dtype=torch.int32, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    ref = oracle.segscan(x, f)
    B.mmv_segscan(xt, ft, z=z, ws=ws)                      # eager
    assert np.array_equal(z.cpu().numpy(), ref)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.mmv_segscan(xt, ft, z=z, ws=ws)
    for rep in range(4):
        z.zero_()                                          # the program's own eager work in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(z.cpu().numpy(), ref), rep
        assert B.mmv_workspace_status(ws) == 0


def test_status_codes_on_device_pointers():
    x = torch.zeros(1000, dtype=torch.int8, device="cuda")
    fl = torch.zeros(32, dtype=torch.int32, device="cuda")
    z = torch.zeros(1000, dtype=torch.int32, device="cuda")
    small = torch.zeros(256, dtype=torch.uint8, device="cuda")
    lib = B.load()
    st = lib.mmv_segscan(x.data_ptr(), fl.data_ptr(), 1000, z.data_ptr(), B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, 0,
                         small.data_ptr(), 256, None)
    assert st == 4                                          # workspace too small
    with pytest.raises(B.MmvError):
        B.mmv_segscan(x, fl, z=z, ws=small)
    st = lib.mmv_segscan(x.data_ptr() + 1, fl.data_ptr(), 999, z.data_ptr(), B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, 0,
                         small.data_ptr(), 256, None)
    assert st == 1                                          # misaligned values
