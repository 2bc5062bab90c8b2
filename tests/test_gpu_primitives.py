"""GPU parity of the stand-alone primitives (SCAN, COMPRESS, DIFF, REVERT of Sec. 4.1) and of the
un-fused compositions SCD and SSCR, each against its plain definition in the CPU oracle.

Integers are bit-exact.  Floating point: SCAN within tol * max(A_i, 1) with A_i = scan of |x| in
fp64 (same rule as the segmented scan); DIFF and REVERT do one fp32 subtraction per element, so
they are within one rounding of the fp64 result; SCD / SSCR on floats carry the rounding of the
global speculative prefix, so their bound is relative to the scan of |x| over the whole vector.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import TOL, dev, flags_dev, packed_dev, random_values

pytestmark = pytest.mark.gpu
TILE = 65536
SIZES = [1, 2, 31, 32, 33, 1000, 2048, 4097, 16384, TILE - 1, TILE, TILE + 1, 3 * TILE + 777, 1_000_003]


def sync_ok(ws):
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 0


# ---- SCAN ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
@pytest.mark.parametrize("dtype", [np.int8, np.float16, np.float32])
def test_scan_sizes(dtype, variant):
    rng = np.random.default_rng(61)
    for n in SIZES:
        x = random_values(rng, n, dtype)
        dt = B._DTYPES[dev(x).dtype]
        ws = B.new_workspace(B.MMV_OP_SCAN, dt, B.MMV_FLAGS_PACKED32, n)
        z = B.mmv_scan(dev(x), n=n, variant=variant, ws=ws)
        sync_ok(ws)
        got, ref = z.cpu().numpy(), oracle.scan(x)
        if dtype == np.int8:
            assert np.array_equal(got, ref), (n, variant)
        else:
            A = oracle.scan(np.abs(x.astype(np.float64)))
            assert (np.abs(got.astype(np.float64) - ref) <= TOL[np.dtype(dtype)] * np.maximum(A, 1.0)).all(), (n, variant)


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_scan_at_the_border_between_one_round_of_workgroups_and_several(dtype):
    """mmv_scan of 16- and 32-bit inputs has tiles of its own length (3 and 2 chunks per wave): exactly one round of
    512 full tiles (equal tiles, every workgroup its own index), one element more (graded tiles, tickets), one less."""
    rng = np.random.default_rng(65)
    dt = B._DTYPES[dev(np.zeros(1, dtype)).dtype]
    full = B.mmv_tile_elems(B.MMV_OP_SCAN, dt, 1 << 40)
    assert full == (3 if dtype == np.float16 else 2) * 16384
    for n in (512 * full - 1, 512 * full, 512 * full + 1):
        x = random_values(rng, n, dtype)
        for variant in ("mfma", "shuffle"):
            z = B.mmv_scan(dev(x), n=n, variant=variant)
            torch.cuda.synchronize()
            got, ref = z.cpu().numpy(), oracle.scan(x)
            A = oracle.scan(np.abs(x.astype(np.float64)))
            assert (np.abs(got.astype(np.float64) - ref) <= TOL[np.dtype(dtype)] * np.maximum(A, 1.0)).all(), (n, variant)


def test_scan_wraps_and_is_segscan_without_flags():
    n = 20_000_000
    x = np.full(n, 127, dtype=np.int8)
    z = B.mmv_scan(dev(x)).cpu().numpy()
    assert np.array_equal(z, oracle.scan(x)) and z[-1] < 0
    rng = np.random.default_rng(62)
    x = rng.integers(-128, 128, size=5 * TILE + 5, dtype=np.int8)
    f = np.zeros(len(x), dtype=np.uint8)
    assert np.array_equal(B.mmv_scan(dev(x)).cpu().numpy(), B.mmv_segscan(dev(x), packed_dev(f), n=len(x)).cpu().numpy())


def test_scan_in_place_fp32_and_bf16():
    rng = np.random.default_rng(63)
    x = random_values(rng, 2 * TILE + 9, np.float32)
    xt = dev(x)
    B.mmv_scan(xt, z=xt)
    A = oracle.scan(np.abs(x.astype(np.float64)))
    assert (np.abs(xt.cpu().numpy().astype(np.float64) - oracle.scan(x)) <= 1e-4 * np.maximum(A, 1.0)).all()
    xb = torch.from_numpy(x).to(torch.bfloat16)
    z = B.mmv_scan(xb.cuda()).cpu().numpy()
    xr = xb.to(torch.float32).numpy()
    A = oracle.scan(np.abs(xr.astype(np.float64)))
    assert (np.abs(z.astype(np.float64) - oracle.scan(xr)) <= 1e-2 * np.maximum(A, 1.0)).all()


# ---- COMPRESS ---------------------------------------------------------------------------------

@pytest.mark.parametrize("packed", [True, False])
def test_compress_sizes_and_densities(packed):
    rng = np.random.default_rng(64)
    ctile = B.mmv_tile_elems(B.MMV_OP_COMPRESS, B.MMV_I8_I32, 1)
    for n in [1, 2, 63, 64, 65, 4095, 4096, 4097, ctile - 1, ctile, ctile + 1, 3 * ctile + 777, 1_000_003]:
        for density in (0.0, 0.001, 0.03, 0.5, 1.0):
            x = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
            m = (rng.random(n) < density).astype(np.uint8)
            if not packed:
                m = m * rng.integers(1, 256, size=n).astype(np.uint8)        # any non-zero byte means "set"
            ref = oracle.compress(x, m)
            out = torch.full((n + 3,), -7, dtype=torch.int32, device="cuda")
            ws = B.new_workspace(B.MMV_OP_COMPRESS, B.MMV_I8_I32, B._flag_fmt(flags_dev(m, packed)), n)
            _, count = B.mmv_compress(dev(x), flags_dev(m, packed), n, out=out, ws=ws)
            sync_ok(ws)
            assert int(count.item()) == len(ref), (n, density)
            got = out.cpu().numpy()
            assert np.array_equal(got[:len(ref)], ref), (n, density)
            assert (got[len(ref):] == -7).all()                              # nothing written beyond the count


def test_compress_worked_example_positions_capacity_and_floats(golden_sec2):
    g = golden_sec2
    out, count = B.mmv_compress(dev(np.array(g["x"], dtype=np.int32)), dev(np.array(g["f"], dtype=np.uint8)), 8)
    assert out.cpu().numpy()[:int(count.item())].tolist() == g["compress"]
    # positions: x = None compresses 0 .. n-1
    m = np.zeros(200_000, dtype=np.uint8)
    pos = [0, 1, 31, 32, 63, 64, 4095, 4096, 32767, 32768, 199_999]
    m[pos] = 1
    out, count = B.mmv_compress(None, packed_dev(m), len(m))
    assert out.cpu().numpy()[:int(count.item())].tolist() == pos
    # bits beyond n in the last mask word are ignored
    words = W.pack_flags(np.ones(40, dtype=np.uint8)).copy()
    words[-1] = 0xFFFFFFFF
    out, count = B.mmv_compress(None, torch.from_numpy(words.view(np.int32)).cuda(), 40)
    assert int(count.item()) == 40 and out.cpu().numpy()[:40].tolist() == list(range(40))
    # capacity smaller than the count: the count is still the true one
    rng = np.random.default_rng(65)
    xf = rng.standard_normal(100_000).astype(np.float32)
    mm = (rng.random(100_000) < 0.5).astype(np.uint8)
    ref = oracle.compress(xf, mm)
    out = torch.full((1000,), 5.0, dtype=torch.float32, device="cuda")
    _, count = B.mmv_compress(dev(xf), packed_dev(mm), 100_000, out=out)
    assert int(count.item()) == len(ref) and np.array_equal(out.cpu().numpy(), ref[:1000])
    _, count = B.mmv_compress(dev(xf), packed_dev(mm), 0)
    assert int(count.item()) == 0


# ---- DIFF, REVERT -----------------------------------------------------------------------------

def test_diff():
    rng = np.random.default_rng(66)
    for n in [1, 2, 3, 4, 5, 255, 256, 257, 1023, 1024, 1025, 100_003]:
        x = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
        z = torch.full((n + 5,), 9, dtype=torch.int32, device="cuda")
        B.mmv_diff(dev(x), n=n, z=z)
        got = z.cpu().numpy()
        assert np.array_equal(got[:n], oracle.diff(x)) and (got[n:] == 9).all(), n
        xf = rng.standard_normal(n).astype(np.float32)
        got = B.mmv_diff(dev(xf)).cpu().numpy()
        ref = oracle.diff(xf)
        assert np.array_equal(got, ref.astype(np.float32)), n      # one correctly rounded fp32 subtraction
    x = rng.integers(-128, 128, size=300_000, dtype=np.int8)
    assert np.array_equal(B.mmv_diff(B.mmv_scan(dev(x))).cpu().numpy(), x.astype(np.int32))   # DIFF inverts SCAN


def _sscr_inputs(x, f):
    g = (f != 0).astype(np.int8)
    g[0] = 1
    xhat = oracle.scan(x)
    fhat = oracle.scan(g)
    w = oracle.compress(xhat.astype(np.int32) if x.dtype == np.int8 else xhat.astype(np.float32),
                        np.concatenate([f[1:], [1]]).astype(np.uint8))
    return xhat, fhat, w


def test_revert():
    rng = np.random.default_rng(67)
    for n, density in [(1, 1.0), (5, 0.5), (1000, 0.1), (1024, 0.0), (100_003, 0.01), (100_003, 1.0)]:
        x = rng.integers(-128, 128, size=n, dtype=np.int8)
        f = W.uniform_density_flags(n, density, 5)
        xhat, fhat, w = _sscr_inputs(x, f)
        ref = oracle.revert(xhat, fhat, w)
        assert np.array_equal(ref, oracle.segscan(x, f))
        got = B.mmv_revert(dev(xhat), dev(fhat), dev(w)).cpu().numpy()
        assert np.array_equal(got[:n], ref), (n, density)
        xt = dev(xhat)
        B.mmv_revert(xt, dev(fhat), dev(w), z=xt)                    # in place
        assert np.array_equal(xt.cpu().numpy(), ref)
    xf = rng.standard_normal(50_000).astype(np.float32)
    f = W.uniform_density_flags(50_000, 0.02, 6)
    xhat = np.cumsum(xf, dtype=np.float32)
    _, fhat, _ = _sscr_inputs(np.zeros(50_000, dtype=np.int8), f)
    w = oracle.compress(xhat, np.concatenate([f[1:], [1]]).astype(np.uint8))
    got = B.mmv_revert(dev(xhat), dev(fhat), dev(w)).cpu().numpy()
    assert np.array_equal(got, oracle.revert(xhat, fhat, w).astype(np.float32))
    # a count that points beyond w subtracts nothing (and nothing is read out of bounds)
    got = B.mmv_revert(dev(np.arange(8, dtype=np.int32)), dev(np.array([1, 2, 3, 4, 900, 2, -5, 0], dtype=np.int32)),
                       dev(np.array([10, 20], dtype=np.int32))).cpu().numpy()
    assert got[:8].tolist() == [0, 1 - 10, 2 - 20, 3, 4, 5 - 10, 6, 7]


# ---- SCD and SSCR, the un-fused compositions ---------------------------------------------------------

@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
def test_scd_and_sscr_int8(variant, packed):
    rng = np.random.default_rng(68)
    for n in [1, 2, 33, 1000, 4097, TILE + 1, 3 * TILE + 777, 1_000_003]:
        for density in (0.0, 0.001, 0.05, 1.0):
            x = rng.integers(-128, 128, size=n, dtype=np.int8)
            f = W.uniform_density_flags(n, density, 7)
            if n > 1:
                f[0] = 0                                              # position 0 opens a segment anyway
            ft = flags_dev(f * (1 if packed else 200), packed)
            ff = B._flag_fmt(ft)
            z = B.mmv_segscan_sscr(dev(x), ft, n=n, variant=variant)
            torch.cuda.synchronize()
            assert np.array_equal(z.cpu().numpy(), oracle.segscan(x, f)), (n, density)
            ref = oracle.segsum(x, f)
            out = torch.full((n + 2,), -7, dtype=torch.int32, device="cuda")
            _, nseg = B.mmv_segsum_scd(dev(x), ft, n=n, out=out, variant=variant,
                                       ws=B.new_workspace(B.MMV_OP_SEGSUM_SCD, B.MMV_I8_I32, ff, n))
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert int(nseg.item()) == len(ref) and np.array_equal(got[:len(ref)], ref), (n, density)
            assert (got[len(ref):] == -7).all()


def test_scd_and_sscr_worked_example_wrap_and_capacity(golden_sec2):
    g = golden_sec2
    x, f = np.array(g["x"], dtype=np.int8), np.array(g["f"], dtype=np.uint8)
    assert B.mmv_segscan_sscr(dev(x), dev(f)).cpu().numpy().tolist() == g["segscan"]
    out, nseg = B.mmv_segsum_scd(dev(x), dev(f))
    assert out.cpu().numpy()[:int(nseg.item())].tolist() == g["segsum"]
    # the speculative scan wraps around 2^31 before the flags; Z/2^32 keeps the results exact
    n = 18_000_000
    x = np.full(n, 127, dtype=np.int8)
    f = np.zeros(n, dtype=np.uint8)
    f[[0, 17_000_000, 17_500_000]] = 1
    assert np.array_equal(B.mmv_segscan_sscr(dev(x), packed_dev(f)).cpu().numpy(), oracle.segscan(x, f))
    out = torch.full((2,), -7, dtype=torch.int32, device="cuda")       # room for two of the three sums
    _, nseg = B.mmv_segsum_scd(dev(x), packed_dev(f), out=out)
    assert int(nseg.item()) == 3 and np.array_equal(out.cpu().numpy(), oracle.segsum(x, f)[:2])


def test_scd_and_sscr_fp32_error_follows_the_global_prefix():
    """Floats are not a group: the un-fused routes subtract two global prefixes, so the error of a
    result is bounded by the rounding of the prefix (a few ulp of the scan of |x| over the whole
    vector), not of the segment.  Bound: 1e-4 * max(scan of |x| up to i, 1)."""
    x, f = W.scan_sum_f32_bernoulli(1 << 20, seed=9)
    z = B.mmv_segscan_sscr(dev(x), packed_dev(f)).cpu().numpy()
    G = oracle.scan(np.abs(x.astype(np.float64)))
    assert (np.abs(z.astype(np.float64) - oracle.segscan(x, f)) <= 1e-4 * np.maximum(G, 1.0)).all()
    out, nseg = B.mmv_segsum_scd(dev(x), packed_dev(f))
    ref = oracle.segsum(x, f)
    ends = np.flatnonzero(np.concatenate([f[1:], [1]]))
    assert int(nseg.item()) == len(ref)
    assert (np.abs(out.cpu().numpy()[:len(ref)].astype(np.float64) - ref) <= 1e-4 * np.maximum(G[ends], 1.0)).all()


# ---- the sizes the benchmark report times --------------------------------------------------------------

def test_scan_and_compress_at_2p28():
    n = 1 << 28
    x, f = W.segscan_i8_uniform_len(n)
    z = B.mmv_scan(dev(x))
    torch.cuda.synchronize()
    ref = oracle.scan(x)
    got = z.cpu().numpy()
    del z
    step = 1 << 26
    for a in range(0, n, step):
        assert np.array_equal(got[a:a + step], ref[a:a + step]), a
    m = W.uniform_density_flags(n, 0.01, 78)
    out, count = B.mmv_compress(None, packed_dev(m), n, out=torch.empty(int(m.sum()) + 8, dtype=torch.int32, device="cuda"))
    pos = np.flatnonzero(m)
    assert int(count.item()) == len(pos) and np.array_equal(out.cpu().numpy()[:len(pos)], pos.astype(np.int32))
    # values through the same mask: COMPRESS(scan, mask) picks the scan at the marked positions
    out, count = B.mmv_compress(dev(ref), packed_dev(m), n, out=torch.empty(len(pos) + 8, dtype=torch.int32, device="cuda"))
    assert int(count.item()) == len(pos) and np.array_equal(out.cpu().numpy()[:len(pos)], ref[pos])


def test_compress_long_masks_with_many_selected_entries():
    """Masks of 2^26 positions and more take four groups of words per wave; beyond one round of workgroups the tiles
    are taken by ticket.  Dense masks (the wave visits every word), a mask that is dense in one half and sparse in
    the other, a ragged end."""
    rng = np.random.default_rng(70)
    for n, density in (((1 << 26) + 12345, 1.0), ((1 << 27) + (1 << 26) + 777, 0.5), ((1 << 26) + 64 * 4096 * 3 + 5, None)):
        if density is None:
            m = np.concatenate([(rng.random(n // 2) < 0.4), (rng.random(n - n // 2) < 0.002)]).astype(np.uint8)
        else:
            m = (rng.random(n) < density).astype(np.uint8) if density < 1.0 else np.ones(n, dtype=np.uint8)
        pos = np.flatnonzero(m).astype(np.int32)
        out = torch.full((len(pos) + 5,), -7, dtype=torch.int32, device="cuda")
        ws = B.new_workspace(B.MMV_OP_COMPRESS, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        print("long mask", n, density, len(pos), flush=True)
        _, count = B.mmv_compress(None, packed_dev(m), n, out=out, ws=ws)
        sync_ok(ws)
        got = out.cpu().numpy()
        assert int(count.item()) == len(pos), (n, density)
        assert np.array_equal(got[:len(pos)], pos), (n, density)
        assert (got[len(pos):] == -7).all()


@pytest.mark.parametrize("density", [1e-3, 1e-2])
def test_scd_and_sscr_at_2p26(density):
    n = 1 << 26
    rng = np.random.default_rng(69)
    x = rng.integers(-8, 9, size=n, dtype=np.int8)
    f = W.uniform_density_flags(n, density, 78)
    xt, ft = dev(x), packed_dev(f)
    z = B.mmv_segscan_sscr(xt, ft)
    torch.cuda.synchronize()
    assert np.array_equal(z.cpu().numpy(), oracle.segscan(x, f))
    del z
    ref = oracle.segsum(x, f)
    out, nseg = B.mmv_segsum_scd(xt, ft, out=torch.empty(len(ref) + 8, dtype=torch.int32, device="cuda"))
    assert int(nseg.item()) == len(ref) and np.array_equal(out.cpu().numpy()[:len(ref)], ref)
