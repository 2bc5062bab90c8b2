"""mmv_segscan_static (the entry point that allocates nothing: its tile descriptors live in an array inside the
library's device code) against mmv_segscan on the same inputs, called through the C ABI: two calls in a row on
the shared array, the second with a smaller input, for integers (bit-exact) and floats (both within the
tolerance of the oracle comparison, and within twice that of each other)."""
import numpy as np
import pytest
import torch

from paper_2506_23906_amd import binding as B
from paper_2506_23906_amd import workloads as W
from parity_util import check_scan, dev, flags_dev

pytestmark = pytest.mark.gpu


def _both(x, f, packed, variant):
    """(result of mmv_segscan_static, result of mmv_segscan), raw C-ABI calls on preallocated buffers."""
    lib = B.load()
    n = len(x)
    xt, ft = dev(x), flags_dev(f, packed)
    dt, ff = B._DTYPES[xt.dtype], B._flag_fmt(ft)
    z_static = torch.full((n,), -3, dtype=B._OUT_DTYPE[dt], device="cuda")
    z_ws = torch.full((n,), -5, dtype=B._OUT_DTYPE[dt], device="cuda")
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, dt, ff, n)
    stream = int(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    st = lib.mmv_segscan_static(xt.data_ptr(), ft.data_ptr(), n, z_static.data_ptr(), dt, ff, B._VARIANTS[variant], stream)
    assert st == 0, st
    st = lib.mmv_segscan(xt.data_ptr(), ft.data_ptr(), n, z_ws.data_ptr(), dt, ff, B._VARIANTS[variant],
                         ws.data_ptr(), ws.numel(), stream)
    assert st == 0, st
    torch.cuda.synchronize()
    assert B.mmv_workspace_status(ws) == 0
    return z_static.cpu().numpy(), z_ws.cpu().numpy()


@pytest.mark.parametrize("variant", ["mfma", "shuffle"])
def test_static_scratch_two_calls_in_a_row_second_smaller(variant):
    tile = B.mmv_tile_elems()
    # a long input first (thousands of descriptors written), then shorter ones that reuse the same array
    for n, max_len in [(40 * tile + 4321, 4096), (3 * tile + 77, 512), (1000, 50), (1, 1)]:
        x, f = W.segscan_i8_uniform_len(n, max_len=max_len, seed=n)
        print("static scratch int8", variant, n, flush=True)
        a, b = _both(x, f, True, variant)
        assert np.array_equal(a, b), n
        check_scan(a, x, f)
    rng = np.random.default_rng(5)
    for n, density in [(20 * tile + 99, 0.0005), (2 * tile + 5, 0.0), (4097, 0.3)]:
        x = (rng.random(n, dtype=np.float32) * 2 - 1).astype(np.float32)
        f = W.uniform_density_flags(n, density, seed=n)
        print("static scratch fp32", variant, n, flush=True)
        a, b = _both(x, f, True, variant)
        check_scan(a, x, f)
        check_scan(b, x, f)
    # one flag byte per element: the packed copy of the flags lives in the array too
    for n in (300_000, 70_000):
        x, f = W.segscan_i8_uniform_len(n, max_len=300, seed=n)
        print("static scratch int8, byte flags", variant, n, flush=True)
        a, b = _both(x, f, False, variant)
        assert np.array_equal(a, b), n
        check_scan(a, x, f)


def test_static_scratch_limits_and_argument_errors():
    lib = B.load()
    x = torch.zeros(4096, dtype=torch.int8, device="cuda")
    fl = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    z = torch.zeros(4096, dtype=torch.int32, device="cuda")
    too_long = 64 << 20     # one flag byte per element: the packed flags alone would need 8 MiB
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_U8, too_long) > B.STATIC_SCRATCH_BYTES
    st = lib.mmv_segscan_static(x.data_ptr(), fl.data_ptr(), too_long, z.data_ptr(), B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, None)
    assert st == 6 and b"built-in scratch" in lib.mmv_status_string(st)    # rejected on the host: nothing was launched
    assert lib.mmv_segscan_static(x.data_ptr(), fl.data_ptr(), 4096, None, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, None) == 2
    assert lib.mmv_segscan_static(x.data_ptr(), fl.data_ptr(), 4096, z.data_ptr(), 9, B.MMV_FLAGS_U8, 0, None) == 1
    assert lib.mmv_segscan_static(x.data_ptr(), fl.data_ptr(), 0, z.data_ptr(), B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, None) == 0
    with pytest.raises(B.MmvError):
        B.mmv_segscan_static(x, fl, z, n=too_long)
