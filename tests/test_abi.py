"""Host-only checks of the C-ABI boundary: the library loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

from conftest import ROOT


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mmvseg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmv_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_agree():
    from paper_2506_23906_amd import binding
    assert _declared_symbols() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol(libmmvseg_path):
    lib = ctypes.CDLL(libmmvseg_path)
    for name in _declared_symbols():
        assert hasattr(lib, name), name


def test_host_only_entry_points(libmmvseg_path):
    from paper_2506_23906_amd import binding as B
    lib = B.load()
    big = 1 << 40
    tile = B.mmv_tile_elems(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, big)
    assert tile % 2048 == 0 and tile >= 8192
    for dt in (B.MMV_F16_F32, B.MMV_BF16_F32, B.MMV_F32_F32):
        t = B.mmv_tile_elems(B.MMV_OP_SEGSCAN, dt, big)
        assert t % 2048 == 0 and 0 < t <= tile
    small = B.mmv_tile_elems(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, 1000)                # short inputs: small tiles
    assert small % 2048 == 0 and small <= tile
    assert B.mmv_tile_elems(B.MMV_OP_SEGSCAN, 9, big) == 0 and B.mmv_tile_elems(99, B.MMV_I8_I32, big) == 0
    assert lib.mmv_status_string(0) == b"ok"
    assert lib.mmv_status_string(4).startswith(b"workspace")
    # header + one 8-byte descriptor per tile, rounded to 256 bytes
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, 1) == 512
    n = 1 << 28
    tile = B.mmv_tile_elems(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, n)
    scan = B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    # one 8-byte descriptor per tile: at least n / (largest tile), and the end of the vector is cut finer
    assert 256 + (n // tile) * 8 <= scan <= 256 + 4 * (n // tile) * 8 and scan % 256 == 0
    ssum = B.mmv_workspace_bytes(B.MMV_OP_SEGSUM, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    # descriptors, 8 bytes of counts per tile, 4 bytes of counts per wave span (8 waves to a tile): 48 bytes per tile
    # (each of the three arrays rounded to 256 bytes); the sum of bytes has longer tiles than the scan, cut finer at both ends
    tsum = B.mmv_tile_elems(B.MMV_OP_SEGSUM, B.MMV_I8_I32, n)
    assert tsum >= tile and 256 + (n // tsum) * 48 <= ssum <= 256 + 4 * (n // tsum) * 48 + 3 * 256 and ssum % 256 == 0
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_U8, n) == scan + n // 8
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN, 7, B.MMV_FLAGS_U8, n) == 0      # bad dtype
    assert B.mmv_workspace_bytes(99, B.MMV_I8_I32, B.MMV_FLAGS_U8, n) == 0         # bad op
    # the un-fused compositions need room for their intermediate vectors (4 bytes per element each)
    assert B.mmv_workspace_bytes(B.MMV_OP_SCAN, B.MMV_I8_I32, B.MMV_FLAGS_U8, n) == scan
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSUM_SCD, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n) >= 8 * n
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN_SSCR, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n) >= 9 * n
    assert B.mmv_workspace_bytes(B.MMV_OP_SPMV_CSR, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n) == 0
    csr = B.mmv_spmv_csr_workspace_bytes(1 << 20, 1 << 25)
    assert csr % 256 == 0 and (1 << 25) // 8 + 4 * (1 << 20) <= csr <= 16 << 20
    assert B.mmv_spmv_csr_workspace_bytes(1 << 31, 4) == 0
    # COMPRESS: a wave owns 16 or 64 mask words of 64 bits, in one, two or four groups, by the length of the mask
    assert B.mmv_tile_elems(B.MMV_OP_COMPRESS, B.MMV_I8_I32, 1 << 20) == 8 * 64 * 16
    assert B.mmv_tile_elems(B.MMV_OP_COMPRESS, B.MMV_I8_I32, 1 << 24) == 8 * 64 * 64
    assert B.mmv_tile_elems(B.MMV_OP_COMPRESS, B.MMV_I8_I32, 1 << 26) == 8 * 64 * 64 * 2
    assert B.mmv_tile_elems(B.MMV_OP_COMPRESS, B.MMV_I8_I32, n) == 8 * 64 * 64 * 4


def test_argument_errors_are_caught_on_the_host(libmmvseg_path):
    """None of these reaches a kernel launch, so they run without a GPU."""
    from paper_2506_23906_amd import binding as B
    lib = B.load()
    OK, INVALID, NULL, WORKSPACE = 0, 1, 2, 4
    a16 = 0x10000   # fake, aligned, never dereferenced on these paths
    # n == 0 is a valid no-op
    assert lib.mmv_segscan(None, None, 0, None, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, None, 0, None) == OK
    assert lib.mmv_segscan(None, None, 0, None, 9, B.MMV_FLAGS_U8, 0, None, 0, None) == INVALID
    assert lib.mmv_spmv_coo(0, 0, 0, None, None, None, None, None, 0, None, 0, None) == OK
    # null pointers
    assert lib.mmv_segscan(None, a16, 10, a16, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 4096, None) == NULL
    assert lib.mmv_segscan(a16, a16, 10, None, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 4096, None) == NULL
    assert lib.mmv_segscan(a16, a16, 10, a16 * 2, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, None, 4096, None) == NULL
    assert lib.mmv_segsum(a16, a16, 10, a16, 10, None, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 4096, None) == NULL
    # misaligned pointers, bad enums
    assert lib.mmv_segscan(a16 + 4, a16, 10, a16 * 2, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_segscan(a16, a16, 10, a16 * 2, 5, B.MMV_FLAGS_U8, 0, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_segscan(a16, a16, 10, a16 * 2, B.MMV_I8_I32, 2, 0, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_segscan(a16, a16, 10, a16 * 2, B.MMV_I8_I32, B.MMV_FLAGS_U8, 2, a16 << 4, 4096, None) == INVALID
    # output may alias the input only when both are fp32
    assert lib.mmv_segscan(a16, a16 * 2, 10, a16, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 4096, None) == INVALID
    # workspace too small / misaligned
    assert lib.mmv_segscan(a16, a16, 10, a16 * 2, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_segscan(a16, a16, 10, a16 * 2, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, (a16 << 4) + 16, 4096, None) == WORKSPACE
    assert lib.mmv_spmv_coo(1 << 31, 4, 4, a16, a16, a16, a16, a16, 0, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_spmv_coo(4, 4, 4, a16, None, a16, a16, a16, 0, a16 << 4, 4096, None) == NULL
    # the primitives, the compositions and the CSR entry point
    assert lib.mmv_scan(None, 0, None, B.MMV_I8_I32, 0, None, 0, None) == OK
    assert lib.mmv_scan(a16, 10, None, B.MMV_I8_I32, 0, a16 << 4, 4096, None) == NULL
    assert lib.mmv_scan(a16, 10, a16, B.MMV_I8_I32, 0, a16 << 4, 4096, None) == INVALID      # aliasing
    assert lib.mmv_scan(a16, 10, a16 * 2, B.MMV_I8_I32, 0, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_compress(a16, a16, 10, a16 * 2, 10, None, B.MMV_FLAGS_U8, a16 << 4, 4096, None) == NULL
    assert lib.mmv_compress(a16, a16, 10, a16 * 2, 10, a16 + 4, B.MMV_FLAGS_U8, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_compress(a16, a16, 10, a16 * 2, 10, a16, 2, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_compress(a16, a16, 10, a16 * 2, 10, a16, B.MMV_FLAGS_U8, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_diff(a16, 10, a16, B.MMV_ELEM_I32, None) == INVALID                         # aliasing
    assert lib.mmv_diff(a16, 10, a16 * 2, 2, None) == INVALID
    assert lib.mmv_diff(None, 0, None, B.MMV_ELEM_F32, None) == OK
    assert lib.mmv_revert(a16, None, a16, 10, 3, a16, B.MMV_ELEM_I32, None) == NULL
    assert lib.mmv_revert(a16, a16, a16, 10, 3, a16, 7, None) == INVALID
    assert lib.mmv_segsum_scd(a16, a16, 10, a16, 10, None, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 1 << 20, None) == NULL
    assert lib.mmv_segsum_scd(a16, a16, 10, a16, 10, a16, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_segscan_sscr(a16, a16, 10, a16 * 2, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_segscan_sscr(a16, a16, 10, a16, B.MMV_I8_I32, B.MMV_FLAGS_U8, 0, a16 << 4, 1 << 20, None) == INVALID
    # the un-fused routes subtract (DIFF, REVERT): not for the group of bytes under exclusive or
    assert lib.mmv_segsum_scd(a16, a16, 10, a16, 10, a16, B.MMV_U8_XOR, B.MMV_FLAGS_U8, 0, a16 << 4, 1 << 20, None) == 3
    assert lib.mmv_segscan_sscr(a16, a16, 10, a16 * 2, B.MMV_U8_XOR, B.MMV_FLAGS_U8, 0, a16 << 4, 1 << 20, None) == 3
    assert B.mmv_workspace_bytes(B.MMV_OP_SEGSCAN, B.MMV_U8_XOR, B.MMV_FLAGS_PACKED32, 1 << 20) > 0
    assert lib.mmv_spmv_csr(0, 0, 0, None, None, None, None, None, 0, None, 0, None) == OK
    assert lib.mmv_spmv_csr(4, 4, 4, None, a16, a16, a16, a16, 0, a16 << 4, 1 << 20, None) == NULL
    assert lib.mmv_spmv_csr(4, 4, 1 << 31, a16, a16, a16, a16, a16, 0, a16 << 4, 1 << 20, None) == INVALID
    assert lib.mmv_spmv_csr(4, 4, 4, a16, a16, a16, a16, a16, 0, a16 << 4, 16, None) == WORKSPACE
    # SpMV in two steps: the same checks in both steps
    assert lib.mmv_spmv_coo_prepare(0, 0, 0, None, None, None, 0, None) == OK
    assert lib.mmv_spmv_coo_prepare(4, 4, 4, a16, None, a16 << 4, 4096, None) == NULL
    assert lib.mmv_spmv_coo_prepare(4, 4, 4, a16 + 4, a16, a16 << 4, 4096, None) == INVALID       # alignment
    assert lib.mmv_spmv_coo_prepare(1 << 31, 4, 4, a16, a16, a16 << 4, 4096, None) == INVALID
    assert lib.mmv_spmv_coo_prepare(4, 4, 4, a16, a16, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_spmv_coo_run(0, 0, 0, None, None, None, None, None, 0, None, 0, None) == OK
    assert lib.mmv_spmv_coo_run(4, 4, 4, a16, a16, None, a16, a16, 0, a16 << 4, 4096, None) == NULL
    assert lib.mmv_spmv_coo_run(4, 4, 4, a16, a16, a16, a16, a16, 7, a16 << 4, 4096, None) == INVALID   # variant
    assert lib.mmv_spmv_coo_run(4, 4, 4, a16, a16, a16, a16, a16, 0, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_spmv_csr_prepare(0, 0, 0, None, None, None, 0, None) == OK
    assert lib.mmv_spmv_csr_prepare(4, 4, 4, None, a16, a16 << 4, 1 << 20, None) == NULL
    assert lib.mmv_spmv_csr_prepare(4, 4, 1 << 31, a16, a16, a16 << 4, 1 << 20, None) == INVALID
    assert lib.mmv_spmv_csr_prepare(4, 4, 4, a16, a16, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_spmv_csr_run(0, 0, 0, None, None, None, None, None, 0, None, 0, None) == OK
    assert lib.mmv_spmv_csr_run(4, 4, 4, a16, a16, a16, None, a16, 0, a16 << 4, 1 << 20, None) == NULL
    assert lib.mmv_spmv_csr_run(4, 4, 4, a16, a16, a16, a16, a16, 0, (a16 << 4) + 16, 1 << 20, None) == WORKSPACE  # alignment of d_ws
    assert lib.mmv_spmv_csr_run(4, 4, 4, a16, a16, a16, a16, a16, 0, a16 << 4, 16, None) == WORKSPACE
    assert lib.mmv_stream_copy(a16, 24, a16, 32, None) == INVALID
    assert lib.mmv_workspace_status(None, None, None) == NULL
    assert lib.mmv_gather_reference(0, None, None, 0, None, None, None) == OK
    assert lib.mmv_gather_reference(8, None, a16, 4, a16, a16, None) == NULL
    assert lib.mmv_gather_reference(8, a16 + 4, a16, 4, a16, a16, None) == INVALID
    assert lib.mmv_gather_reference(8, a16, a16, 0, a16, a16, None) == INVALID


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2506_23906_amd import binding as B
    import pytest
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libmmvseg.so"))
    with pytest.raises(B.MmvError):
        B.load()
