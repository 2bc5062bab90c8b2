"""Seeded synthetic inputs for the segmented-operation workloads.

This module only draws random inputs (values, segment-start flags, COO
triples) and converts between the two flag encodings.  It holds none of the
method's arithmetic, so both the tests' CPU oracle and the GPU library can be
fed from it without sharing anything else.

The five main workloads mirror the shapes the paper measures on: uniformly random
segment-start flags over a range of densities (Sec. 5.2.1, density sweep) and
the row-length structure of sparse matrices (Sec. 5.2.1 / 5.2.3), which are
not available offline; these generators stand in for them.

Every generator takes ``n`` (or the matrix size) so that a scaled-down twin
with the same distribution can be produced for fast parity tests.
"""
from __future__ import annotations

import numpy as np

SEEDS = {
    "scan_sum_f32_bernoulli": 2390601,
    "segsum_f16_geometric": 2390602,
    "segscan_i8_uniform_len": 2390603,
    "spmv_coo_zipf": 2390604,
    "stress_f32_three_regimes": 2390605,
    "blocked_sparse_attention": 2390606,
}


# ---- flag helpers -------------------------------------------------------------

def flags_from_lengths(lengths: np.ndarray, n: int) -> np.ndarray:
    """One byte per element, 1 at the first element of every segment.

    ``lengths`` are consecutive segment lengths; segments that would start at
    or beyond ``n`` are dropped and the last one is truncated.
    """
    f = np.zeros(n, dtype=np.uint8)
    if n == 0:
        return f
    starts = np.cumsum(lengths, dtype=np.int64) - lengths
    f[starts[starts < n]] = 1
    f[0] = 1
    return f


def draw_lengths_until(rng, n: int, draw) -> np.ndarray:
    """Call ``draw(rng, k)`` for batches of k lengths until their sum reaches n."""
    out, total = [], 0
    while total < n:
        k = max(1024, int((n - total) / 8) + 16)
        part = draw(rng, k).astype(np.int64)
        out.append(part)
        total += int(part.sum())
    return np.concatenate(out)


def pack_flags(flags_u8: np.ndarray) -> np.ndarray:
    """Bit-pack flags: bit (i mod 32) of 32-bit word floor(i/32), least significant bit first.

    The result has ceil(n/32) words; bits beyond n are zero.
    """
    n = flags_u8.shape[0]
    nwords = (n + 31) // 32
    b = np.packbits(flags_u8 != 0, bitorder="little")
    buf = np.zeros(nwords * 4, dtype=np.uint8)
    buf[:b.shape[0]] = b
    return buf.view("<u4")


def unpack_flags(words: np.ndarray, n: int) -> np.ndarray:
    return np.unpackbits(words.view(np.uint8), bitorder="little")[:n].astype(np.uint8)


# ---- the five workloads ---------------------------------------------------------

def scan_sum_f32_bernoulli(n: int = 1 << 16, p: float = 1.0 / 64, seed: int | None = None):
    """fp32 values ~ U(-1, 1); flags ~ Bernoulli(p) with flag[0] = 1."""
    rng = np.random.default_rng(SEEDS["scan_sum_f32_bernoulli"] if seed is None else seed)
    x = (rng.random(n, dtype=np.float32) * np.float32(2) - np.float32(1)).astype(np.float32)
    f = (rng.random(n) < p).astype(np.uint8)
    if n:
        f[0] = 1
    return x, f


def segsum_f16_geometric(n: int = 1 << 24, mean_len: float = 32.0, seed: int | None = None):
    """fp16 values ~ N(0, 1) (rounded to fp16); segment lengths geometric with the given mean."""
    rng = np.random.default_rng(SEEDS["segsum_f16_geometric"] if seed is None else seed)
    x = rng.standard_normal(n, dtype=np.float32).astype(np.float16)
    lengths = draw_lengths_until(rng, n, lambda r, k: r.geometric(1.0 / mean_len, size=k))
    return x, flags_from_lengths(lengths, n)


def segscan_i8_uniform_len(n: int = 1 << 28, max_len: int = 4096, seed: int | None = None):
    """int8 values uniform in [-8, 8]; segment lengths uniform in [1, max_len]."""
    rng = np.random.default_rng(SEEDS["segscan_i8_uniform_len"] if seed is None else seed)
    x = rng.integers(-8, 9, size=n, dtype=np.int8)
    lengths = draw_lengths_until(rng, n, lambda r, k: r.integers(1, max_len + 1, size=k))
    return x, flags_from_lengths(lengths, n)


def zipf_truncated(rng, size: int, s: float, kmax: int) -> np.ndarray:
    """Samples from P(k) proportional to k^-s on {1..kmax} by inverse CDF."""
    k = np.arange(1, kmax + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    return (np.searchsorted(cdf, rng.random(size), side="left") + 1).astype(np.int64)


def zipf_truncated_mean(s: float, kmax: int) -> float:
    k = np.arange(1, kmax + 1, dtype=np.float64)
    w = k ** (-s)
    return float((k * w).sum() / w.sum())


def spmv_coo_zipf(n_rows: int = 1 << 20, n_cols: int = 1 << 20, target_nnz: int = 1 << 25,
                  s: float = 1.5, cap: int = 1 << 14, seed: int | None = None):
    """Row-sorted COO matrix with Zipf(s) row lengths capped at ``cap`` and empty rows.

    A row is empty with probability 1 - q, otherwise its length is a truncated
    Zipf draw; q is set so that the expected number of non-zeros is
    ``target_nnz``.  Column indices are uniform (duplicates allowed); values and
    the dense vector are N(0, 1) in fp32.  Returns (row, col, val, x).
    """
    rng = np.random.default_rng(SEEDS["spmv_coo_zipf"] if seed is None else seed)
    cap = min(cap, max(1, n_cols))
    q = min(1.0, target_nnz / (n_rows * zipf_truncated_mean(s, cap)))
    nonempty = rng.random(n_rows) < q
    lengths = np.zeros(n_rows, dtype=np.int64)
    lengths[nonempty] = zipf_truncated(rng, int(nonempty.sum()), s, cap)
    nnz = int(lengths.sum())
    row = np.repeat(np.arange(n_rows, dtype=np.int32), lengths)
    col = rng.integers(0, n_cols, size=nnz, dtype=np.int32)
    val = rng.standard_normal(nnz, dtype=np.float32)
    x = rng.standard_normal(n_cols, dtype=np.float32)
    return row, col, val, x


def stress_f32_three_regimes(n: int = 1 << 30, max_len: int = 64, seed: int | None = None):
    """fp32 values ~ U(-1, 1).  First half: every flag set; then one segment over a
    quarter of the vector; the last quarter has segment lengths uniform in [1, max_len]."""
    rng = np.random.default_rng(SEEDS["stress_f32_three_regimes"] if seed is None else seed)
    x = np.empty(n, dtype=np.float32)
    step = 1 << 24
    for a in range(0, n, step):                      # in pieces: keeps the temporaries small
        b = min(n, a + step)
        x[a:b] = rng.random(b - a, dtype=np.float32) * np.float32(2) - np.float32(1)
    f = np.zeros(n, dtype=np.uint8)
    half, quarter = n // 2, n // 4
    f[:half] = 1
    tail0 = half + quarter
    if n - tail0 > 0:
        lengths = draw_lengths_until(rng, n - tail0, lambda r, k: r.integers(1, max_len + 1, size=k))
        f[tail0:] = flags_from_lengths(lengths, n - tail0)
    if n:
        f[0] = 1
        if half < n:
            f[half] = 1
    return x, f


def uniform_density_flags(n: int, density: float, seed: int) -> np.ndarray:
    """Uniformly random flags at a given density (the paper's density sweep), flag[0] = 1."""
    rng = np.random.default_rng(seed)
    f = (rng.random(n) < density).astype(np.uint8)
    if n:
        f[0] = 1
    return f


# ---- CSR inputs (Sec. 4.3, Algorithm "MMV-RAM CSR SpMV"; Sec. 5.2.3 workloads) --------------------

def csr_rowptr(row: np.ndarray, n_rows: int) -> np.ndarray:
    """Row pointers (n_rows + 1 int32 entries) of a row-sorted COO index vector: a format conversion."""
    counts = np.bincount(np.asarray(row, dtype=np.int64), minlength=n_rows)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    return rowptr.astype(np.int32)


def blocked_sparse_attention(n: int = 1 << 16, block: int = 64, n_random: int = 2, n_global: int = 2,
                             n_window: int = 3, seed: int | None = None):
    """Blocked sparse-attention matrix in CSR form, after the synthetic matrices of Sec. 5.2.3.

    The n x n matrix is cut into blocks of ``block`` x ``block``; the paper states the size
    (65,536), two blocks of global attention, three blocks of window attention, block sizes
    {2, 4, 16, 64} and {2, 4, 8} random blocks, and nothing else.  Reading taken here: block row
    i holds the first ``n_global`` block columns, the ``n_window`` block columns centred on i
    (clipped at the borders) and ``n_random`` block columns drawn uniformly (a draw that hits a
    block already present adds nothing); the first ``n_global`` block rows are full.  Every entry
    of a present block is a non-zero ~ N(0, 1); x ~ N(0, 1).  Returns (rowptr, col, val, x).
    """
    if n % block:
        raise ValueError("n must be a multiple of the block size")
    rng = np.random.default_rng(SEEDS["blocked_sparse_attention"] + 1000 * block + n_random
                                if seed is None else seed)
    nb = n // block
    half = n_window // 2
    inner = np.arange(block, dtype=np.int64)
    cols, lens = [], np.empty(nb, dtype=np.int64)
    for i in range(nb):
        if i < n_global:
            bc = np.arange(nb, dtype=np.int64)
        else:
            window = np.arange(i - half, i - half + n_window, dtype=np.int64)
            window = window[(window >= 0) & (window < nb)]
            bc = np.unique(np.concatenate([np.arange(min(n_global, nb), dtype=np.int64), window,
                                           rng.integers(0, nb, size=n_random)]))
        one_row = (bc[:, None] * block + inner[None, :]).ravel()
        cols.append(np.tile(one_row, block))
        lens[i] = one_row.shape[0]
    col = np.concatenate(cols).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.repeat(lens, block), out=rowptr[1:])
    val = rng.standard_normal(col.shape[0], dtype=np.float32)
    x = rng.standard_normal(n, dtype=np.float32)
    return rowptr.astype(np.int32), col, val, x
