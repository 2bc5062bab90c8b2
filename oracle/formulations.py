"""The paper's other routes to the segmented scan / sum, in plain numpy.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Nothing here is fast;
everything works on Python integers or int64 so that results are exact, and is
used to pin the sequential definitions in ``mmvseg_oracle.c`` against
formulations that share no code with them:

* ``definitional_segscan`` - z(i) = sum of x(k) for k from the start of i's
  segment to i, start(i) = max{k <= i : k == 0 or f(k) == 1}; O(n^2), Python
  integers (what Problem 2.1 of Sec. 2 unrolls to).
* ``matmul_op`` - MATMUL(x, A) of Sec. 1.1 (Notation): x viewed as a
  ceil(n/s) x s row-major matrix, zero padded, times A, flattened.
* ``scan_alg`` - the recursion behind Algorithm "Scan in MMV-RAM" (Sec. 4): scans of s-blocks as products
  with U_s, the same scan applied to the block totals, every block shifted by the total before it.
* ``compress``, ``diff``, ``scd`` - Algorithm SCD (Sec. 4.1): DIFF o COMPRESS o SCAN.
* ``revert``, ``sscr`` - Algorithm SSCR (Sec. 4.1).
* ``revspec_lemma`` - the filter-matrix construction of the REVSPEC lemma
  (appendix, block-recursive algorithm).
* ``revert_spec_simple`` - what Algorithm "Revert Speculative Prefix Sums" (appendix) reaches, from its
  definition: inside a block every position loses the speculative value just before the start of its segment.
* ``block_recursive_segscan`` - the recursion of Algorithm "Block-recursive segmented scan" (appendix): blocks
  scanned speculatively and reverted, the (last value, any flag) pairs of the blocks scanned by the same
  function, the result of the block before added to the positions ahead of a block's first flag.
These three are written from what the algorithms compute (the lemma, Problem 2.1, the recursion on block
aggregates), on 2-D block views; they do not follow the printed instruction sequences.

Readings taken where the printed pseudo-code cannot be right as it stands:

* REVERT (Sec. 4.1) as printed compares the flag scan with idx+1 for idx from
  0; with f(0) = 1 that would subtract w(0) from the first segment and turn
  the paper's own worked example into (-2, 0, ...).  Here an element whose
  inclusive flag count is k >= 2 gets w(k-2) subtracted and k == 1 is left
  alone; all corrections apply to one output vector.
* "Revert Speculative Prefix Sums" updates z_s in place inside a parallel loop
  while reading z_s(offset); offsets are read from the un-reverted speculative
  scan.
* UpdateFirstSegment builds its mask from "flag count equals the count at the
  block start", which read literally also selects the first position of the shifted
  block, whose value is the carry itself.  Here the carry of the block before goes to
  the positions of a block ahead of its first flag, nothing else.
* COMPRESS inside the SCD/SSCR proof masks with the end markers f^- and writes
  to the 1-based position g(i), i.e. output index g(i) - 1.
"""
from __future__ import annotations

import numpy as np


# ---- definitions -----------------------------------------------------------

def definitional_segscan(x, f):
    """O(n^2) unrolled definition on Python integers."""
    x = [int(v) for v in x]
    f = [1 if v else 0 for v in f]
    n = len(x)
    z = []
    for i in range(n):
        start = 0
        for k in range(i, -1, -1):
            if k == 0 or f[k] == 1:
                start = k
                break
        z.append(sum(x[start:i + 1]))
    return z


def definitional_segsum(x, f):
    z = definitional_segscan(x, f)
    n = len(z)
    return [z[i] for i in range(n) if i == n - 1 or f[i + 1]]


# ---- matrices of the paper -------------------------------------------------

def U(s):
    """Upper-triangular all-ones matrix, diagonal included (Sec. 1.1)."""
    return np.triu(np.ones((s, s), dtype=np.int64))


def D(s):
    """Bidiagonal difference matrix, 1 on the diagonal, -1 above it (Eq. for D_s)."""
    return np.eye(s, dtype=np.int64) - np.eye(s, k=1, dtype=np.int64)


def _pad(x, s):
    x = np.asarray(x, dtype=np.int64)
    r = (-len(x)) % s
    return np.concatenate([x, np.zeros(r, dtype=np.int64)]) if r else x


def matmul_op(x, A):
    """MATMUL(x, A): ceil(n/s) x s row-major view (zero padded) times A; padded length."""
    s = A.shape[0]
    xp = _pad(x, s)
    return (xp.reshape(-1, s) @ A).reshape(-1)


# ---- unsegmented scan --------------------------------------------------------

def scan_alg(x, s):
    """Blocked scan: every s-block scanned by the product with U_s, the block totals scanned by the same function,
    every block shifted by the scanned total of the block before it."""
    n = len(x)
    local = matmul_op(x, U(s)).reshape(-1, s)          # row b = inclusive scan of block b alone
    if local.shape[0] > 1:
        upto = scan_alg(local[:, -1], s)               # inclusive scan of the block totals
        local[1:] += upto[:-1, None]
    return local.reshape(-1)[:n]


# ---- SCD / SSCR ----------------------------------------------------------------

def end_markers(f):
    """f^-: f shifted left by one with a 1 appended (segment ends)."""
    f = np.asarray(f, dtype=np.int64)
    return np.concatenate([f[1:], [1]]) if len(f) else f


def compress(x, f):
    """Entries of x where f is 1, placed by the 1-based scan of the mask."""
    x = np.asarray(x, dtype=np.int64)
    f = (np.asarray(f) != 0).astype(np.int64)
    g = np.cumsum(f) * f            # non-zero entries: 1-based output position
    out = np.zeros(int(f.sum()), dtype=np.int64)
    for i in range(len(x)):
        if g[i]:
            out[g[i] - 1] = x[i]
    return out


def diff(z):
    """z_diff(i) = z(i) - z(i-1) with z(-1) = 0."""
    z = np.asarray(z, dtype=np.int64)
    return z - np.concatenate([[0], z[:-1]]) if len(z) else z


def diff_matmul(z, s):
    """DIFF through D_s on s-blocks plus the vector fix of block boundaries (Sec. 4.1)."""
    n = len(z)
    if n == 0:
        return np.asarray(z, dtype=np.int64)
    zp = _pad(z, s)
    # (row) x D_s yields out(j) = a(j) - a(j-1) for j >= 1 and out(0) = a(0)
    d = matmul_op(zp, D(s))
    for b in range(1, len(zp) // s):
        d[b * s] -= zp[b * s - 1]
    return d[:n]


def scd(x, f, s):
    """Segmented sum = DIFF(COMPRESS(SCAN(x), f^-))."""
    if len(x) == 0:
        return np.zeros(0, dtype=np.int64)
    xhat = scan_alg(x, s)
    return diff(compress(xhat, end_markers(f)))


def revert(xhat, fhat, w):
    """REVERT with the off-by-one reading stated in the module header."""
    z = np.asarray(xhat, dtype=np.int64).copy()
    for idx in range(len(w)):
        z -= (np.asarray(fhat) == idx + 2).astype(np.int64) * int(w[idx])
    return z


def sscr(x, f, s):
    """Segmented scan = REVERT(COMPRESS(SCAN x, f^-), SCAN x, SCAN f)."""
    n = len(x)
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    f = (np.asarray(f) != 0).astype(np.int64)
    f[0] = 1                       # position 0 always opens a segment
    xhat = scan_alg(x, s)
    fhat = scan_alg(f, s)
    w = compress(xhat, end_markers(f))
    return revert(xhat, fhat, w)


# ---- per-block revert ---------------------------------------------------------

def revspec_lemma(xbar, fbar):
    """REVSPEC on one block through the filter matrix Q and update vector u."""
    s = len(xbar)
    u = [0] * s
    for j in range(s):
        for i in range(j):
            q = (fbar[i] != fbar[i + 1]) and (fbar[j] == fbar[i + 1])
            if q:
                u[j] |= int(xbar[i])      # at most one i qualifies: the OR is a select
    return np.array([int(xbar[j]) - u[j] for j in range(s)], dtype=np.int64)


def _count_selected(xbar, fbar):
    """Number of i < j that satisfy the lemma's two conditions, per j (must be <= 1)."""
    s = len(xbar)
    return [sum(1 for i in range(j) if fbar[i] != fbar[i + 1] and fbar[j] == fbar[i + 1])
            for j in range(s)]


def revspec(xbar, fbar, s):
    """REVSPEC vector instruction: the lemma applied to every s-block."""
    out = np.empty(len(xbar), dtype=np.int64)
    for b in range(0, len(xbar), s):
        out[b:b + s] = revspec_lemma(xbar[b:b + s], fbar[b:b + s])
    return out


def revert_spec_simple(x, f, s):
    """Speculative block scans with the mis-speculation taken back, from the definition of the result: a position
    whose segment starts inside its block at position p >= 1 loses the speculative value at p - 1; positions
    ahead of the block's first flag, and segments that start at the block's first position, keep theirs.
    (Blocks without a flag, or with their only flag in front, therefore stay as they are, and a block whose
    every position is flagged turns back into its input: the shortcut cases of the appendix algorithm.)"""
    n = len(x)
    spec = matmul_op(x, U(s)).reshape(-1, s)
    flags = _pad((np.asarray(f) != 0).astype(np.int64), s).reshape(-1, s)
    pos = np.arange(s)
    start = np.maximum.accumulate(np.where(flags != 0, pos, -1), axis=1)     # last flagged position at or before each position
    before = np.where(start >= 1, np.take_along_axis(spec, np.maximum(start - 1, 0), axis=1), 0)
    return (spec - before).reshape(-1)[:n]


# ---- block-recursive segmented scan ------------------------------------------------

def block_recursive_segscan(x, f, s):
    """Segmented scan by recursion on blocks of s: each block scanned on its own (speculation through U_s, taken back
    by REVSPEC as the lemma defines it), the blocks' (last value, any flag) pairs scanned by this same function,
    and the scanned value of the block before added wherever a block continues it (ahead of its first flag)."""
    n = len(x)
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    xp = _pad(x, s)
    fp = _pad((np.asarray(f) != 0).astype(np.int64), s)
    z = revspec(matmul_op(xp, U(s)), matmul_op(fp, U(s)), s).reshape(-1, s)
    fb = fp.reshape(-1, s)
    if z.shape[0] > 1:
        carried = block_recursive_segscan(z[:, -1], fb.any(axis=1), s)      # segmented scan over the blocks
        open_ahead = np.cumsum(fb, axis=1) == 0                              # positions with no flag at or before them
        z[1:] += np.where(open_ahead[1:], carried[:-1, None], 0)
    return z.reshape(-1)[:n]
