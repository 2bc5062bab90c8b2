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
* ``scan_alg`` - Algorithm "Scan in MMV-RAM" (Sec. 4).
* ``compress``, ``diff``, ``scd`` - Algorithm SCD (Sec. 4.1): DIFF o COMPRESS o SCAN.
* ``revert``, ``sscr`` - Algorithm SSCR (Sec. 4.1).
* ``revspec_lemma`` - the filter-matrix construction of the REVSPEC lemma
  (appendix, block-recursive algorithm).
* ``revert_spec_simple`` - Algorithm "Revert Speculative Prefix Sums"
  (appendix), with its per-block shortcuts.
* ``block_recursive_segscan`` - Algorithm "Block-recursive segmented scan"
  (appendix): SegScan / Recurse / BlockSegScan / UpdateFirstSegment.

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
  block start", which also holds for the block's first position itself; adding
  the filled value there would double it.  The first position of every shifted
  block is excluded, as matrix B_s of Algorithm Scan does.
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


def B(s):
    """Identity with an all-ones first row (Algorithm Scan)."""
    m = np.eye(s, dtype=np.int64)
    m[0, :] = 1
    return m


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


def gathers(x, s):
    """GATHERS: last element of every s-block."""
    return _pad(x, s)[s - 1::s].copy()


def scatters(z, zs, s):
    """SCATTERS: write element i of zs to the last position of the i-th s-block of z."""
    z = z.copy()
    z[s - 1::s] = zs[:len(z[s - 1::s])]
    return z


def fills(x, s):
    """FILLS: copy the first element of every s-block over the whole block."""
    xp = _pad(x, s)
    return np.repeat(xp[0::s], s)


# ---- unsegmented scan --------------------------------------------------------

def scan_alg(x, s):
    """Algorithm Scan: local block scans, recursive scan of block lasts, B_s carry add."""
    n = len(x)
    z = matmul_op(x, U(s))
    if n <= s:
        return z[:n]
    xs = gathers(z, s)
    zs = scan_alg(xs, s)
    z = scatters(z, zs, s)
    tail = matmul_op(z[s - 1:], B(s))
    z[s - 1:] = tail[:len(z) - (s - 1)]
    return z[:n]


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
    """Speculative block scans reverted block by block with the shortcut cases."""
    n = len(x)
    z = matmul_op(x, U(s))
    fbar = matmul_op((np.asarray(f) != 0).astype(np.int64), U(s))
    xp = _pad(x, s)
    for b in range(0, len(z), s):
        zs, fb = z[b:b + s], fbar[b:b + s]
        mu = fb[s - 1]
        if mu == 0 or (mu == 1 and fb[0] == 1):
            continue                          # speculation already correct
        if mu == s:
            zs[:] = xp[b:b + s]               # s segments of one element
            continue
        spec = zs.copy()                      # offsets come from the speculative values
        for idx in range(int(fb[0]) + 1, int(mu) + 1):
            offset = int((fb < idx).sum()) - 1
            zs -= (fb == idx).astype(np.int64) * int(spec[offset])
    return z[:n]


# ---- block-recursive segmented scan ------------------------------------------------

def _block_seg_scan(x, f, s):
    xbar = matmul_op(x, U(s))
    fbar = matmul_op(f, U(s))
    return revspec(xbar, fbar, s)


def _update_first_segment(z, f, s):
    n = len(z)
    fbar = matmul_op(f, U(s))
    fstart = fills(fbar, s)
    m = ((fbar - fstart) == 0).astype(np.int64)
    m &= 1 - _pad(f, s)
    m[0::s] = 0                                # see module header
    w = fills(_pad(z, s), s) * m
    return (_pad(z, s) + w)[:n]


def _recurse(z, f, s):
    if len(z) <= s:
        return z
    z, f = _pad(z, s).copy(), _pad(f, s)
    fbar = matmul_op(f, U(s))
    fs = (gathers(fbar, s) != 0).astype(np.int64)
    zs = gathers(z, s)
    zs = _block_seg_scan(zs, fs, s)
    zs = _recurse(zs, fs, s)
    z = scatters(z, zs, s)
    z[s - 1:] = _update_first_segment(z[s - 1:], f[s - 1:], s)
    return z


def block_recursive_segscan(x, f, s):
    """SegScan(x, f; s): speculative block scans, REVSPEC, recursion on block lasts."""
    n = len(x)
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    xp = _pad(x, s)
    fp = _pad((np.asarray(f) != 0).astype(np.int64), s)
    z = _block_seg_scan(xp, fp, s)
    return _recurse(z, fp, s)[:n]
