"""Quantization configuration search of the dense weights.  Test infrastructure only.

What is followed: the paper's "Quantization Configuration Search" section.  For every output
row and every group of its input columns, the step size s and the zero point z of the linear
asymmetric quantiser are chosen from a two-dimensional grid of narrowed ("truncated") ranges so
that rounding to nearest with clamping changes the weights least; the weak columns stay in
fp16 and take no part (they are neither in the range nor in the error).

The paper names the search and its objective and leaves the grid open.  The reading taken here
(the same one the library documents for owq_search_config):

    C          the non-weak columns of the group, w[c] the fp16 weights of the row there
    lo, hi     min and max of w over C;  R = hi - lo
               R == 0: lo = min(lo, 0), hi = max(hi, 0), R = hi - lo; still 0, or C empty:
               s = 1, z = 0, every code 0
    grid       i in [0, n_lo), j in [0, n_hi):
               lo_i = lo + a_i R,  hi_j = hi - b_j R,
               a_i = shrink * i / (n_lo - 1),  b_j = shrink * j / (n_hi - 1)   (0 if n == 1)
    candidate  s = fp16(max((hi_j - lo_i) / qmax, 2^-14)),  qmax = 2^bits - 1
               z = clamp(rint(-lo_i * (1 / s)), -2048, 2048)          (an integer)
    codes      q[c] = clamp(rint(w[c] * (1 / s)) + z, 0, qmax)
    error      E = sum over C of (w[c] - s (q[c] - z))^2
    choice     the candidate with the least E; among equal E the least i * n_hi + j

Where floating point decides an integer (s as an fp16 value, z, q), the decision is taken in
IEEE binary32 with one rounding per operation and round-half-even `rint`, the precision of the
GPU kernel: every such step below is a numpy float32 operation.  The error E that ranks the
candidates is evaluated in fp64 here (the kernel sums it in fp32; a test compares the two
choices through their errors, not through the index).

Pins (tests/test_oracle_search.py): weights that lie exactly on a quantiser grid, with and
without one outlier that only a narrowed range can absorb (closed-form s, z, codes and error);
the mirrored case; a weak column that must not move anything; the reported error against the
reconstruction error computed by the pinned dequantiser of owq_ref; optimality against nested
Python loops over the grid on tiny inputs; a 1 x 1 grid against plain min-max quantisation.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def cut_fractions(n: int, shrink: float) -> np.ndarray:
    """a_i (or b_j): fraction of the range cut from one end by grid point i, as float32."""
    if n == 1:
        return np.zeros(1, dtype=F32)
    return np.array([F32(np.float64(F32(shrink)) * i / (n - 1)) for i in range(n)], dtype=F32)


def candidate(lo: np.float32, hi: np.float32, a: np.float32, b: np.float32, qmax: int):
    """(s, inv, z) of one grid point; lo, hi float32 range of the group, a, b cut fractions."""
    r = F32(hi - lo)
    lo_i = F32(lo + F32(a * r))
    hi_j = F32(hi - F32(b * r))
    s32 = F32(F32(hi_j - lo_i) / F32(qmax))
    s32 = max(s32, F32(2.0 ** -14))
    s = F32(np.float16(s32))                      # the stored step size, exactly
    inv = F32(F32(1.0) / s)
    z = np.rint(F32(F32(-lo_i) * inv))
    z = F32(min(max(z, F32(-2048.0)), F32(2048.0)))
    if z == 0:
        z = F32(0.0)                              # no negative zero in the stored pattern
    return s, inv, z


def quantize(w32: np.ndarray, inv: np.float32, z: np.float32, qmax: int) -> np.ndarray:
    """Codes of float32 weights under (1/s, z): round to nearest, shift, clamp.  float32."""
    t = np.rint((w32 * inv).astype(F32)).astype(F32)
    return np.clip((t + z).astype(F32), F32(0.0), F32(qmax)).astype(F32)


def _range(w32: np.ndarray):
    """(lo, hi) of the kept weights after the degenerate-range rule, or None if nothing to search."""
    if w32.size == 0:
        return None
    lo, hi = F32(w32.min()), F32(w32.max())
    if hi == lo:
        lo, hi = min(lo, F32(0.0)), max(hi, F32(0.0))
        if hi == lo:
            return None
    return lo, hi


def grid(w32: np.ndarray, bits: int, n_lo: int, n_hi: int, shrink: float):
    """Every grid point for the kept float32 weights w32: yields (index, s, z, q, E)."""
    qmax = (1 << bits) - 1
    lo, hi = _range(w32)
    a, b = cut_fractions(n_lo, shrink), cut_fractions(n_hi, shrink)
    w64 = w32.astype(np.float64)
    for i in range(n_lo):
        for j in range(n_hi):
            s, inv, z = candidate(lo, hi, a[i], b[j], qmax)
            q = quantize(w32, inv, z, qmax)
            e = float(np.sum((w64 - np.float64(s) * (q.astype(np.float64) - np.float64(z))) ** 2))
            yield i * n_hi + j, s, z, q, e


def search_group(w16: np.ndarray, keep: np.ndarray, bits: int, n_lo: int, n_hi: int, shrink: float):
    """One (row, group).  w16: fp16 weights of the group; keep: True at non-weak columns.

    Returns (s fp16, z fp16, codes uint8 (0 at weak columns), error fp64, choice int).
    """
    codes = np.zeros(w16.size, dtype=np.uint8)
    w32 = np.asarray(w16, dtype=np.float16).astype(F32)[keep]
    if _range(w32) is None:
        return np.float16(1.0), np.float16(0.0), codes, 0.0, 0
    best = None
    for idx, s, z, q, e in grid(w32, bits, n_lo, n_hi, shrink):
        if best is None or e < best[4]:
            best = (idx, s, z, q, e)
    idx, s, z, q, e = best
    codes[keep] = q.astype(np.uint8)
    return np.float16(s), np.float16(z), codes, e, idx


def search_config(w16: np.ndarray, weak_idx, bits: int, group_size: int,
                  n_lo: int, n_hi: int, shrink: float):
    """Whole matrix.  w16 [d_out, d_in] fp16.  Returns scale, zero (fp16 [d_out, G]),
    codes (uint8 [d_out, d_in]), err (fp64 [d_out, G]), choice (int32 [d_out, G])."""
    w16 = np.asarray(w16, dtype=np.float16)
    d_out, d_in = w16.shape
    g = d_in if group_size == 0 else group_size
    n_g = (d_in + g - 1) // g
    keep = np.ones(d_in, dtype=bool)
    keep[np.asarray(weak_idx, dtype=np.int64)] = False
    scale = np.empty((d_out, n_g), dtype=np.float16)
    zero = np.empty((d_out, n_g), dtype=np.float16)
    codes = np.empty((d_out, d_in), dtype=np.uint8)
    err = np.empty((d_out, n_g), dtype=np.float64)
    choice = np.empty((d_out, n_g), dtype=np.int32)
    for r in range(d_out):
        for gi in range(n_g):
            c0, c1 = gi * g, min(d_in, (gi + 1) * g)
            s, z, q, e, ch = search_group(w16[r, c0:c1], keep[c0:c1], bits, n_lo, n_hi, shrink)
            scale[r, gi], zero[r, gi], err[r, gi], choice[r, gi] = s, z, e, ch
            codes[r, c0:c1] = q
    return scale, zero, codes, err, choice


def candidate_errors(w16_group: np.ndarray, keep: np.ndarray, bits: int,
                     n_lo: int, n_hi: int, shrink: float) -> np.ndarray:
    """fp64 error of every grid point of one (row, group), [n_lo * n_hi]; inf if nothing to search."""
    w32 = np.asarray(w16_group, dtype=np.float16).astype(F32)[keep]
    out = np.full(n_lo * n_hi, np.inf)
    if _range(w32) is None:
        return out
    for idx, _, _, _, e in grid(w32, bits, n_lo, n_hi, shrink):
        out[idx] = e
    return out


def search_group_plain(w16: np.ndarray, keep: np.ndarray, bits: int, n_lo: int, n_hi: int, shrink: float):
    """The same search with every decision taken from the plain definition in binary64: the cut
    fractions, the narrowed range and the step size before its one rounding to fp16 are exact
    quotients, the zero point is rint(-lo_i / s) and a code rint(w / s) + z with a true division
    (not a multiplication by a rounded reciprocal).  Shares no arithmetic with the functions above
    except the fp16 rounding of s, which is what the layer stores.  A test counts how often the
    binary32 reading above decides differently from this one.

    Returns (s fp16, z fp16, codes uint8 (0 at weak columns), error fp64, choice int)."""
    codes = np.zeros(w16.size, dtype=np.uint8)
    w = np.asarray(w16, dtype=np.float16).astype(np.float64)[keep]
    if w.size == 0:
        return np.float16(1.0), np.float16(0.0), codes, 0.0, 0
    lo, hi = float(w.min()), float(w.max())
    if hi == lo:
        lo, hi = min(lo, 0.0), max(hi, 0.0)
        if hi == lo:
            return np.float16(1.0), np.float16(0.0), codes, 0.0, 0
    qmax = (1 << bits) - 1
    rng = hi - lo
    best = None
    for i in range(n_lo):
        a = 0.0 if n_lo == 1 else shrink * i / (n_lo - 1)
        for j in range(n_hi):
            b = 0.0 if n_hi == 1 else shrink * j / (n_hi - 1)
            lo_i, hi_j = lo + a * rng, hi - b * rng
            s = float(np.float16(max((hi_j - lo_i) / qmax, 2.0 ** -14)))
            z = float(min(max(np.rint(-lo_i / s), -2048.0), 2048.0)) + 0.0
            q = np.clip(np.rint(w / s) + z, 0.0, float(qmax))
            e = float(np.sum((w - s * (q - z)) ** 2))
            if best is None or e < best[4]:
                best = (i * n_hi + j, s, z, q, e)
    idx, s, z, q, e = best
    codes[keep] = q.astype(np.uint8)
    return np.float16(s), np.float16(z), codes, e, idx
