"""Pins of the configuration-search oracle (oracle/search.py) against closed forms, symmetries,
the pinned dequantiser and nested loops on tiny inputs.  CPU only."""
import itertools

import numpy as np
import pytest

from oracle import owq_ref, search


def grid_weights(n=128, step=0.5, qmax=7, seed=0):
    """Weights that lie exactly on {0, step, ..., qmax*step}, every level present."""
    rng = np.random.default_rng(seed)
    q = rng.integers(0, qmax + 1, size=n)
    q[: qmax + 1] = np.arange(qmax + 1)
    return (q * step).astype(np.float16), q.astype(np.uint8)


def test_exact_grid_is_found_without_truncation():
    # Weights on s0*(q - z0) with s0 a power of two: min-max quantisation reproduces them (paper,
    # "Quantization Configuration Search": the search minimises the weight difference; 0 is minimal).
    w, q = grid_weights()
    w = (w.astype(np.float32) - 1.5).astype(np.float16)            # s0 = 0.5, z0 = 3
    s, z, codes, e, ch = search.search_group(w, np.ones(128, bool), 3, 4, 4, 0.3)
    assert (float(s), float(z), e, ch) == (0.5, 3.0, 0.0, 0)
    assert np.array_equal(codes, q)


def test_outlier_is_truncated_closed_form():
    # 127 weights on {0..7}*0.5 and one at 4.0.  With b = (0, 0.125, 0.25) the middle candidate has
    # hi' = 4 - 0.125*4 = 3.5, s = 0.5, z = 0: only the outlier errs, by 0.5, so E = 0.25.
    # Min-max (s = 4/7) misplaces most of the 127 grid weights: E is far larger.
    w, q = grid_weights()
    w[8], q[8] = 4.0, 7
    s, z, codes, e, ch = search.search_group(w, np.ones(128, bool), 3, 1, 3, 0.25)
    assert (float(s), float(z), ch) == (0.5, 0.0, 1)
    assert e == pytest.approx(0.25, abs=0)
    assert np.array_equal(codes, q)
    e_minmax = search.candidate_errors(w, np.ones(128, bool), 3, 1, 3, 0.25)[0]
    assert e_minmax > 1.0


def test_mirrored_outlier_cuts_the_lower_end():
    # The same weights negated: the cut must come from the lower end (index i), z = 7, codes 7 - q.
    w, q = grid_weights()
    w[8], q[8] = 4.0, 7
    wn = (-w.astype(np.float32)).astype(np.float16)
    s, z, codes, e, ch = search.search_group(wn, np.ones(128, bool), 3, 3, 1, 0.25)
    assert (float(s), float(z), ch, e) == (0.5, 7.0, 1, 0.25)
    assert np.array_equal(codes, 7 - q)
    # a grid over the upper end only cannot absorb it
    _, _, _, e_hi, _ = search.search_group(wn, np.ones(128, bool), 3, 1, 3, 0.25)
    assert e_hi > 1.0
    # index order is i * n_hi + j: with a 3 x 2 grid the winner (i = 1, j = 0) is index 2
    assert search.search_group(wn, np.ones(128, bool), 3, 3, 2, 0.25)[4] == 2


def test_weak_columns_take_no_part():
    # A huge value at a weak column changes neither range nor error; its code is 0.
    w, q = grid_weights()
    keep = np.ones(128, bool)
    ref = search.search_group(w, keep, 3, 3, 3, 0.25)
    w2 = w.copy()
    w2[20] = 1000.0
    keep2 = keep.copy()
    keep2[20] = False
    got = search.search_group(w2, keep2, 3, 3, 3, 0.25)
    assert (got[0], got[1], got[4]) == (ref[0], ref[1], ref[4])
    assert got[2][20] == 0
    m = np.arange(128) != 20
    assert np.array_equal(got[2][m], ref[2][m])
    assert got[3] == 0.0 and float(got[0]) == 0.5


def test_degenerate_groups():
    keep = np.ones(16, bool)
    s, z, codes, e, ch = search.search_group(np.zeros(16, np.float16), keep, 4, 3, 3, 0.2)
    assert (float(s), float(z), e, ch) == (1.0, 0.0, 0.0, 0) and not codes.any()
    s, z, codes, e, ch = search.search_group(np.zeros(16, np.float16), ~keep, 4, 3, 3, 0.2)
    assert (float(s), float(z), e, ch) == (1.0, 0.0, 0.0, 0) and not codes.any()
    # a constant group: the range is widened to reach 0, the constant sits on its upper end
    s, z, codes, e, ch = search.search_group(np.full(16, 1.5, np.float16), keep, 4, 1, 1, 0.0)
    assert (float(s), float(z), e) == (0.0999755859375, 0.0, pytest.approx(16 * (1.5 - 15 * 0.0999755859375) ** 2))
    assert (codes == 15).all()
    s, z, codes, e, ch = search.search_group(np.full(16, -3.0, np.float16), keep, 3, 1, 1, 0.0)
    assert float(z) == 7.0 and not codes.any()


def test_one_by_one_grid_is_min_max_quantisation():
    rng = np.random.default_rng(3)
    w = rng.normal(0, 0.02, size=256).astype(np.float16)
    s, z, codes, e, ch = search.search_group(w, np.ones(256, bool), 4, 1, 1, 0.4)
    lo, hi = float(w.min()), float(w.max())
    assert float(s) == pytest.approx((hi - lo) / 15, rel=2 ** -10)
    assert abs(float(z) - (-lo / float(s))) <= 0.5 + 1e-3
    assert codes.min() == 0 and codes.max() == 15 and ch == 0


@pytest.mark.parametrize("bits,gs", [(3, 0), (4, 128), (3, 256)])
def test_reported_error_is_the_reconstruction_error(bits, gs):
    # The error the search reports equals |W - Deq(codes, s, z)|^2 over the non-weak columns, with the
    # dequantiser that the linear-layer oracle is pinned through.
    rng = np.random.default_rng(bits + gs)
    d_out, d_in = 6, 512
    w = rng.normal(0, 0.02, size=(d_out, d_in)).astype(np.float16)
    w[rng.integers(0, d_out, 5), rng.integers(0, d_in, 5)] *= 8
    weak = np.sort(rng.choice(d_in, 7, replace=False))
    scale, zero, codes, err, choice = search.search_config(w, weak, bits, gs, 4, 5, 0.3)
    deq = owq_ref.dequantize_dense(codes, scale, zero, gs, weak)
    d = w.astype(np.float64) - deq
    d[:, weak] = 0.0
    g = d_in if gs == 0 else gs
    by_group = (d ** 2).reshape(d_out, d_in // g, g).sum(axis=2)
    assert np.allclose(by_group, err, rtol=1e-12, atol=0)
    assert not codes[:, weak].any()
    assert codes.max() <= (1 << bits) - 1


def test_choice_is_optimal_by_nested_loops():
    # Tiny input, every grid point evaluated with plain Python floats from the stored outputs' formulas:
    # no candidate reconstructs the weights better than the chosen one.
    rng = np.random.default_rng(11)
    w = rng.normal(0, 1, size=24).astype(np.float16)
    w[3] = 9.0
    bits, n_lo, n_hi, shrink = 3, 3, 4, 0.3
    s, z, codes, e, ch = search.search_group(w, np.ones(24, bool), bits, n_lo, n_hi, shrink)
    lo, hi = float(w.min()), float(w.max())
    best = None
    for i, j in itertools.product(range(n_lo), range(n_hi)):
        a = float(np.float32(shrink)) * i / (n_lo - 1)
        b = float(np.float32(shrink)) * j / (n_hi - 1)
        lo_i, hi_j = lo + a * (hi - lo), hi - b * (hi - lo)
        sc = float(np.float16((hi_j - lo_i) / 7))
        zc = round(-lo_i / sc)
        tot = 0.0
        for x in w.astype(np.float64):
            q = min(max(round(x / sc) + zc, 0), 7)
            tot += (x - sc * (q - zc)) ** 2
        if best is None or tot < best[0] - 1e-12:
            best = (tot, i * n_hi + j, sc, zc)
    assert e == pytest.approx(best[0], rel=1e-6)
    assert (ch, float(s), float(z)) == (best[1], best[2], best[3])
    assert e < search.candidate_errors(w, np.ones(24, bool), bits, n_lo, n_hi, shrink)[0]


def test_groups_are_searched_independently():
    rng = np.random.default_rng(5)
    w = rng.normal(0, 0.02, size=(3, 512)).astype(np.float16)
    full = search.search_config(w, [], 4, 128, 3, 3, 0.2)
    for gi in range(4):
        part = search.search_config(w[:, 128 * gi:128 * (gi + 1)], [], 4, 0, 3, 3, 0.2)
        assert np.array_equal(full[0][:, gi], part[0][:, 0])
        assert np.array_equal(full[1][:, gi], part[1][:, 0])
        assert np.array_equal(full[2][:, 128 * gi:128 * (gi + 1)], part[2])
    # ragged last group
    r = search.search_config(w[:, :300], [5, 299], 4, 128, 2, 2, 0.2)
    assert r[0].shape == (3, 3) and not r[2][:, [5, 299]].any()


def test_binary32_reading_against_the_plain_definition():
    """The oracle takes every integer decision (s as fp16, z, q) in binary32 with a multiplication by
    the rounded reciprocal 1/s, the arithmetic the library documents; the plain definition divides in
    exact arithmetic.  Count, on the synthetic weights the GPU tests use, how often the two readings
    decide differently, and bound what a difference can cost: a differing code sits on a rounding tie
    of w/s (the two candidates are then equally far from w up to one ulp), a differing grid point or
    zero point changes the error of the group by a relative amount far below the ranking tolerance of
    the GPU parity test (2e-4)."""
    from synth import make_weights
    groups = diff_choice = diff_sz = diff_codes = codes_total = 0
    worst = 0.0
    for bits, seed in ((3, 5), (4, 6)):
        w, idx = make_weights(24, 1024, 8, seed=seed)
        keep = np.ones(1024, dtype=bool)
        keep[idx] = False
        for r in range(w.shape[0]):
            for g in range(8):
                sl = slice(128 * g, 128 * g + 128)
                s1, z1, q1, e1, c1 = search.search_group(w[r, sl], keep[sl], bits, 16, 16, 0.4)
                s2, z2, q2, e2, c2 = search.search_group_plain(w[r, sl], keep[sl], bits, 16, 16, 0.4)
                groups += 1
                diff_choice += int(c1 != c2)
                diff_sz += int(c1 == c2 and (s1 != s2 or z1 != z2))
                if c1 == c2 and s1 == s2 and z1 == z2:
                    diff_codes += int(np.count_nonzero(q1 != q2))
                    codes_total += int(keep[sl].sum())
                worst = max(worst, abs(e1 - e2) / max(e2, 1e-30))
    print(f"groups {groups}: other grid point {diff_choice}, same point other (s, z) {diff_sz}, "
          f"codes differing {diff_codes} of {codes_total}, worst relative error difference {worst:.2e}")
    assert groups == 384
    assert diff_sz == 0                      # the stored step size and zero point agree wherever the grid point does
    assert diff_choice <= groups // 50       # at most 2 % of the groups rank two near-equal candidates the other way
    assert diff_codes <= codes_total // 2000
    assert worst <= 2e-5
