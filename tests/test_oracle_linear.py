"""Pins for oracle/owq_ref.py (CPU only)."""
import json
import math
import os

import numpy as np
import pytest

from oracle import owq_ref
from synth import LayerSpec, make_layer, make_x

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _small(bits=3, group=0, k=5, d_in=96, d_out=7, seed=11):
    return make_layer(LayerSpec("t", d_in, d_out, bits, group, k, seed))


def test_hand_enumerated_layers():
    # tiny layers whose outputs were summed term by term by hand
    cases = json.load(open(os.path.join(GOLD, "hand_layers.json")))
    for name in ("A", "B"):
        c = cases[name]
        y = owq_ref.owq_linear_ref(np.array(c["codes"], dtype=np.uint8), np.array(c["scale"]),
                                   np.array(c["zero"]), c["group_size"], c["weak_idx"],
                                   np.array(c["weak_w"]), np.array(c["x"]))
        assert y.shape == (len(c["x"]), len(c["codes"]))
        np.testing.assert_array_equal(y, np.array(c["y"]))   # all values are dyadic: exact
        yl = owq_ref.owq_linear_loops(c["codes"], c["scale"], c["zero"], c["group_size"],
                                      c["weak_idx"], c["weak_w"], c["x"])
        np.testing.assert_array_equal(np.array(yl), np.array(c["y"]))


@pytest.mark.parametrize("bits,group", [(3, 0), (4, 0), (3, 32), (4, 16)])
def test_k0_is_plain_quantised_matmul(bits, group):
    # k = 0: textbook asymmetric-quantised matmul, coded a different way here
    # (per-row lookup table of the 2^bits dequantised levels + einsum).
    L = _small(bits=bits, group=group, k=0, d_in=64, d_out=9)
    x = make_x(L, 3)
    levels = np.arange(1 << bits, dtype=np.float64)
    G = L.n_groups
    gs = L.d_in if group == 0 else group
    lut = L.scale.astype(np.float64)[:, :, None] * (levels[None, None, :] - L.zero.astype(np.float64)[:, :, None])
    w = np.empty((L.d_out, L.d_in))
    for i in range(L.d_out):
        for g in range(G):
            sl = slice(g * gs, min(L.d_in, (g + 1) * gs))
            w[i, sl] = lut[i, g][L.codes[i, sl]]
    want = np.einsum("ij,nj->ni", w, x.astype(np.float64))
    got = owq_ref.owq_linear_layer(L, x)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_all_columns_weak_is_fp16_matmul():
    # every column weak: the codes, scales and zeros must not matter at all
    rng = np.random.default_rng(5)
    d_out, d_in = 6, 40
    w16 = rng.normal(0, 0.02, size=(d_out, d_in)).astype(np.float16)
    x = rng.normal(0, 1, size=(2, d_in)).astype(np.float16)
    codes = rng.integers(0, 8, size=(d_out, d_in), dtype=np.uint8)
    scale = rng.uniform(0.5, 2, size=(d_out, 1)).astype(np.float16)
    zero = rng.integers(1, 8, size=(d_out, 1)).astype(np.float16)
    got = owq_ref.owq_linear_ref(codes, scale, zero, 0, np.arange(d_in), w16, x)
    want = np.matmul(x.astype(np.float64), w16.astype(np.float64).T)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)
    # and against exactly rounded sums
    for n in range(2):
        for i in range(d_out):
            exact = math.fsum(float(w16[i, j]) * float(x[n, j]) for j in range(d_in))
            assert abs(got[n, i] - exact) <= 1e-15 * max(1.0, abs(exact)) * d_in


def test_one_hot_reads_back_effective_matrix():
    # x = e_j reconstructs column j: s*(q-z) for dense j, the fp16 weight for weak j
    L = _small(bits=4, group=32, k=6, d_in=96, d_out=5, seed=3)
    eye = np.eye(L.d_in, dtype=np.float16)
    y = owq_ref.owq_linear_layer(L, eye)          # [d_in, d_out]
    weak = {int(j): t for t, j in enumerate(L.weak_idx)}
    for j in range(L.d_in):
        for i in range(L.d_out):
            if j in weak:
                want = float(L.weak_w[i, weak[j]])
            else:
                g = j // 32
                want = float(L.scale[i, g]) * (int(L.codes[i, j]) - float(L.zero[i, g]))
            assert y[j, i] == want


def test_moving_an_exact_column_to_the_weak_set_changes_nothing():
    # s = 2^-m and integer z make s*(q-z) an fp16 number, so a column may sit in
    # either representation; the weak set only changes where the value is stored.
    rng = np.random.default_rng(8)
    d_out, d_in = 8, 48
    codes = rng.integers(0, 16, size=(d_out, d_in), dtype=np.uint8)
    scale = (2.0 ** -rng.integers(1, 6, size=(d_out, 1))).astype(np.float16)
    zero = rng.integers(0, 16, size=(d_out, 1)).astype(np.float16)
    x = rng.normal(0, 1, size=(3, d_in)).astype(np.float16)
    base = owq_ref.owq_linear_ref(codes, scale, zero, 0, [], np.zeros((d_out, 0)), x)
    idx = np.array([3, 17, 40])
    ww = (scale.astype(np.float64) * (codes[:, idx].astype(np.float64) - zero.astype(np.float64))).astype(np.float16)
    garbage = codes.copy()
    garbage[:, idx] = 9                           # what sits at a weak position is ignored
    moved = owq_ref.owq_linear_ref(garbage, scale, zero, 0, idx, ww, x)
    np.testing.assert_allclose(moved, base, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("bits,group,k", [(3, 0, 4), (4, 16, 3), (3, 8, 0)])
def test_loops_twin_agrees(bits, group, k):
    L = _small(bits=bits, group=group, k=k, d_in=32, d_out=4, seed=21)
    x = make_x(L, 2)
    a = owq_ref.owq_linear_layer(L, x)
    b = np.array(owq_ref.owq_linear_loops(L.codes.tolist(), L.scale.tolist(), L.zero.tolist(),
                                          group, L.weak_idx.tolist(), L.weak_w.tolist(), x.tolist()))
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_weak_pairing_and_order():
    # Ww[:, t] pairs with idx[t]: swapping two weak columns' weights must change y
    L = _small(bits=3, group=0, k=2, d_in=32, d_out=3, seed=2)
    x = make_x(L, 1)
    y = owq_ref.owq_linear_layer(L, x)
    swapped = owq_ref.owq_linear_ref(L.codes, L.scale, L.zero, 0, L.weak_idx, L.weak_w[:, ::-1], x)
    assert not np.allclose(y, swapped)
    # direct check of the weak term alone: zero scale kills the dense term
    z = owq_ref.owq_linear_ref(L.codes, np.zeros_like(L.scale), L.zero, 0, L.weak_idx, L.weak_w, x)
    want = x[:, L.weak_idx].astype(np.float64) @ L.weak_w.astype(np.float64).T
    np.testing.assert_allclose(z, want, rtol=1e-13)


def test_row_chunking_is_invisible():
    L = _small(bits=4, group=0, k=3, d_in=64, d_out=37, seed=4)
    x = make_x(L, 2)
    a = owq_ref.owq_linear_layer(L, x, row_chunk=5)
    b = owq_ref.owq_linear_layer(L, x, row_chunk=1000)
    np.testing.assert_array_equal(a, b)


def test_fp16_rounding_and_error_measures():
    y = np.array([[1.0 + 2 ** -11, 1.0 + 3 * 2 ** -11, 70000.0]])
    h = owq_ref.to_fp16(y)
    assert h[0, 0] == np.float16(1.0)                    # tie -> even
    assert h[0, 1] == np.float16(1.0 + 2 ** -9)          # tie -> even (up)
    assert np.isinf(h[0, 2])
    rel, mx = owq_ref.parity_errors(np.array([3.0, 4.0 + 0.5]), np.array([3.0, 4.0]))
    assert rel == pytest.approx(0.5 / 5.0)
    assert mx == pytest.approx(0.5 / math.sqrt(12.5))


# ---- several tasks sharing the dense matrix (section "Weak Column Tuning") ------------------

def _multi_case(seed=21, d_in=256, d_out=24, k=6, n_sets=3, batch=7):
    rng = np.random.default_rng(seed)
    L = make_layer(LayerSpec("multi", d_in, d_out, 3, 128, k, seed))
    sets = [rng.normal(0, 0.02, size=(d_out, k)).astype(np.float16) for _ in range(n_sets)]
    task = rng.integers(0, n_sets, size=batch)
    x = make_x(L, batch)
    return L, sets, task, x


def test_multi_task_with_one_task_is_the_single_task_layer():
    L, sets, task, x = _multi_case()
    for t in range(len(sets)):
        want = owq_ref.owq_linear_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, sets[t], x)
        got = owq_ref.owq_linear_multi_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, sets,
                                           [t] * x.shape[0], x)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


def test_multi_task_difference_is_the_difference_of_the_weak_columns():
    # moving token n from task a to task b changes y[n] by (Ww_b - Ww_a) x[n, idx] and nothing else
    L, sets, task, x = _multi_case(seed=22)
    base = owq_ref.owq_linear_multi_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, sets, task, x)
    task2 = task.copy()
    n = 3
    task2[n] = (task[n] + 1) % len(sets)
    moved = owq_ref.owq_linear_multi_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, sets, task2, x)
    xw = x[n, L.weak_idx].astype(np.float64)
    delta = (sets[task2[n]].astype(np.float64) - sets[task[n]].astype(np.float64)) @ xw
    np.testing.assert_allclose(moved[n] - base[n], delta, rtol=0, atol=1e-12)
    keep = np.arange(x.shape[0]) != n
    np.testing.assert_array_equal(moved[keep], base[keep])


def test_multi_task_tiny_layer_by_loops():
    L, sets, task, x = _multi_case(seed=23, d_in=128, d_out=3, k=2, n_sets=2, batch=4)
    got = owq_ref.owq_linear_multi_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, sets, task, x)
    for n in range(4):
        want = owq_ref.owq_linear_loops(L.codes.tolist(), L.scale.tolist(), L.zero.tolist(), L.group_size,
                                        L.weak_idx.tolist(), sets[task[n]].tolist(), [x[n].tolist()])
        np.testing.assert_allclose(got[n], np.array(want[0]), rtol=1e-12, atol=1e-12)
