"""Pins of the backward oracle (oracle/backward.py).  CPU only."""
import numpy as np
import pytest

from oracle import backward, owq_ref
from synth import LayerSpec, make_layer, make_x


def small_layer(bits=3, gs=128, k=5, d_in=256, d_out=24, seed=3):
    return make_layer(LayerSpec("b", d_in, d_out, bits, gs, k, seed))


def rand16(rng, shape, scale=1.0):
    return (rng.normal(0, scale, size=shape)).astype(np.float16)


@pytest.mark.parametrize("bits,gs,k", [(3, 0, 5), (4, 128, 7), (3, 128, 0)])
def test_adjoint_of_the_forward_oracle(bits, gs, k):
    # The layer is linear in X: <dY, F(X)> = <dX, X>.  It is linear in Ww as well:
    # <dY, F(X; Ww + E) - F(X; Ww)> = <dWw, E>.  F is the pinned forward oracle.
    L = small_layer(bits, gs, k)
    rng = np.random.default_rng(1)
    x, dy = make_x(L, 6), rand16(rng, (6, L.d_out))
    dx, dww = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x, dy)
    y = owq_ref.owq_linear_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x)
    lhs = np.sum(dy.astype(np.float64) * y)
    assert lhs == pytest.approx(np.sum(dx * x.astype(np.float64)), rel=1e-11)
    e = rand16(rng, L.weak_w.shape, 0.01)
    ww2 = L.weak_w.astype(np.float64) + e.astype(np.float64)
    y2 = owq_ref.owq_linear_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, ww2, x)
    assert np.sum(dy.astype(np.float64) * (y2 - y)) == pytest.approx(np.sum(dww * e.astype(np.float64)), rel=1e-9, abs=1e-12)
    assert dww.shape == (L.d_out, k)


def test_every_entry_by_unit_vectors():
    # dX[n, j] is the response of <dY[n], F(e_j)>: entry by entry against the forward oracle, which
    # catches a transposed operand, a wrong group or a weak column taken from the dense matrix.
    L = small_layer(4, 128, 4, d_in=256, d_out=8)
    rng = np.random.default_rng(2)
    dy = rand16(rng, (2, L.d_out))
    x = make_x(L, 2)
    dx, dww = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x, dy)
    eye = np.eye(L.d_in, dtype=np.float16)
    cols = owq_ref.owq_linear_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, eye)   # [d_in, d_out]: W^T
    assert np.allclose(dx, dy.astype(np.float64) @ cols.T, rtol=1e-12, atol=1e-15)
    for t, j in enumerate(L.weak_idx):
        assert np.allclose(cols[j], L.weak_w[:, t].astype(np.float64))
    assert np.allclose(dww, dy.astype(np.float64).T @ x.astype(np.float64)[:, L.weak_idx], rtol=1e-12)


def test_loops_agree():
    L = small_layer(3, 0, 3, d_in=128, d_out=5)
    rng = np.random.default_rng(4)
    x, dy = make_x(L, 3), rand16(rng, (3, 5))
    a = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x, dy)
    b = backward.owq_backward_loops(L.codes.tolist(), L.scale.tolist(), L.zero.tolist(), 0, L.weak_idx.tolist(),
                                    L.weak_w.tolist(), x.tolist(), dy.tolist())
    assert np.allclose(a[0], np.array(b[0]), rtol=1e-12, atol=1e-14)
    assert np.allclose(a[1], np.array(b[1]), rtol=1e-12, atol=1e-14)


def test_central_differences_of_the_forward_loops():
    # L = sum(dY * F): the derivative with respect to one activation and to one weak weight, by central
    # differences of the loop version of the forward oracle (exact up to rounding: F is linear).
    L = small_layer(4, 0, 2, d_in=128, d_out=4)
    rng = np.random.default_rng(5)
    x, dy = make_x(L, 2).astype(np.float64), rand16(rng, (2, 4)).astype(np.float64)
    dx, dww = backward.owq_backward_ref(L.codes, L.scale, L.zero, 0, L.weak_idx, L.weak_w, x, dy)

    def loss(xv, wwv):
        y = np.array(owq_ref.owq_linear_loops(L.codes.tolist(), L.scale.tolist(), L.zero.tolist(), 0,
                                              L.weak_idx.tolist(), wwv.tolist(), xv.tolist()))
        return float(np.sum(dy * y))
    ww = L.weak_w.astype(np.float64)
    for n, j in [(0, 0), (1, int(L.weak_idx[0])), (1, 77)]:
        xp, xm = x.copy(), x.copy()
        xp[n, j] += 0.5
        xm[n, j] -= 0.5
        assert loss(xp, ww) - loss(xm, ww) == pytest.approx(dx[n, j], rel=1e-9, abs=1e-12)
    for i, t in [(0, 0), (3, 1)]:
        wp, wm = ww.copy(), ww.copy()
        wp[i, t] += 0.5
        wm[i, t] -= 0.5
        assert loss(x, wp) - loss(x, wm) == pytest.approx(dww[i, t], rel=1e-9, abs=1e-12)


def test_all_columns_weak_is_the_fp16_product():
    rng = np.random.default_rng(6)
    d_out, d_in = 6, 128
    ww = rand16(rng, (d_out, d_in), 0.02)
    codes = np.zeros((d_out, d_in), np.uint8)
    s, z = np.ones((d_out, 1), np.float16), np.zeros((d_out, 1), np.float16)
    x, dy = rand16(rng, (3, d_in)), rand16(rng, (3, d_out))
    dx, dww = backward.owq_backward_ref(codes, s, z, 0, np.arange(d_in), ww, x, dy)
    assert np.array_equal(dx, dy.astype(np.float64) @ ww.astype(np.float64))
    assert np.array_equal(dww, dy.astype(np.float64).T @ x.astype(np.float64))
