"""Backward of the OWQ linear layer for weak-column tuning, in fp64.  Test infrastructure only.

What is followed: the paper's section "PEFT with Weak Column Tuning".  The layer is quantised
once; afterwards only its fp16 weak columns Ww are trained, the low-bit matrix stays as it is.
Training needs the two derivatives of the layer the forward oracle states,

    Y[n, i] = sum_{j not in S} s[i, g(j)] (q[i, j] - z[i, g(j)]) X[n, j] + sum_t Ww[i, t] X[n, idx[t]]

with respect to what lies upstream and to what is trained.  With dY = dL/dY they are, by the
chain rule (the paper prints neither: the layer is linear, so they are its transposes):

    dX[n, j]       = sum_i dY[n, i] s[i, g(j)] (q[i, j] - z[i, g(j)])        j not weak
    dX[n, idx[t]]  = sum_i dY[n, i] Ww[i, t]
    dWw[i, t]      = sum_n dY[n, i] X[n, idx[t]]

dY, X, s, z and Ww are fp16 values taken exactly into fp64; every product and sum is fp64.

Pins (tests/test_oracle_backward.py): the adjoint identities <dY, F(X)> = <dX, X> and
<dY, F(X; Ww + E) - F(X; Ww)> = <dWw, E> against the pinned forward oracle; central differences
of the forward oracle's loop version on a tiny layer; k = 0 (a plain product with the
dequantised matrix) and all columns weak (the plain fp16 products); nested Python loops.
"""
from __future__ import annotations

import numpy as np


def _groups(p, d_in: int, group_size: int) -> np.ndarray:
    p = np.asarray(p, dtype=np.float64)
    if group_size == 0:
        return np.broadcast_to(p[:, :1], (p.shape[0], d_in))
    return p[:, np.arange(d_in) // group_size]


def owq_backward_ref(codes, scale, zero, group_size, weak_idx, weak_w, x, dy):
    """(dX fp64 [batch, d_in], dWw fp64 [d_out, k]) for dY [batch, d_out] and X [batch, d_in]."""
    codes = np.asarray(codes)
    d_out, d_in = codes.shape
    idx = np.asarray(weak_idx, dtype=np.int64)
    dy64 = np.asarray(dy, dtype=np.float64)
    x64 = np.asarray(x, dtype=np.float64)
    assert dy64.shape[1] == d_out and x64.shape == (dy64.shape[0], d_in)
    w = _groups(scale, d_in, group_size) * (codes.astype(np.float64) - _groups(zero, d_in, group_size))
    w[:, idx] = np.asarray(weak_w, dtype=np.float64).reshape(d_out, idx.size)   # the weak columns as they are
    dx = dy64 @ w
    dww = dy64.T @ x64[:, idx]
    return dx, dww


def owq_backward_loops(codes, scale, zero, group_size, weak_idx, weak_w, x, dy):
    """The same as nested Python loops over plain floats (tiny shapes only)."""
    d_out, d_in = len(codes), len(codes[0])
    weak = [int(j) for j in weak_idx]
    pos = {j: t for t, j in enumerate(weak)}
    batch = len(dy)
    dx = [[0.0] * d_in for _ in range(batch)]
    dww = [[0.0] * len(weak) for _ in range(d_out)]
    for n in range(batch):
        for j in range(d_in):
            acc = 0.0
            for i in range(d_out):
                if j in pos:
                    wij = float(weak_w[i][pos[j]])
                else:
                    g = 0 if group_size == 0 else j // group_size
                    wij = float(scale[i][g]) * (int(codes[i][j]) - float(zero[i][g]))
                acc += float(dy[n][i]) * wij
            dx[n][j] = acc
    for i in range(d_out):
        for t, j in enumerate(weak):
            acc = 0.0
            for n in range(batch):
                acc += float(dy[n][i]) * float(x[n][j])
            dww[i][t] = acc
    return dx, dww
