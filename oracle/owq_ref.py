"""What the OWQ linear layer computes, in fp64.  Test infrastructure only.

Definition followed (paper, storage paragraph of the "Outlier-Aware Weight
Quantization" section and the "Acceleration on Real Device" section; shapes
from Eq. (3): W is C_out x C_in, X is C_in x N):

    Y[n, i] = sum_{j not in S} s[i, g(j)] * (q[i, j] - z[i, g(j)]) * x[n, j]
            + sum_{t < k}      Ww[i, t] * x[n, idx[t]]

    S = {idx[0], ..., idx[k-1]}      the weak columns
    g(j) = j // group_size           (0 when there is one group per row)

The low-bit matrix is stored with its weak-column positions "zero-filled";
the reading taken here is that the dense term contributes exactly nothing at
those positions (a stored code of 0 would otherwise dequantise to -s*z).
The quantiser is linear and asymmetric (step size s, zero point z), per
output channel or per group of consecutive input columns of a row.
s, z, Ww and x are fp16 values taken exactly into fp64; every product and sum
is fp64.
"""
from __future__ import annotations

import numpy as np


def _expand_groups(p: np.ndarray, d_in: int, group_size: int) -> np.ndarray:
    """[d_out, G] per-group parameter -> [d_out, d_in] per-column, fp64."""
    p = np.asarray(p, dtype=np.float64)
    if group_size == 0:
        assert p.shape[1] == 1
        return np.broadcast_to(p, (p.shape[0], d_in))
    g_of_j = np.arange(d_in) // group_size
    return p[:, g_of_j]


def dequantize_dense(codes, scale, zero, group_size, weak_idx) -> np.ndarray:
    """fp64 [d_out, d_in] matrix s*(q - z) with the weak columns set to 0."""
    codes = np.asarray(codes)
    d_out, d_in = codes.shape
    s = _expand_groups(scale, d_in, group_size)
    z = _expand_groups(zero, d_in, group_size)
    w = s * (codes.astype(np.float64) - z)
    w = np.array(w, copy=True)
    w[:, np.asarray(weak_idx, dtype=np.int64)] = 0.0
    return w


def owq_linear_ref(codes, scale, zero, group_size, weak_idx, weak_w, x,
                   row_chunk: int = 1024) -> np.ndarray:
    """Y (fp64, [batch, d_out]) for x (fp16 or float, [batch, d_in])."""
    codes = np.asarray(codes)
    d_out, d_in = codes.shape
    x64 = np.asarray(x, dtype=np.float64)
    assert x64.ndim == 2 and x64.shape[1] == d_in
    idx = np.asarray(weak_idx, dtype=np.int64)
    ww = np.asarray(weak_w, dtype=np.float64)
    assert ww.shape == (d_out, idx.size)
    y = np.empty((x64.shape[0], d_out), dtype=np.float64)
    xw = x64[:, idx]                                  # [batch, k] gathered activations
    for r0 in range(0, d_out, row_chunk):
        r1 = min(d_out, r0 + row_chunk)
        dense = dequantize_dense(codes[r0:r1], np.asarray(scale)[r0:r1],
                                 np.asarray(zero)[r0:r1], group_size, idx)
        y[:, r0:r1] = x64 @ dense.T + xw @ ww[r0:r1].T
    return y


def owq_linear_layer(layer, x, **kw) -> np.ndarray:
    """Convenience: same as owq_linear_ref on a synth.Layer-like object."""
    return owq_linear_ref(layer.codes, layer.scale, layer.zero, layer.group_size,
                          layer.weak_idx, layer.weak_w, x, **kw)


def owq_linear_loops(codes, scale, zero, group_size, weak_idx, weak_w, x):
    """The same definition as nested Python loops over plain floats.

    Shares nothing with owq_linear_ref (no numpy arithmetic): for tiny shapes.
    """
    d_out = len(codes)
    d_in = len(codes[0])
    weak = [int(j) for j in weak_idx]
    weak_set = set(weak)
    out = []
    for n in range(len(x)):
        row_out = []
        for i in range(d_out):
            acc = 0.0
            for j in range(d_in):
                if j in weak_set:
                    continue
                g = 0 if group_size == 0 else j // group_size
                acc += float(scale[i][g]) * (int(codes[i][j]) - float(zero[i][g])) * float(x[n][j])
            for t, j in enumerate(weak):
                acc += float(weak_w[i][t]) * float(x[n][j])
            row_out.append(acc)
        out.append(row_out)
    return out


def to_fp16(y64: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp64 -> fp16 (overflow goes to +-inf)."""
    with np.errstate(over="ignore"):
        return np.asarray(y64, dtype=np.float64).astype(np.float16)


def parity_errors(y_test, y_ref64):
    """(relative L2 error, max-abs error / rms(y_ref)) of y_test against the fp64 result."""
    a = np.asarray(y_test, dtype=np.float64)
    b = np.asarray(y_ref64, dtype=np.float64)
    den = np.sqrt(np.sum(b * b))
    rel = np.sqrt(np.sum((a - b) ** 2)) / den if den > 0 else float(np.sqrt(np.sum((a - b) ** 2)))
    rms = np.sqrt(np.mean(b * b))
    mx = np.max(np.abs(a - b)) / rms if rms > 0 else float(np.max(np.abs(a - b)))
    return float(rel), float(mx)


def owq_linear_multi_ref(codes, scale, zero, group_size, weak_idx, weak_sets, task_id, x,
                         row_chunk: int = 1024) -> np.ndarray:
    """Several tasks sharing one dense low-bit matrix (paper, section "Weak Column Tuning":
    only the weak columns are tuned per task, the dense matrix and the indices are shared).

        Y[n, i] = sum_{j not in S} s[i, g(j)] (q[i, j] - z[i, g(j)]) x[n, j]
                + sum_{t < k} Ww[task_id[n]][i, t] x[n, idx[t]]

    weak_sets: sequence of [d_out, k] fp16 arrays, task_id: [batch] ints in [0, len(weak_sets)).
    Written token by token, each with its own weak columns; no sharing of work between tokens.
    """
    codes = np.asarray(codes)
    d_out, d_in = codes.shape
    x64 = np.asarray(x, dtype=np.float64)
    idx = np.asarray(weak_idx, dtype=np.int64)
    task_id = [int(t) for t in task_id]
    assert len(task_id) == x64.shape[0] and all(0 <= t < len(weak_sets) for t in task_id)
    y = np.empty((x64.shape[0], d_out), dtype=np.float64)
    for r0 in range(0, d_out, row_chunk):
        r1 = min(d_out, r0 + row_chunk)
        dense = dequantize_dense(codes[r0:r1], np.asarray(scale)[r0:r1], np.asarray(zero)[r0:r1],
                                 group_size, idx)
        for n in range(x64.shape[0]):
            ww = np.asarray(weak_sets[task_id[n]], dtype=np.float64)[r0:r1]
            y[n, r0:r1] = dense @ x64[n] + ww @ x64[n, idx]
    return y
