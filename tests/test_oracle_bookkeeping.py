"""oracle/bookkeeping.py against the numbers the paper prints (CPU only)."""
import json
import os

import pytest

from oracle import bookkeeping as bk

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_bookkeeping.json")))


def test_weak_column_fraction_and_extra_bits():
    d = 4096
    k = bk.weak_columns(3.01, 3, d)
    c = G["weak_column_fraction_3p01_opt"]
    assert abs(k / d - c["value"]) <= c["tol"]
    c = G["extra_bit_per_layer_3p01_opt"]
    assert abs(0.01 / 6 - c["value"]) <= c["tol"]
    # k fp16 columns instead of 3-bit ones add (16-3)*k/d bits to a d x d layer
    assert (16 - 3) * bk.fp16_ratio_per_block(3.01, 3) / 6 == pytest.approx(0.01 * 12 / 6)


def test_zero_filled_effective_bits():
    d = 4096 * 16                                 # large d so that rounding of k does not matter
    k = bk.weak_columns(3.01, 3, d)
    c = G["zero_filled_effective_bits_3p01"]
    sf = bk.effective_bits(d, d, 3, k, zero_filled=False)
    zf = bk.effective_bits(d, d, 3, k, zero_filled=True)
    # the per-layer share of the 0.01 extra bits is 0.02 for a d x d layer (1/6 of 12 d^2 * 0.01 over d^2)
    assert sf == pytest.approx(3.02, abs=1e-4)
    assert abs(3 + (zf - 3) / 2 - c["value"]) <= c["tol"]


def test_group_equivalences():
    for c in G["overhead_equivalences"]:
        a = bk.overhead_owq(c["d"], c["t"], c["w"])
        b = bk.overhead_group(c["d"], c["g"])
        assert abs(a - b) / b <= c["rel_tol"]


def test_wct_parameter_ratio():
    c = G["wct_params"]
    a, b = bk.wct_vs_qlora_params(c["d"], c["D"], c["k"], c["r"])
    assert (a, b) == (339968, 4997120)
    assert abs(a / b - c["ratio"]) <= c["tol"]


def test_memory_overhead_low_end_of_sweep():
    c = G["memory_overhead_low_end"]
    for t, pct in zip(c["t"], c["percent"]):
        # zero-filled: every extra 13 bits of budget stores a 16-bit weight on top of the kept 3-bit slot
        got = 100 * (t - 3) * 16 / 13 / 3
        assert abs(got - pct) <= c["tol"], (t, got, pct)


def test_opt175b_extra_storage():
    c = G["opt175b_extra_mb"]
    weights = 12 * c["d"] ** 2 * c["blocks"]
    mb = weights * 0.01 * 16 / 13 / 8 / 1e6
    assert abs(mb - c["value_mb"]) / c["value_mb"] <= c["rel_tol"]
