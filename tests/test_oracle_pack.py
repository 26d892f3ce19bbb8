"""Pins for oracle/packfmt.py (CPU only)."""
import json
import os

import numpy as np
import pytest

from oracle import packfmt
from synth import LayerSpec, make_layer

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_tile_shapes_derived_by_hand():
    # nblk -> (CW, R): largest divisor <= 64 that keeps at least 60 of 64 lanes busy
    want = {1: (1, 64), 8: (8, 8), 32: (32, 2), 128: (64, 1), 40: (20, 3), 108: (12, 5),
            72: (12, 5), 288: (32, 2), 2: (2, 32), 7: (7, 9), 64: (64, 1), 63: (63, 1), 61: (61, 1),
            59: (1, 64)}
    for nblk, shape in want.items():
        assert packfmt.tile_shape(nblk) == shape, nblk


def test_hand_derived_bytes():
    g = json.load(open(os.path.join(GOLD, "pack_bytes.json")))
    c = g["b4_one_row"]
    geo = packfmt.geometry(c["d_out"], c["d_in"], c["bits"], 0, 0)
    sec = packfmt.pack_codes(np.array(c["codes"], dtype=np.uint8), geo)
    for off, b in c["bytes_at"].items():
        assert sec[int(off):int(off) + len(b)].tolist() == b
    c = g["b3_straddle"]
    codes = np.zeros((c["d_out"], c["d_in"]), dtype=np.uint8)
    for i, j, q in c["sparse_codes"]:
        codes[i, j] = q
    geo = packfmt.geometry(c["d_out"], c["d_in"], c["bits"], 0, 0)
    sec = packfmt.pack_codes(codes, geo)
    for off, b in c["bytes_at"].items():
        assert sec[int(off):int(off) + len(b)].tolist() == b
    assert int(sec.astype(np.int64).sum()) == 128 + 192 + 1 + 2


def test_tile_layout_hand_derived_bytes():
    c = json.load(open(os.path.join(GOLD, "pack_bytes.json")))["tile_b4"]
    codes = np.zeros((c["d_out"], c["d_in"]), dtype=np.uint8)
    for i, j, q in c["sparse_codes"]:
        codes[i, j] = q
    geo = packfmt.geometry(c["d_out"], c["d_in"], c["bits"], 0, 0, c["layout"])
    assert (geo.n_rt, geo.nbp, geo.nblk, geo.d_out_pad) == (1, 1, 2, 32)
    sec = packfmt.pack_codes(codes, geo)
    assert sec.size == 32 * 256 * 4 // 8
    for off, b in c["bytes_at"].items():
        assert sec[int(off):int(off) + len(b)].tolist() == b
    assert int(np.count_nonzero(sec)) == 3


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("d_out,d_in", [(1, 1), (70, 600), (33, 256), (5, 1000)])
def test_tile_layout_round_trip_and_twin(bits, d_out, d_in):
    rng = np.random.default_rng(d_out + d_in + bits)
    codes = rng.integers(0, 1 << bits, size=(d_out, d_in), dtype=np.uint8)
    geo = packfmt.geometry(d_out, d_in, bits, 0, 0, 1)
    sec = packfmt.pack_codes(codes, geo)
    assert sec.size == geo.d_out_pad * geo.nblk * 128 * bits // 8
    blob = np.zeros(geo.total_bytes, dtype=np.uint8)
    blob[:sec.size] = sec
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), codes)
    if d_out * d_in < 30000:
        np.testing.assert_array_equal(packfmt.pack_codes_bitwise(codes, geo), sec)


def test_tile_layout_blob_sections():
    L = make_layer(LayerSpec("t", 700, 45, 3, 256, 11, 5))
    blob, geo = packfmt.pack_layer(L.codes, L.scale, L.zero, 256, L.weak_idx, L.weak_w, 3, layout=1)
    assert geo.layout == 1 and blob.size == geo.total_bytes
    for off in (geo.off_sz, geo.off_weak_w, geo.off_weak_idx, geo.off_wmask, geo.off_scratch):
        assert off % 256 == 0
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), L.codes)
    s, z, ix, ww = packfmt.unpack_params(blob, geo)
    np.testing.assert_array_equal(ix, L.weak_idx)
    np.testing.assert_array_equal(ww.view(np.uint16), L.weak_w.view(np.uint16))
    np.testing.assert_array_equal(s.view(np.uint16), L.scale.view(np.uint16))
    np.testing.assert_array_equal(z.view(np.uint16), L.zero.view(np.uint16))
    # group-major: the dword of (row 7, group 2) sits at off_sz + (2 * d_out_pad + 7) * 4
    assert geo.d_out_pad == 64 and geo.n_groups == 3
    at = geo.off_sz + (2 * 64 + 7) * 4
    want = int(L.scale.view(np.uint16)[7, 2]) | (int(L.zero.view(np.uint16)[7, 2]) << 16)
    assert int.from_bytes(blob[at:at + 4].tobytes(), "little") == want
    mask = np.unpackbits(blob[geo.off_wmask:geo.off_wmask + geo.nbp * 32], bitorder="little")
    assert np.flatnonzero(mask).tolist() == L.weak_idx.tolist()
    assert not blob[geo.off_scratch:].any()


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("d_out,d_in", [(1, 1), (5, 200), (16, 256), (9, 128 * 7), (64, 128 * 40), (3, 128 * 65)])
def test_round_trip_and_size(bits, d_out, d_in):
    rng = np.random.default_rng(d_out * 1000 + d_in + bits)
    codes = rng.integers(0, 1 << bits, size=(d_out, d_in), dtype=np.uint8)
    geo = packfmt.geometry(d_out, d_in, bits, 0, 0)
    sec = packfmt.pack_codes(codes, geo)
    assert sec.size == geo.d_out_pad * geo.nblk * 128 * bits // 8       # exactly `bits` per stored code
    blob = np.zeros(geo.total_bytes, dtype=np.uint8)
    blob[:sec.size] = sec
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), codes)


@pytest.mark.parametrize("bits", [3, 4])
def test_extreme_patterns_round_trip(bits):
    d_out, d_in = 4, 256
    geo = packfmt.geometry(d_out, d_in, bits, 0, 0)
    top = (1 << bits) - 1
    pats = [np.zeros((d_out, d_in), np.uint8), np.full((d_out, d_in), top, np.uint8)]
    for b in range(bits):                      # walking one over the bit planes
        pats.append(np.full((d_out, d_in), 1 << b, np.uint8))
    alt = np.zeros((d_out, d_in), np.uint8)
    alt[:, ::2] = top
    pats.append(alt)
    for p in pats:
        sec = packfmt.pack_codes(p, geo)
        blob = np.zeros(geo.total_bytes, np.uint8)
        blob[:sec.size] = sec
        np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), p)
        # population count is preserved: no bit lost, none invented
        assert int(np.unpackbits(sec).sum()) == int(np.unpackbits(p).sum())


@pytest.mark.parametrize("bits,d_out,d_in", [(3, 5, 160), (4, 3, 136), (3, 70, 128)])
def test_bitwise_twin_builds_the_same_bytes(bits, d_out, d_in):
    rng = np.random.default_rng(bits + d_out + d_in)
    codes = rng.integers(0, 1 << bits, size=(d_out, d_in), dtype=np.uint8)
    geo = packfmt.geometry(d_out, d_in, bits, 0, 0)
    np.testing.assert_array_equal(packfmt.pack_codes_bitwise(codes, geo), packfmt.pack_codes(codes, geo))


def test_every_bit_has_its_own_address():
    geo = packfmt.geometry(7, 256, 3, 0, 0)
    seen = set()
    for i in range(7):
        for j in range(256):
            for b in range(3):
                a = packfmt.bit_address(geo, i, j, b)
                assert a not in seen
                seen.add(a)
    assert len(seen) == 7 * 256 * 3


@pytest.mark.parametrize("bits,group,k", [(3, 0, 5), (4, 128, 9), (3, 256, 0), (4, 0, 16)])
def test_whole_blob_round_trip(bits, group, k):
    L = make_layer(LayerSpec("t", 512, 21, bits, group, k, 77))
    dirty = L.codes.copy()
    dirty[:, L.weak_idx] = (1 << bits) - 1               # must be canonicalised to 0
    blob, geo = packfmt.pack_layer(dirty, L.scale, L.zero, group, L.weak_idx, L.weak_w, bits)
    assert blob.size == geo.total_bytes and geo.total_bytes % 256 == 0
    for off in (geo.off_codes, geo.off_sz, geo.off_weak_w, geo.off_weak_idx):
        assert off % 256 == 0
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), L.codes)
    s, z, ix, ww = packfmt.unpack_params(blob, geo)
    np.testing.assert_array_equal(s.view(np.uint16), L.scale.view(np.uint16))
    np.testing.assert_array_equal(z.view(np.uint16), L.zero.view(np.uint16))
    np.testing.assert_array_equal(ix, L.weak_idx)
    np.testing.assert_array_equal(ww.view(np.uint16), L.weak_w.view(np.uint16))
    assert geo.kp % 8 == 0 and geo.kp >= k
    raw_idx = np.frombuffer(blob.tobytes(), dtype="<i4", count=geo.kp, offset=geo.off_weak_idx)
    assert (raw_idx[k:] == -1).all()


def test_sz_dword_layout_by_hand():
    # scale 1.0 = 0x3C00, zero 2.0 = 0x4000 -> dword 0x40003C00 -> bytes 00 3C 00 40
    codes = np.zeros((1, 128), np.uint8)
    blob, geo = packfmt.pack_layer(codes, np.array([[1.0]], np.float16), np.array([[2.0]], np.float16),
                                   0, [], np.zeros((1, 0), np.float16), 4)
    assert blob[geo.off_sz:geo.off_sz + 4].tolist() == [0x00, 0x3C, 0x00, 0x40]


# ---------------------------------------------------------------------------
# storage-favoured layout (layout 2): the weak columns are not stored
# ---------------------------------------------------------------------------

def test_compact_layout_by_hand():
    # 1 row, 136 columns, 8 of them weak: 128 stored columns = exactly one block
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 8, size=(1, 136), dtype=np.uint8)
    idx = np.array([0, 9, 10, 64, 127, 128, 130, 135], dtype=np.int32)
    codes[:, idx] = 0
    scale = np.array([[0.5]], dtype=np.float16)
    zero = np.array([[3.0]], dtype=np.float16)
    ww = rng.normal(size=(1, 8)).astype(np.float16)
    blob, geo = packfmt.pack_layer(codes, scale, zero, 0, idx, ww, 3, layout=2)
    assert (geo.layout, geo.nblk, geo.k, geo.kp) == (2, 1, 8, 8)
    # the codes section is that of a 128-column layer holding the other columns in order
    kept = np.delete(codes, idx, axis=1)
    assert kept.shape == (1, 128)
    plain, geo0 = packfmt.pack_layer(kept, scale, zero, 0, np.zeros(0, np.int32), np.zeros((1, 0), np.float16), 3)
    assert geo.off_sz == geo0.off_sz
    np.testing.assert_array_equal(blob[:geo.off_sz], plain[:geo0.off_sz])
    # bookkeeping dwords, typed in by hand: unit i covers columns 8i .. 8i+7
    meta = np.frombuffer(blob.tobytes(), dtype="<u4", count=17, offset=geo.off_wmask)
    want_mask = {0: 0b00000001, 1: 0b00000110, 8: 0b00000001, 15: 0b10000000, 16: 0b10000101}
    before = {0: 0, 1: 1, 2: 3, 8: 3, 9: 4, 15: 4, 16: 5}
    count = 0
    for i in range(17):
        assert (meta[i] & 0xFF) == want_mask.get(i, 0), i
        assert (meta[i] >> 8) == count, i
        if i in before:
            assert count == before[i]
        count += bin(want_mask.get(i, 0)).count("1")
    assert count == 8
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), codes)


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("d_out,d_in,k", [(5, 200, 7), (16, 256, 0), (9, 1000, 104), (3, 130, 130), (20, 128 * 9 + 5, 5)])
def test_compact_layout_round_trip_and_size(bits, d_out, d_in, k):
    L = make_layer(LayerSpec("c", d_in, d_out, bits, 0, k, 31 + k))
    blob, geo = packfmt.pack_layer(L.codes, L.scale, L.zero, 0, L.weak_idx, L.weak_w, bits, layout=2)
    plain = packfmt.geometry(d_out, d_in, bits, 0, k, 0)
    stored = max(d_in - k, 1)
    assert -(-stored // 128) <= geo.nblk <= plain.nblk and geo.nslab <= plain.nslab
    # bytes of codes: rows (padded to whole tiles) x stored blocks x 16-byte chunks
    assert geo.off_sz == -(-(geo.d_out_pad * geo.nblk * geo.chunks * 16) // 256) * 256
    assert geo.nblk <= plain.nblk
    assert blob.size == geo.total_bytes
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), L.codes)
    s, z, ix, ww = packfmt.unpack_params(blob, geo)
    np.testing.assert_array_equal(ix, L.weak_idx)
    np.testing.assert_array_equal(ww.view(np.uint16), L.weak_w.view(np.uint16))
    np.testing.assert_array_equal(s.view(np.uint16), L.scale.view(np.uint16))


def test_compact_layout_needs_one_scale_per_row():
    L = make_layer(LayerSpec("c", 256, 8, 3, 128, 4, 1))
    with pytest.raises(AssertionError):
        packfmt.pack_layer(L.codes, L.scale, L.zero, 128, L.weak_idx, L.weak_w, 3, layout=2)
