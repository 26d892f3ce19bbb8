"""Host-side checks of libowq.so that need no GPU: it loads, exports what include/owq.h
declares, packs exactly the bytes the oracle's format code produces, and rejects bad input."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import packfmt
from synth import LayerSpec, make_layer

B = pytest.importorskip("paper_2306_02272_amd.binding")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return B.lib()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "owq.h")).read()
    declared = set(re.findall(r"\b(owq_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes_match_header(lib):
    # 16 + 2 + 8 int32 and 5 + 2 uint64 in the info record; 5 int32 (+pad), 5 pointers and one
    # int32 (+pad) in the description
    assert C.sizeof(B.LayerInfo) == 26 * 4 + 7 * 8
    assert C.sizeof(B.LayerDesc) == 24 + 5 * 8 + 8


@pytest.mark.parametrize("spec", [
    LayerSpec("a", 512, 21, 3, 0, 5, 1), LayerSpec("b", 1000, 33, 4, 128, 9, 2),
    LayerSpec("c", 128 * 40, 10, 3, 256, 0, 3), LayerSpec("d", 128 * 108, 7, 4, 128, 138, 4),
    LayerSpec("e", 1, 1, 3, 0, 1, 5), LayerSpec("f", 4096, 64, 3, 128, 32, 6)])
def test_host_pack_equals_oracle_pack(lib, spec):
    L = make_layer(spec)
    dirty = L.codes.copy()
    dirty[:, L.weak_idx] = 255                     # ignored at weak columns, stored as 0
    d = B.make_desc(L.d_out, L.d_in, L.bits, L.group_size, L.k, dirty, L.scale, L.zero,
                    L.weak_idx, L.weak_w)
    blob = B.owq_pack_host(d)
    want, geo = packfmt.pack_layer(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, L.bits)
    info = B.owq_geometry(d)
    for f in ("nblk", "cw", "r", "nact", "nslab", "n_rt", "d_out_pad", "chunks", "n_groups", "kp",
              "off_codes", "off_sz", "off_weak_w", "off_weak_idx", "total_bytes"):
        assert getattr(info, f) == getattr(geo, f), f
    assert B.owq_packed_bytes(d) == geo.total_bytes
    np.testing.assert_array_equal(blob, want)
    np.testing.assert_array_equal(B.owq_unpack_codes(blob, info), L.codes)
    np.testing.assert_array_equal(packfmt.unpack_codes(blob, geo), L.codes)


@pytest.mark.parametrize("spec", [
    LayerSpec("ta", 700, 45, 3, 256, 11, 21), LayerSpec("tb", 256, 32, 4, 0, 0, 22),
    LayerSpec("tc", 1000, 70, 4, 128, 9, 23), LayerSpec("td", 130, 3, 3, 0, 130, 24)])
def test_tile_layout_host_pack_equals_oracle_pack(lib, spec):
    L = make_layer(spec)
    d = B.desc_from_layer(L, B.OWQ_LAYOUT_TILE)
    blob = B.owq_pack_host(d)
    want, geo = packfmt.pack_layer(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, L.bits,
                                   layout=1)
    info = B.owq_geometry(d)
    for f in ("layout", "nbp", "nblk", "n_rt", "d_out_pad", "chunks", "n_groups", "kp", "off_codes", "off_sz",
              "off_weak_w", "off_weak_idx", "off_wmask", "off_scratch"):
        assert getattr(info, f) == getattr(geo, f), f
    # the format ends at off_scratch; what follows is the library's working memory, zero in a fresh blob
    assert geo.total_bytes == geo.off_scratch and info.total_bytes >= geo.off_scratch and info.total_bytes % 256 == 0
    np.testing.assert_array_equal(blob[:geo.off_scratch], want)
    assert blob.size == info.total_bytes and not blob[geo.off_scratch:].any()
    np.testing.assert_array_equal(B.owq_unpack_codes(blob, info), L.codes)
    bad = B.desc_from_layer(L, 7)
    assert _status(B.owq_packed_bytes, bad) == B.OWQ_ERR_LAYOUT


@pytest.mark.parametrize("spec", [
    LayerSpec("ca", 700, 45, 3, 0, 11, 21), LayerSpec("cb", 256, 32, 4, 0, 0, 22),
    LayerSpec("cc", 1003, 70, 4, 0, 107, 23), LayerSpec("cd", 130, 3, 3, 0, 130, 24),
    LayerSpec("ce", 128 * 6 + 8, 9, 3, 0, 8, 25)])
def test_storage_favoured_layout_host_pack_equals_oracle_pack(lib, spec):
    L = make_layer(spec)
    d = B.desc_from_layer(L, B.OWQ_LAYOUT_COMPACT)
    blob = B.owq_pack_host(d)
    want, geo = packfmt.pack_layer(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, L.bits,
                                   layout=2)
    info = B.owq_geometry(d)
    for f in ("layout", "nblk", "cw", "r", "nact", "nslab", "n_rt", "d_out_pad", "chunks", "n_groups", "kp",
              "off_codes", "off_sz", "off_weak_w", "off_weak_idx", "off_wmask", "total_bytes"):
        assert getattr(info, f) == getattr(geo, f), f
    np.testing.assert_array_equal(blob, want)
    np.testing.assert_array_equal(B.owq_unpack_codes(blob, info), L.codes)
    # fewer bytes than the full-size matrix whenever whole blocks of columns are saved
    plain = B.owq_geometry(B.desc_from_layer(L, B.OWQ_LAYOUT_GEMV))
    assert info.nblk <= plain.nblk


def test_storage_favoured_layout_needs_one_scale_per_row(lib):
    L = make_layer(LayerSpec("cg", 512, 8, 3, 128, 4, 9))
    assert _status(B.owq_packed_bytes, B.desc_from_layer(L, B.OWQ_LAYOUT_COMPACT)) == B.OWQ_ERR_GROUP


def _status(fn, *a):
    try:
        fn(*a)
    except B.OwqError as e:
        return e.status
    return B.OWQ_OK


def test_rejects_bad_descriptions(lib):
    L = make_layer(LayerSpec("t", 256, 8, 3, 0, 4, 9))

    def desc(**kw):
        f = dict(d_out=L.d_out, d_in=L.d_in, bits=L.bits, group_size=0, k=L.k, codes=L.codes,
                 scale=L.scale, zero=L.zero, weak_idx=L.weak_idx, weak_w=L.weak_w)
        f.update(kw)
        return B.make_desc(**f)

    assert _status(B.owq_pack_host, desc()) == B.OWQ_OK
    assert _status(B.owq_pack_host, desc(bits=5)) == B.OWQ_ERR_BITS
    assert _status(B.owq_pack_host, desc(bits=2)) == B.OWQ_ERR_BITS
    assert _status(B.owq_pack_host, desc(d_out=0)) == B.OWQ_ERR_SHAPE
    assert _status(B.owq_pack_host, desc(d_in=-4)) == B.OWQ_ERR_SHAPE
    assert _status(B.owq_pack_host, desc(group_size=64)) == B.OWQ_ERR_GROUP
    assert _status(B.owq_pack_host, desc(group_size=-128)) == B.OWQ_ERR_GROUP
    assert _status(B.owq_pack_host, desc(k=L.d_in + 1)) == B.OWQ_ERR_INDEX
    assert _status(B.owq_pack_host, desc(k=-1)) == B.OWQ_ERR_INDEX
    assert _status(B.owq_pack_host, desc(codes=None)) == B.OWQ_ERR_NULL
    assert _status(B.owq_pack_host, desc(weak_w=None)) == B.OWQ_ERR_NULL
    bad = L.codes.copy()
    free_col = [j for j in range(L.d_in) if j not in set(L.weak_idx.tolist())][0]
    bad[3, free_col] = 8
    assert _status(B.owq_pack_host, desc(codes=bad)) == B.OWQ_ERR_CODE_RANGE
    for idx in ([5, 5, 6, 7], [9, 3, 20, 21], [0, 1, 2, 256], [-1, 1, 2, 3]):
        assert _status(B.owq_pack_host, desc(weak_idx=np.array(idx, np.int32))) == B.OWQ_ERR_INDEX
    # too small a buffer
    d = desc()
    n = B.owq_packed_bytes(d)
    small = np.empty(n - 1, np.uint8)
    assert B.lib().owq_pack_host(C.byref(d), small.ctypes.data, small.size) == B.OWQ_ERR_BUFFER
    # null arguments
    assert B.lib().owq_pack_host(None, small.ctypes.data, 0) == B.OWQ_ERR_NULL
    assert B.lib().owq_packed_bytes(C.byref(d), None) == B.OWQ_ERR_NULL


def test_dead_handles_are_refused(lib):
    assert B.lib().owq_linear(None, None, None, 1, None) == B.OWQ_ERR_HANDLE
    assert B.lib().owq_free_layer(None) == B.OWQ_ERR_HANDLE
    fake = (C.c_uint32 * 64)()                      # zeroed memory is not a handle
    assert B.lib().owq_linear(C.addressof(fake), None, None, 1, None) == B.OWQ_ERR_HANDLE
    info = B.LayerInfo()
    assert B.lib().owq_layer_info(C.addressof(fake), C.byref(info)) == B.OWQ_ERR_HANDLE


def test_status_strings(lib):
    seen = {B.owq_status_str(s) for s in range(13)}
    assert len(seen) == 13 and "ok" in seen
    assert B.owq_status_str(99) == "unknown status"


def test_layers_of_4_gib_or_more_are_refused(lib):
    # the kernels address a blob with 32-bit byte offsets: shapes only, no data is touched
    ok = B.make_desc(65536, 65536, 4, 0, 0)                   # 2 GiB of codes
    assert B.owq_packed_bytes(ok) > 2 ** 31
    big = B.make_desc(131072, 65536, 4, 0, 0)                 # 4 GiB of codes
    assert _status(B.owq_packed_bytes, big) == B.OWQ_ERR_SHAPE
    big3 = B.make_desc(200000, 65536, 3, 128, 0)
    assert _status(B.owq_geometry, big3) == B.OWQ_ERR_SHAPE
    tile = B.make_desc(131072, 65536, 4, 0, 0, layout=B.OWQ_LAYOUT_TILE)
    assert _status(B.owq_packed_bytes, tile) == B.OWQ_ERR_SHAPE


def test_dead_handles_are_refused_by_the_weak_column_calls(lib):
    fake = (C.c_uint32 * 64)()
    n = C.c_size_t(0)
    assert B.lib().owq_weak_set_bytes(None, C.byref(n)) == B.OWQ_ERR_HANDLE
    assert B.lib().owq_update_weak(C.addressof(fake), None, None) == B.OWQ_ERR_HANDLE
    assert B.lib().owq_pack_weak_set(None, None, None, 0, None) == B.OWQ_ERR_HANDLE
    assert B.lib().owq_linear_multi(C.addressof(fake), None, 1, None, None, None, 1, None) == B.OWQ_ERR_HANDLE
    assert B.lib().owq_set_launch(None, 1, 1, 1, 2) == B.OWQ_ERR_HANDLE


def test_search_rejects_bad_arguments(lib):
    # Every check of owq_search_config comes before its launch, so the error paths need no GPU.
    # The pointers are never dereferenced on these paths.
    assert C.sizeof(B.SearchDesc) == 8 * 4
    p = 256

    def call(desc, w=p, idx=p, scale=p, zero=p, codes=p):
        try:
            B.owq_search_config(desc, w, idx, scale, zero, codes)
        except B.OwqError as e:
            return e.status
        return B.OWQ_OK

    good = dict(d_out=4, d_in=256, bits=3, group_size=128, k=2, n_lo=4, n_hi=4, shrink=0.3)

    def desc(**kw):
        f = dict(good, **kw)
        return B.SearchDesc(f["d_out"], f["d_in"], f["bits"], f["group_size"], f["k"], f["n_lo"], f["n_hi"],
                            f["shrink"])
    assert call(desc(), w=0) == B.OWQ_ERR_NULL
    assert call(desc(), codes=0) == B.OWQ_ERR_NULL
    assert call(desc(), idx=0) == B.OWQ_ERR_NULL
    assert call(desc(d_out=0)) == B.OWQ_ERR_SHAPE
    assert call(desc(d_in=0)) == B.OWQ_ERR_SHAPE
    assert call(desc(bits=5)) == B.OWQ_ERR_BITS
    assert call(desc(group_size=100)) == B.OWQ_ERR_GROUP
    assert call(desc(group_size=-128)) == B.OWQ_ERR_GROUP
    assert call(desc(k=-1)) == B.OWQ_ERR_INDEX
    assert call(desc(k=257)) == B.OWQ_ERR_INDEX
    assert call(desc(n_lo=0)) == B.OWQ_ERR_SHAPE
    assert call(desc(n_hi=17)) == B.OWQ_ERR_SHAPE
    assert call(desc(shrink=0.5)) == B.OWQ_ERR_SHAPE
    assert call(desc(shrink=-0.1)) == B.OWQ_ERR_SHAPE
    assert call(desc(shrink=float("nan"))) == B.OWQ_ERR_SHAPE
    assert call(desc(d_out=2 ** 31 - 1, d_in=2 ** 30, k=0)) == B.OWQ_ERR_SHAPE
    # a row whose weak-column bit mask would not fit the kernel's share of LDS (47 KiB = 385024 columns)
    assert call(desc(d_out=1, d_in=385024 + 32, group_size=0, k=0)) == B.OWQ_ERR_UNSUPPORTED
