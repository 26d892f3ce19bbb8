"""Packed storage format v1 of an OWQ layer, on the CPU.  Test infrastructure only.

The paper fixes what is stored (a full-size low-bit matrix with zero-filled
weak-column positions, fp16 weak columns, one integer index per weak column,
a step size and zero point per channel or group; storage paragraph of the
"Outlier-Aware Weight Quantization" section and appendix B.2) but no bit
layout.  The layout below is this project's own definition; this file writes
it out with numpy, independently of the library's C++ packer, so that the two
can be compared byte for byte.

Geometry
  A *block* is 128 consecutive input columns of one output row.
  nblk  = ceil(d_in / 128)                  column blocks per row (columns past
                                             d_in hold code 0)
  CW    = the largest divisor c of nblk with c <= 64 and floor(64/c)*c >= 60
  R     = floor(64 / CW)                    rows per tile
  nact  = R * CW                            (row, block) pairs per tile
  nslab = nblk / CW                         tiles per row tile
  n_rt  = ceil(d_out / R),  d_out_pad = n_rt * R   (rows past d_out hold code 0,
                                             scale 0, zero 0, weak weights 0)
  C     = 3 (3-bit) or 4 (4-bit)            16-byte chunks per block

Blob = four sections, each starting on a 256-byte boundary, in this order:
  codes     n_rt * nslab tiles, tile (rt, s) at index rt*nslab + s; a tile is
            [chunk c][lane a][16 bytes]; lane a = rloc*CW + bloc stands for
            row rt*R + rloc and block s*CW + bloc.  The lane's C*4 little-endian
            dwords v = 4c + e (e = dword within the chunk) hold:
              3-bit: quad u = v // 3 covers columns 32u .. 32u+31 of the block;
                     column 2t goes to the 48-bit stream L at bits [3t, 3t+3),
                     column 2t+1 to the stream H at the same bits; dword
                     w = v % 3 of the quad is (L >> 16w) & 0xffff in its low
                     half and (H >> 16w) & 0xffff in its high half.
              4-bit: dword v covers columns 8v .. 8v+7; column 2t sits at bits
                     [4t, 4t+4) of the low half, column 2t+1 at the same bits
                     of the high half.
  sz        d_out_pad * G dwords, row-major; low half = fp16 bits of the step
            size, high half = fp16 bits of the zero point.
  weak_w    d_out_pad * kp fp16, row-major, kp = k rounded up to a multiple of
            8, padding 0.
  weak_idx  kp int32, padding -1.

Tile layout (layout = 1, for batched calls on the matrix cores).  Same sections,
with these differences:
  * a tile is 32 rows by one *block pair* (256 consecutive columns); nbp =
    ceil(d_in / 256), nblk = 2 * nbp, n_rt = ceil(d_out / 32), all 64 lanes busy.
    Lane a stands for row rt*32 + a % 32 and half kg = a // 32 of both blocks:
    its 128 codes are "lane columns" c = 64*b + 8*t + e  (b = 0, 1 the block of the
    pair, t = 0..7, e = 0..7) and lane column c is input column
    256*bp + 128*b + 16*t + 8*kg + e.  The 128 lane columns are packed into the
    lane's dwords exactly as the 128 columns of a block are in layout 0.
    Tiles are ordered [row tile][block pair]; a tile is [chunk][lane][16 bytes].
  * sz and weak_w have n_rt*32 rows; sz is stored group-major, [G][n_rt*32] dwords (the
    rows of a tile next to each other).
  * two more sections follow weak_idx: wmask, one byte per 8 input columns
    (bit e = column 8i+e is weak), nbp*32 bytes.  The format ends there, at off_scratch
    (= total_bytes here).  The library's blob goes on with working memory of its kernels,
    whose size is the library's own business and no part of the format: all this module
    says of it is that a freshly packed blob holds zeros there.

Storage-favoured layout (layout = 2; appendix B.2 of the paper: the weak columns are taken
out of the low-bit matrix).  One scale per row only.  The codes section holds the d_in - k
columns that are not weak, in their original order, as a layout-0 matrix of nblk blocks,
nblk = the smallest count n >= max(1, ceil((d_in - k) / 128)) and <= ceil(d_in / 128) with
n / CW(n) <= ceil(d_in / 128) / CW(ceil(d_in / 128)), i.e. no more tiles per row tile than the
full row has (zero columns fill up the last blocks);
everything else as in layout 0.  One more section follows weak_idx:
wmeta, one little-endian dword per 8 input columns: low byte = weak mask (bit e = column
8i+e is weak), upper 24 bits = number of weak columns before column 8i.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

ALIGN = 256
BLOCK = 128


@dataclass(frozen=True)
class Geometry:
    d_out: int
    d_in: int
    bits: int
    group_size: int
    k: int
    nblk: int
    cw: int
    r: int
    nact: int
    nslab: int
    n_rt: int
    d_out_pad: int
    chunks: int
    n_groups: int
    kp: int
    off_codes: int
    off_sz: int
    off_weak_w: int
    off_weak_idx: int
    total_bytes: int
    layout: int = 0
    nbp: int = 0
    off_wmask: int = 0
    off_scratch: int = 0


def _align(n: int) -> int:
    return (n + ALIGN - 1) // ALIGN * ALIGN


def tile_shape(nblk: int):
    best = 1
    for c in range(1, min(nblk, 64) + 1):
        if nblk % c == 0 and (64 // c) * c >= 60:
            best = c
    return best, 64 // best


TILE_ROWS = 32


def geometry(d_out: int, d_in: int, bits: int, group_size: int, k: int, layout: int = 0) -> Geometry:
    assert bits in (3, 4) and d_out >= 1 and d_in >= 1 and 0 <= k <= d_in
    assert group_size == 0 or group_size % BLOCK == 0
    if layout == 1:
        nbp = -(-d_in // (2 * BLOCK))
        nblk = 2 * nbp
        n_rt = -(-d_out // TILE_ROWS)
        d_out_pad = n_rt * TILE_ROWS
        chunks = 3 if bits == 3 else 4
        n_groups = 1 if group_size == 0 else -(-d_in // group_size)
        kp = -(-k // 8) * 8
        off_sz = _align(n_rt * nbp * 64 * chunks * 16)
        off_weak_w = _align(off_sz + d_out_pad * n_groups * 4)
        off_weak_idx = _align(off_weak_w + d_out_pad * kp * 2)
        off_wmask = _align(off_weak_idx + kp * 4)
        off_scratch = _align(off_wmask + nbp * 32)
        total = off_scratch
        return Geometry(d_out, d_in, bits, group_size, k, nblk, 1, TILE_ROWS, 64, nbp, n_rt,
                        d_out_pad, chunks, n_groups, kp, 0, off_sz, off_weak_w, off_weak_idx,
                        total, 1, nbp, off_wmask, off_scratch)
    if layout == 2:
        assert group_size == 0, "storage-favoured layout: one scale per row"
    nblk = -(-d_in // BLOCK)
    if layout == 2:
        # the stored columns, padded with zero columns up to the first block count that needs
        # no more tiles per row tile than the full row
        full_slabs = nblk // tile_shape(nblk)[0]
        nb = -(-max(d_in - k, 1) // BLOCK)
        while nb < nblk and nb // tile_shape(nb)[0] > full_slabs:
            nb += 1
        nblk = nb
    cw, r = tile_shape(nblk)
    nact = r * cw
    nslab = nblk // cw
    n_rt = -(-d_out // r)
    d_out_pad = n_rt * r
    chunks = 3 if bits == 3 else 4
    n_groups = 1 if group_size == 0 else -(-d_in // group_size)
    kp = -(-k // 8) * 8
    off_codes = 0
    off_sz = _align(off_codes + d_out_pad * nblk * chunks * 16)
    off_weak_w = _align(off_sz + d_out_pad * n_groups * 4)
    off_weak_idx = _align(off_weak_w + d_out_pad * kp * 2)
    total = _align(off_weak_idx + kp * 4)
    if layout == 2:
        off_wmeta = total
        total = _align(off_wmeta + -(-d_in // 8) * 4)
        return Geometry(d_out, d_in, bits, group_size, k, nblk, cw, r, nact, nslab, n_rt,
                        d_out_pad, chunks, n_groups, kp, off_codes, off_sz, off_weak_w,
                        off_weak_idx, total, 2, 0, off_wmeta, 0)
    return Geometry(d_out, d_in, bits, group_size, k, nblk, cw, r, nact, nslab, n_rt,
                    d_out_pad, chunks, n_groups, kp, off_codes, off_sz, off_weak_w,
                    off_weak_idx, total)


# ---------------------------------------------------------------------------
# vectorised packer
# ---------------------------------------------------------------------------

def _lane_dwords(block_codes: np.ndarray, bits: int) -> np.ndarray:
    """[..., 128] uint8 codes of one block -> [..., C*4] uint32 dwords of its lane."""
    lead = block_codes.shape[:-1]
    if bits == 3:
        c = block_codes.reshape(lead + (4, 16, 2)).astype(np.uint64)
        sh = (3 * np.arange(16, dtype=np.uint64)).reshape((1,) * len(lead) + (1, 16))
        lo = np.bitwise_or.reduce(c[..., 0] << sh, axis=-1)       # [..., 4] 48-bit streams
        hi = np.bitwise_or.reduce(c[..., 1] << sh, axis=-1)
        out = np.empty(lead + (4, 3), dtype=np.uint32)
        for w in range(3):
            s = np.uint64(16 * w)
            out[..., w] = (((lo >> s) & np.uint64(0xFFFF)) |
                           (((hi >> s) & np.uint64(0xFFFF)) << np.uint64(16))).astype(np.uint32)
        return out.reshape(lead + (12,))
    c = block_codes.reshape(lead + (16, 4, 2)).astype(np.uint32)
    sh = (4 * np.arange(4, dtype=np.uint32)).reshape((1,) * len(lead) + (1, 4))
    lo = np.bitwise_or.reduce(c[..., 0] << sh, axis=-1)
    hi = np.bitwise_or.reduce(c[..., 1] << sh, axis=-1)
    return (lo | (hi << np.uint32(16))).astype(np.uint32)


def pack_codes(codes: np.ndarray, geo: Geometry) -> np.ndarray:
    """uint8 [d_out, d_in] -> uint8 bytes of the codes section."""
    codes = np.asarray(codes, dtype=np.uint8)
    # layout 2: the caller passes the stored columns only
    assert codes.shape == (geo.d_out, geo.d_in - geo.k if geo.layout == 2 else geo.d_in)
    assert int(codes.max(initial=0)) < (1 << geo.bits)
    full = np.zeros((geo.d_out_pad, geo.nblk * BLOCK), dtype=np.uint8)
    full[:geo.d_out, :codes.shape[1]] = codes
    if geo.layout == 1:
        # [rt, row, bp, b, t, kg, e] -> lanes [rt, bp, kg, row] with lane columns [b, t, e]
        t = full.reshape(geo.n_rt, TILE_ROWS, geo.nbp, 2, 8, 2, 8)
        t = t.transpose(0, 2, 5, 1, 3, 4, 6).reshape(geo.n_rt, geo.nbp, 64, BLOCK)
        dw = _lane_dwords(t, geo.bits).reshape(geo.n_rt, geo.nbp, 64, geo.chunks, 4)
        dw = dw.transpose(0, 1, 3, 2, 4)
        return np.ascontiguousarray(dw).astype("<u4").view(np.uint8).reshape(-1)
    t = full.reshape(geo.n_rt, geo.r, geo.nslab, geo.cw, BLOCK)
    t = t.transpose(0, 2, 1, 3, 4).reshape(geo.n_rt, geo.nslab, geo.nact, BLOCK)
    dw = _lane_dwords(t, geo.bits)                                  # [rt, s, a, C*4]
    dw = dw.reshape(geo.n_rt, geo.nslab, geo.nact, geo.chunks, 4)
    dw = dw.transpose(0, 1, 3, 2, 4)                                # [rt, s, c, a, e]
    return np.ascontiguousarray(dw).astype("<u4").view(np.uint8).reshape(-1)


def pack_layer(codes, scale, zero, group_size, weak_idx, weak_w, bits, layout: int = 0) -> tuple[np.ndarray, Geometry]:
    """The whole blob (uint8) and its geometry.  Codes at weak columns are stored as 0."""
    codes = np.array(codes, dtype=np.uint8, copy=True)
    d_out, d_in = codes.shape
    idx = np.asarray(weak_idx, dtype=np.int32)
    geo = geometry(d_out, d_in, bits, group_size, int(idx.size), layout)
    codes[:, idx] = 0
    blob = np.zeros(geo.total_bytes, dtype=np.uint8)
    is_weak_col = np.zeros(d_in, dtype=bool)
    is_weak_col[idx] = True
    sec = pack_codes(codes[:, ~is_weak_col] if layout == 2 else codes, geo)
    blob[geo.off_codes:geo.off_codes + sec.size] = sec

    s_bits = np.asarray(scale, dtype=np.float16).view(np.uint16).astype(np.uint32)
    z_bits = np.asarray(zero, dtype=np.float16).view(np.uint16).astype(np.uint32)
    assert s_bits.shape == (d_out, geo.n_groups) and z_bits.shape == (d_out, geo.n_groups)
    sz = np.zeros((geo.d_out_pad, geo.n_groups), dtype=np.uint32)
    sz[:d_out] = s_bits | (z_bits << np.uint32(16))
    if geo.layout == 1:
        sz = np.ascontiguousarray(sz.T)               # group-major
    b = sz.astype("<u4").view(np.uint8).reshape(-1)
    blob[geo.off_sz:geo.off_sz + b.size] = b

    ww = np.zeros((geo.d_out_pad, geo.kp), dtype=np.float16)
    ww[:d_out, :geo.k] = np.asarray(weak_w, dtype=np.float16)
    b = ww.view(np.uint8).reshape(-1)
    blob[geo.off_weak_w:geo.off_weak_w + b.size] = b

    ix = np.full(geo.kp, -1, dtype=np.int32)
    ix[:geo.k] = idx
    b = ix.astype("<i4").view(np.uint8).reshape(-1)
    blob[geo.off_weak_idx:geo.off_weak_idx + b.size] = b

    if geo.layout == 1:
        is_weak = np.zeros(geo.nbp * 256, dtype=np.uint8)
        is_weak[idx] = 1
        b = np.packbits(is_weak.reshape(-1, 8), axis=1, bitorder="little").reshape(-1)
        blob[geo.off_wmask:geo.off_wmask + b.size] = b
    if geo.layout == 2:
        padded = np.zeros(-(-d_in // 8) * 8, dtype=np.uint32)
        padded[:d_in] = is_weak_col
        per_unit = padded.reshape(-1, 8)
        mask = (per_unit << np.arange(8, dtype=np.uint32)).sum(axis=1).astype(np.uint32)
        before = np.concatenate([[0], np.cumsum(per_unit.sum(axis=1))[:-1]]).astype(np.uint32)
        b = (mask | (before << np.uint32(8))).astype("<u4").view(np.uint8).reshape(-1)
        blob[geo.off_wmask:geo.off_wmask + b.size] = b
    return blob, geo


# ---------------------------------------------------------------------------
# unpacker (inverse of pack_codes), written as a gather over bit positions
# ---------------------------------------------------------------------------

def _unpack_lanes(dw: np.ndarray, bits: int) -> np.ndarray:
    """[..., C*4] dwords of a lane -> [..., 128] uint8 lane columns (inverse of _lane_dwords)."""
    lead = dw.shape[:-1]
    if bits == 3:
        q = dw.reshape(lead + (4, 3)).astype(np.uint64)
        lo = np.zeros(q.shape[:-1], dtype=np.uint64)
        hi = np.zeros(q.shape[:-1], dtype=np.uint64)
        for w in range(3):
            lo |= (q[..., w] & np.uint64(0xFFFF)) << np.uint64(16 * w)
            hi |= (q[..., w] >> np.uint64(16)) << np.uint64(16 * w)
        sh = 3 * np.arange(16, dtype=np.uint64)
        c = np.stack([(lo[..., None] >> sh) & np.uint64(7), (hi[..., None] >> sh) & np.uint64(7)], axis=-1)
    else:
        q = dw.astype(np.uint32)
        sh = 4 * np.arange(4, dtype=np.uint32)
        c = np.stack([((q & np.uint32(0xFFFF))[..., None] >> sh) & np.uint32(15),
                      ((q >> np.uint32(16))[..., None] >> sh) & np.uint32(15)], axis=-1)
    return c.astype(np.uint8).reshape(lead + (BLOCK,))


def unpack_codes(blob: np.ndarray, geo: Geometry) -> np.ndarray:
    """Codes section of a blob -> uint8 [d_out, d_in]."""
    n_dw = geo.d_out_pad * geo.nblk * geo.chunks * 4
    dw = np.frombuffer(np.asarray(blob, dtype=np.uint8).tobytes(), dtype="<u4",
                       count=n_dw, offset=geo.off_codes)
    if geo.layout == 1:
        lanes = _unpack_lanes(dw.reshape(geo.n_rt, geo.nbp, geo.chunks, 64, 4).transpose(0, 1, 3, 2, 4)
                              .reshape(geo.n_rt, geo.nbp, 64, geo.chunks * 4), geo.bits)
        t = lanes.reshape(geo.n_rt, geo.nbp, 2, TILE_ROWS, 2, 8, 8)          # [rt, bp, kg, row, b, t, e]
        full = t.transpose(0, 3, 1, 4, 5, 2, 6).reshape(geo.d_out_pad, geo.nblk * BLOCK)
        return np.ascontiguousarray(full[:geo.d_out, :geo.d_in])
    dw = dw.reshape(geo.n_rt, geo.nslab, geo.chunks, geo.nact, 4)
    dw = dw.transpose(0, 1, 3, 2, 4).reshape(geo.n_rt, geo.nslab, geo.nact, geo.chunks * 4)
    if geo.bits == 3:
        q = dw.reshape(geo.n_rt, geo.nslab, geo.nact, 4, 3).astype(np.uint64)
        lo = np.zeros(q.shape[:-1], dtype=np.uint64)
        hi = np.zeros(q.shape[:-1], dtype=np.uint64)
        for w in range(3):
            lo |= (q[..., w] & np.uint64(0xFFFF)) << np.uint64(16 * w)
            hi |= (q[..., w] >> np.uint64(16)) << np.uint64(16 * w)
        sh = 3 * np.arange(16, dtype=np.uint64)
        c = np.stack([(lo[..., None] >> sh) & np.uint64(7),
                      (hi[..., None] >> sh) & np.uint64(7)], axis=-1)   # [..., 4, 16, 2]
    else:
        q = dw.astype(np.uint32)
        sh = 4 * np.arange(4, dtype=np.uint32)
        c = np.stack([((q & np.uint32(0xFFFF))[..., None] >> sh) & np.uint32(15),
                      ((q >> np.uint32(16))[..., None] >> sh) & np.uint32(15)], axis=-1)
    blocks = c.astype(np.uint8).reshape(geo.n_rt, geo.nslab, geo.r, geo.cw, BLOCK)
    full = blocks.transpose(0, 2, 1, 3, 4).reshape(geo.d_out_pad, geo.nblk * BLOCK)
    if geo.layout == 2:
        # the stored columns go back to their places; weak columns read as 0
        ix = np.frombuffer(np.asarray(blob, dtype=np.uint8).tobytes(), dtype="<i4", count=geo.kp,
                           offset=geo.off_weak_idx)[:geo.k]
        keep = np.ones(geo.d_in, dtype=bool)
        keep[ix] = False
        out = np.zeros((geo.d_out, geo.d_in), dtype=np.uint8)
        out[:, keep] = full[:geo.d_out, :geo.d_in - geo.k]
        return out
    return np.ascontiguousarray(full[:geo.d_out, :geo.d_in])


def unpack_params(blob: np.ndarray, geo: Geometry):
    """(scale fp16 [d_out,G], zero fp16 [d_out,G], weak_idx int32 [k], weak_w fp16 [d_out,k])."""
    raw = np.asarray(blob, dtype=np.uint8).tobytes()
    sz = np.frombuffer(raw, dtype="<u4", count=geo.d_out_pad * geo.n_groups, offset=geo.off_sz)
    if geo.layout == 1:
        sz = sz.reshape(geo.n_groups, geo.d_out_pad).T[:geo.d_out]
    else:
        sz = sz.reshape(geo.d_out_pad, geo.n_groups)[:geo.d_out]
    scale = (sz & 0xFFFF).astype(np.uint16).view(np.float16)
    zero = (sz >> 16).astype(np.uint16).view(np.float16)
    ww = np.frombuffer(raw, dtype=np.float16, count=geo.d_out_pad * geo.kp, offset=geo.off_weak_w)
    ww = ww.reshape(geo.d_out_pad, geo.kp)[:geo.d_out, :geo.k]
    ix = np.frombuffer(raw, dtype="<i4", count=geo.kp, offset=geo.off_weak_idx)[:geo.k]
    return scale.copy(), zero.copy(), ix.astype(np.int32), ww.copy()


# ---------------------------------------------------------------------------
# scalar address function: one bit of one code at a time
# ---------------------------------------------------------------------------

def bit_address(geo: Geometry, row: int, col: int, bitno: int):
    """(byte offset in the blob, bit within that byte) of bit `bitno` of code (row, col)."""
    if geo.layout == 1:
        rt, rloc = divmod(row, TILE_ROWS)
        bp, c256 = divmod(col, 2 * BLOCK)
        b, c128 = divmod(c256, BLOCK)
        t16, c16 = divmod(c128, 16)
        kg, e = divmod(c16, 8)
        lane = kg * TILE_ROWS + rloc
        tile = rt * geo.nbp + bp
        cin = 64 * b + 8 * t16 + e
    else:
        rt, rloc = divmod(row, geo.r)
        blk, cin = divmod(col, BLOCK)
        s, bloc = divmod(blk, geo.cw)
        lane = rloc * geo.cw + bloc
        tile = rt * geo.nslab + s
    if geo.bits == 3:
        u, within = divmod(cin, 32)
        t, half = divmod(within, 2)
        stream_bit = 3 * t + bitno
        w, bit16 = divmod(stream_bit, 16)
        v = 3 * u + w
    else:
        v, within = divmod(cin, 8)
        t, half = divmod(within, 2)
        bit16 = 4 * t + bitno
    bit32 = bit16 + 16 * half
    chunk, e = divmod(v, 4)
    byte = geo.off_codes + ((tile * geo.chunks + chunk) * geo.nact + lane) * 16 + 4 * e + bit32 // 8
    return byte, bit32 % 8


def pack_codes_bitwise(codes, geo: Geometry) -> np.ndarray:
    """Codes section built one bit at a time through bit_address (slow; tiny layers)."""
    sec = np.zeros(geo.off_sz - geo.off_codes, dtype=np.uint8)
    for i in range(geo.d_out):
        for j in range(geo.d_in):
            q = int(codes[i][j])
            for b in range(geo.bits):
                if (q >> b) & 1:
                    byte, bit = bit_address(geo, i, j, b)
                    sec[byte - geo.off_codes] |= np.uint8(1 << bit)
    return sec[:geo.d_out_pad * geo.nblk * geo.chunks * 16]
