// Host side of the packed format: geometry, validation, packing and unpacking.
//
// What is stored follows the storage paragraph of the paper's "Outlier-Aware
// Weight Quantization" section and appendix B.2 (latency-favoured format): the
// full-size low-bit matrix with zero-filled weak positions, per-channel or
// per-group step size and zero point, fp16 weak columns and their indices.
// The bit layout is this library's own (the paper gives none); it is chosen so
// that a lane of the GEMV kernel fetches one block of 128 codes with three or
// four coalesced 16-byte loads and extracts pairs of codes straight into the
// mantissas of two packed fp16 numbers.
#include <cstring>

#include "owq_internal.h"

namespace owq {

static inline uint64_t align_up(uint64_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

TileScratch tile_scratch(const owq_layer_info_t &g) {
  TileScratch t{};
  t.n_rg = (g.n_rt + kTileGroupTiles - 1) / kTileGroupTiles;
  const int64_t steps = (int64_t)t.n_rg * g.nbp;
  t.grid_max = steps < kTileGridMax ? (int32_t)steps : kTileGridMax;
  t.off_xs = 0;
  t.off_bsum = t.off_xs + (uint64_t)kScratchBatch * g.nbp * 256 * 2;
  t.off_tsum = t.off_bsum + (uint64_t)g.nblk * kScratchBatch * 8;
  t.off_xw = t.off_tsum + 16384;
  t.off_slots = t.off_xw + (uint64_t)kScratchBatch * g.kp * 2;
  t.total = t.off_slots + (uint64_t)(t.grid_max + 2 * t.n_rg) * kTileSlotBytes;
  return t;
}

owq_status_t compute_geometry(int32_t d_out, int32_t d_in, int32_t bits, int32_t group_size,
                              int32_t k, int32_t layout, owq_layer_info_t *g) {
  if (d_out < 1 || d_in < 1) return OWQ_ERR_SHAPE;
  if (bits != 3 && bits != 4) return OWQ_ERR_BITS;
  if (group_size < 0 || (group_size != 0 && group_size % kBlockCols != 0)) return OWQ_ERR_GROUP;
  if (k < 0 || k > d_in) return OWQ_ERR_INDEX;
  if (layout != OWQ_LAYOUT_GEMV && layout != OWQ_LAYOUT_TILE && layout != OWQ_LAYOUT_COMPACT) return OWQ_ERR_LAYOUT;
  if (layout == OWQ_LAYOUT_COMPACT && group_size != 0) return OWQ_ERR_GROUP;
  std::memset(g, 0, sizeof(*g));
  g->format_version = OWQ_FORMAT_VERSION;
  g->d_out = d_out; g->d_in = d_in; g->bits = bits; g->group_size = group_size; g->k = k;
  g->layout = layout;
  if (layout == OWQ_LAYOUT_TILE) {
    // 32 rows x one pair of blocks per tile; lane = (half of the pair's columns, row).
    g->nbp = (d_in + 2 * kBlockCols - 1) / (2 * kBlockCols);
    g->nblk = 2 * g->nbp;
    g->cw = 1; g->r = kTileRows; g->nact = 64; g->nslab = g->nbp;
    g->n_rt = (d_out + kTileRows - 1) / kTileRows;
    g->d_out_pad = g->n_rt * kTileRows;
    g->chunks = bits == 3 ? 3 : 4;
    g->n_groups = group_size == 0 ? 1 : (d_in + group_size - 1) / group_size;
    g->kp = (k + 7) / 8 * 8;
    g->off_codes = 0;
    g->off_sz = align_up((uint64_t)g->n_rt * g->nbp * 64 * g->chunks * 16);
    g->off_weak_w = align_up(g->off_sz + (uint64_t)g->d_out_pad * g->n_groups * 4);
    g->off_weak_idx = align_up(g->off_weak_w + (uint64_t)g->d_out_pad * g->kp * 2);
    g->off_wmask = align_up(g->off_weak_idx + (uint64_t)g->kp * 4);
    g->off_scratch = align_up(g->off_wmask + (uint64_t)g->nbp * 32);
    const TileScratch ts = tile_scratch(*g);
    const uint64_t scratch = ts.total;
    g->total_bytes = align_up(g->off_scratch + scratch);
    if (g->total_bytes >= (1ull << 32)) return OWQ_ERR_SHAPE;
    return OWQ_OK;
  }
  // Tile width of a row of nb blocks: as many blocks side by side as the wave can hold while
  // keeping at least 60 of its 64 lanes busy.
  auto tile_width = [](int32_t nb) {
    int c1 = 1;
    for (int c = 1; c <= 64 && c <= nb; ++c)
      if (nb % c == 0 && (64 / c) * c >= 60) c1 = c;
    return c1;
  };
  const int32_t nblk_full = (d_in + kBlockCols - 1) / kBlockCols;
  g->nblk = nblk_full;
  if (layout == OWQ_LAYOUT_COMPACT) {
    // storage-favoured: only the columns that are not weak are stored (at least one block, of
    // zeros), padded with zero columns up to the first block count that needs no more tiles per
    // row tile than the full row: narrow tiles cost far more time than the blocks saved
    const int32_t d_dense = d_in - k > 0 ? d_in - k : 1;
    int32_t nb = (d_dense + kBlockCols - 1) / kBlockCols;
    while (nb < nblk_full && nb / tile_width(nb) > nblk_full / tile_width(nblk_full)) ++nb;
    g->nblk = nb;
  }
  const int cw = tile_width(g->nblk);
  g->cw = cw;
  g->r = 64 / cw;
  g->nact = g->r * cw;
  g->nslab = g->nblk / cw;
  g->n_rt = (d_out + g->r - 1) / g->r;
  g->d_out_pad = g->n_rt * g->r;
  g->chunks = bits == 3 ? 3 : 4;
  g->n_groups = group_size == 0 ? 1 : (d_in + group_size - 1) / group_size;
  g->kp = (k + 7) / 8 * 8;
  const uint64_t codes_bytes = (uint64_t)g->d_out_pad * g->nblk * g->chunks * 16;
  g->off_codes = 0;
  g->off_sz = align_up(codes_bytes);
  g->off_weak_w = align_up(g->off_sz + (uint64_t)g->d_out_pad * g->n_groups * 4);
  g->off_weak_idx = align_up(g->off_weak_w + (uint64_t)g->d_out_pad * g->kp * 2);
  g->total_bytes = align_up(g->off_weak_idx + (uint64_t)g->kp * 4);
  if (layout == OWQ_LAYOUT_COMPACT) {
    g->off_wmask = g->total_bytes;        // per 8 input columns: weak mask | weak columns before << 8
    g->total_bytes = align_up(g->off_wmask + (uint64_t)((d_in + 7) / 8) * 4);
  }
  // The kernels address the blob with 32-bit byte offsets.
  if (g->total_bytes >= (1ull << 32)) return OWQ_ERR_SHAPE;
  return OWQ_OK;
}

owq_status_t validate_desc(const owq_layer_desc_t *d) {
  if (!d) return OWQ_ERR_NULL;
  owq_layer_info_t g;
  owq_status_t st = compute_geometry(d->d_out, d->d_in, d->bits, d->group_size, d->k, d->layout, &g);
  if (st != OWQ_OK) return st;
  if (!d->codes || !d->scale || !d->zero) return OWQ_ERR_NULL;
  if (d->k > 0 && (!d->weak_idx || !d->weak_w)) return OWQ_ERR_NULL;
  int32_t prev = -1;
  for (int32_t t = 0; t < d->k; ++t) {
    const int32_t j = d->weak_idx[t];
    if (j <= prev || j >= d->d_in) return OWQ_ERR_INDEX;
    prev = j;
  }
  std::vector<uint8_t> weak(d->d_in, 0);
  for (int32_t t = 0; t < d->k; ++t) weak[d->weak_idx[t]] = 1;
  const uint8_t limit = (uint8_t)(1u << d->bits);
  for (int64_t i = 0; i < d->d_out; ++i) {
    const uint8_t *row = d->codes + i * (int64_t)d->d_in;
    uint8_t bad = 0;
    for (int32_t j = 0; j < d->d_in; ++j) bad |= (uint8_t)((row[j] >= limit) & !weak[j]);
    if (bad) return OWQ_ERR_CODE_RANGE;
  }
  return OWQ_OK;
}

// Codes of one block (128 columns of one row, weak and out-of-range columns
// already forced to 0) -> the 12 or 16 dwords its lane owns.
static void block_to_dwords(const uint8_t *q, int bits, uint32_t *dw) {
  if (bits == 3) {
    for (int u = 0; u < 4; ++u) {          // 32 codes -> two 48-bit streams -> 3 dwords
      uint64_t even = 0, odd = 0;
      for (int t = 0; t < 16; ++t) {
        even |= (uint64_t)q[32 * u + 2 * t] << (3 * t);
        odd |= (uint64_t)q[32 * u + 2 * t + 1] << (3 * t);
      }
      for (int w = 0; w < 3; ++w)
        dw[3 * u + w] = (uint32_t)((even >> (16 * w)) & 0xffffu) |
                        ((uint32_t)((odd >> (16 * w)) & 0xffffu) << 16);
    }
  } else {
    for (int v = 0; v < 16; ++v) {
      uint32_t even = 0, odd = 0;
      for (int t = 0; t < 4; ++t) {
        even |= (uint32_t)q[8 * v + 2 * t] << (4 * t);
        odd |= (uint32_t)q[8 * v + 2 * t + 1] << (4 * t);
      }
      dw[v] = even | (odd << 16);
    }
  }
}

void pack_weak_section(const owq_layer_info_t &g, const uint16_t *weak_w, uint16_t *out) {
  std::memset(out, 0, (size_t)g.d_out_pad * g.kp * 2);
  for (int64_t i = 0; i < g.d_out; ++i)
    for (int32_t t = 0; t < g.k; ++t) out[i * g.kp + t] = weak_w[i * (int64_t)g.k + t];
}

void pack_blob(const owq_layer_desc_t *d, const owq_layer_info_t &g, uint8_t *out) {
  std::memset(out, 0, g.total_bytes);
  std::vector<uint8_t> weak(d->d_in, 0);
  for (int32_t t = 0; t < d->k; ++t) weak[d->weak_idx[t]] = 1;

  uint32_t *codes = reinterpret_cast<uint32_t *>(out + g.off_codes);
  uint8_t q[kBlockCols];
  uint32_t dw[16];
  const int ndw = g.chunks * 4;
  if (g.layout == OWQ_LAYOUT_TILE) {
    for (int32_t row = 0; row < g.d_out; ++row) {
      const int32_t rt = row / kTileRows, rloc = row % kTileRows;
      const uint8_t *src = d->codes + (int64_t)row * d->d_in;
      for (int32_t bp = 0; bp < g.nbp; ++bp)
        for (int kg = 0; kg < 2; ++kg) {
          // the lane's 128 codes: for both blocks of the pair, 8 octets at stride 16
          for (int b = 0; b < 2; ++b)
            for (int t = 0; t < 8; ++t)
              for (int e = 0; e < 8; ++e) {
                const int32_t j = bp * 256 + b * 128 + t * 16 + kg * 8 + e;
                q[b * 64 + t * 8 + e] = (j < d->d_in && !weak[j]) ? src[j] : 0;
              }
          block_to_dwords(q, g.bits, dw);
          const int64_t tile = (int64_t)rt * g.nbp + bp;
          const int32_t lane = kg * kTileRows + rloc;
          for (int v = 0; v < ndw; ++v) {
            const int64_t unit = (tile * g.chunks + v / 4) * 64 + lane;
            codes[unit * 4 + (v & 3)] = dw[v];
          }
        }
    }
    uint8_t *wm = out + g.off_wmask;
    for (int32_t j = 0; j < d->d_in; ++j)
      if (weak[j]) wm[j >> 3] |= (uint8_t)(1u << (j & 7));
  } else {
  // stored column -> input column: all of them, or (storage-favoured) those that are not weak
  std::vector<int32_t> col;
  for (int32_t j = 0; j < d->d_in; ++j)
    if (g.layout != OWQ_LAYOUT_COMPACT || !weak[j]) col.push_back(j);
  const int32_t ncol = (int32_t)col.size();
  for (int32_t row = 0; row < g.d_out; ++row) {
    const int32_t rt = row / g.r, rloc = row % g.r;
    const uint8_t *src = d->codes + (int64_t)row * d->d_in;
    for (int32_t blk = 0; blk < g.nblk; ++blk) {
      const int32_t s = blk / g.cw, bloc = blk % g.cw;
      for (int c = 0; c < kBlockCols; ++c) {
        const int32_t jc = blk * kBlockCols + c;
        q[c] = (jc < ncol && !weak[col[jc]]) ? src[col[jc]] : 0;
      }
      block_to_dwords(q, g.bits, dw);
      const int64_t tile = (int64_t)rt * g.nslab + s;
      const int32_t lane = rloc * g.cw + bloc;
      for (int v = 0; v < ndw; ++v) {
        const int64_t unit = (tile * g.chunks + v / 4) * g.nact + lane;   // 16-byte unit
        codes[unit * 4 + (v & 3)] = dw[v];
      }
    }
  }
  if (g.layout == OWQ_LAYOUT_COMPACT) {
    uint32_t *wm = reinterpret_cast<uint32_t *>(out + g.off_wmask);
    uint32_t before = 0;
    for (int32_t i = 0; i < (d->d_in + 7) / 8; ++i) {
      uint32_t m = 0;
      for (int e = 0; e < 8; ++e)
        if (8 * i + e < d->d_in && weak[8 * i + e]) m |= 1u << e;
      wm[i] = m | (before << 8);
      before += (uint32_t)__builtin_popcount(m);
    }
  }
  }

  // single-token layout: [row][group]; tile layout: [group][row], so that the rows of a tile
  // are contiguous
  uint32_t *sz = reinterpret_cast<uint32_t *>(out + g.off_sz);
  for (int64_t i = 0; i < g.d_out; ++i)
    for (int32_t gr = 0; gr < g.n_groups; ++gr) {
      const int64_t src = i * g.n_groups + gr;
      const int64_t dst = g.layout == OWQ_LAYOUT_TILE ? (int64_t)gr * g.d_out_pad + i : src;
      sz[dst] = (uint32_t)d->scale[src] | ((uint32_t)d->zero[src] << 16);
    }

  if (g.k > 0) pack_weak_section(g, d->weak_w, reinterpret_cast<uint16_t *>(out + g.off_weak_w));

  int32_t *ix = reinterpret_cast<int32_t *>(out + g.off_weak_idx);
  for (int32_t t = 0; t < g.kp; ++t) ix[t] = t < g.k ? d->weak_idx[t] : -1;

}

// ---------------------------------------------------------------------------
// launch shape
// ---------------------------------------------------------------------------

int32_t lds_bytes_for(const owq_layer_info_t &g, int32_t rtw, int32_t *xpitch) {
  const int32_t pitch = (g.nblk & 1) ? g.nblk : g.nblk + 1;   // odd pitch: conflict-free transposed writes
  if (xpitch) *xpitch = pitch;
  const int64_t xs = (int64_t)16 * pitch * 16;
  const int64_t xw = ((int64_t)g.kp * 2 + 15) / 16 * 16;
  const int64_t part = ((int64_t)rtw * g.r * g.nblk * 4 + 15) / 16 * 16;
  // the scales and the weak weights of the workgroup's rows, copied as they lie in the layer (scales from
  // the 16-byte unit their first byte falls in: one unit more)
  const int64_t sz = (((int64_t)rtw * g.r * g.n_groups + 3) / 4 + 1) * 16;
  const int64_t wk = (int64_t)rtw * g.r * (g.kp / 8) * 16;
  const int64_t total = xs + xw + part + sz + wk;
  return total > 0x7fffffff ? 0x7fffffff : (int32_t)total;
}

// magic such that n / d == (n * magic) >> 16 for every n in [0, nmax]; 0 if there is none
static uint32_t magic16(uint32_t d, uint32_t nmax) {
  if (d == 0) return 0;
  const uint32_t m = 65536u / d + 1u;
  if ((uint64_t)nmax * m >= (1ull << 32)) return 0;
  for (uint32_t n = 0; n <= nmax; ++n)
    if (((n * m) >> 16) != n / d) return 0;
  return m;
}

bool make_magics(const owq_layer_info_t &g, LaunchShape *s) {
  s->cw_magic = magic16((uint32_t)g.cw, 63);
  s->nslab_magic = magic16((uint32_t)g.nslab, (uint32_t)(g.nslab * s->rsplit));
  s->rsplit_magic = magic16((uint32_t)s->rsplit, (uint32_t)(s->rtw + s->rsplit));
  const uint32_t bpg = g.group_size ? (uint32_t)(g.group_size / kBlockCols) : 1u;
  s->bpg_magic = magic16(bpg, (uint32_t)g.nblk);
  return s->cw_magic && s->nslab_magic && s->rsplit_magic && s->bpg_magic;
}

bool shape_is_valid(const owq_layer_info_t &g, const LaunchShape &s) {
  if (s.rtw < 1 || s.rsplit < 1 || s.waves < 1 || s.waves > 8) return false;
  if (s.rtw % s.rsplit != 0) return false;
  if (((int64_t)g.nslab * s.rsplit) % s.waves != 0) return false;
  if (s.depth != 2 && s.depth != 3 && s.depth != 4 && s.depth != 8) return false;
  if (s.depth == 8 && s.waves > 4) return false;   // that variant is built for 256 threads at most
  return true;
}

LaunchShape default_shape(const owq_layer_info_t &g, int32_t lds_limit) {
  // Small search over (row tiles per workgroup, row splits, waves per workgroup) with a
  // cost model fitted to measurements on MI355X, in units of one tile of one wave:
  // a launch pays a fixed start-up (first bytes from HBM), every wave pays a set-up per
  // (slab, split) item plus its tiles, waves beyond one per SIMD share the SIMD, and
  // staging the activations costs in proportion to the 16-byte units per thread.
  const int kCUs = 256;
  const double startup = 6.0, setup = 1.0, stage_per_unit = 0.2;
  LaunchShape best{};
  double best_cost = 1e300;
  for (int rtw = 1; rtw <= g.n_rt && rtw <= 1024; ++rtw) {
    int32_t xpitch = 0;
    const int32_t lds = lds_bytes_for(g, rtw, &xpitch);
    if (lds > lds_limit) break;
    const int nwg = (g.n_rt + rtw - 1) / rtw;
    for (int rsplit = 1; rsplit <= rtw && rsplit <= 8; ++rsplit) {
      if (rtw % rsplit) continue;
      const int64_t items = (int64_t)g.nslab * rsplit;
      for (int waves = 1; waves <= 8; ++waves) {
        if (items % waves) continue;
        const int ipw = (int)(items / waves);
        const int iters = rtw / rsplit;
        int wg_per_cu = 8 / waves;                       // at most two waves per SIMD
        const int by_lds = (160 * 1024) / (lds > 0 ? lds : 1);
        if (wg_per_cu > by_lds) wg_per_cu = by_lds;
        if (wg_per_cu < 1) wg_per_cu = 1;
        const int rounds = (nwg + kCUs * wg_per_cu - 1) / (kCUs * wg_per_cu);
        int wg_on_cu = (nwg + kCUs - 1) / kCUs;
        if (wg_on_cu > wg_per_cu) wg_on_cu = wg_per_cu;
        const int share = (waves * wg_on_cu + 3) / 4;    // waves per SIMD
        const double units_per_thread = (double)g.nblk * 16 / (waves * 64);
        const double wave_work = ipw * (setup + iters) * share + stage_per_unit * units_per_thread * wg_on_cu;
        double cost = rounds * (startup + wave_work);
        if (nwg < kCUs) cost *= 1.0 + 0.5 * (kCUs - nwg) / (double)kCUs;   // idle CUs
        cost += 1e-3 * waves - 1e-4 * iters;             // ties: fewer waves, more tiles per wave
        if (cost < best_cost) {
          best_cost = cost;
          best.rtw = rtw; best.rsplit = rsplit; best.waves = waves;
          best.nwg = nwg; best.lds_bytes = lds; best.xpitch = xpitch;
        }
      }
    }
  }
  // Tiles in flight per wave.  Every load instruction in flight holds one of a compute unit's request slots
  // (measured: beyond about 48 of them further loads wait at issue and the waves with them), and a deeper
  // pipeline only pays with enough tiles per wave to fill it; a wave with several (slab, split) items drains
  // its pipeline at every item, which a depth above 3 made worse on the layers measured.
  best.depth = 2;
  if (best.rtw >= 1) {
    const int iters = best.rtw / best.rsplit;
    const int items_per_wave = (int)(((int64_t)g.nslab * best.rsplit) / best.waves);
    if (iters >= 5) {
      for (int d = 3; d <= 4; ++d)
        if (best.waves * d * g.chunks <= 48) best.depth = d;
      if (items_per_wave > 1 && best.depth > 3) best.depth = 3;
    }
  }
  if (best.rtw >= 1 && !make_magics(g, &best)) best.rtw = 0;
  return best;
}

}  // namespace owq

// ---------------------------------------------------------------------------
// entry points that need no GPU (see include/owq.h)
// ---------------------------------------------------------------------------
using namespace owq;

extern "C" {

owq_status_t owq_geometry(const owq_layer_desc_t *desc, owq_layer_info_t *info) {
  if (!desc || !info) return OWQ_ERR_NULL;
  return compute_geometry(desc->d_out, desc->d_in, desc->bits, desc->group_size, desc->k, desc->layout, info);
}

owq_status_t owq_packed_bytes(const owq_layer_desc_t *desc, size_t *bytes) {
  if (!desc || !bytes) return OWQ_ERR_NULL;
  owq_layer_info_t g;
  owq_status_t st = compute_geometry(desc->d_out, desc->d_in, desc->bits, desc->group_size, desc->k, desc->layout, &g);
  if (st != OWQ_OK) return st;
  *bytes = (size_t)g.total_bytes;
  return OWQ_OK;
}

owq_status_t owq_pack_host(const owq_layer_desc_t *desc, void *host_buf, size_t bytes) {
  if (!desc || !host_buf) return OWQ_ERR_NULL;
  owq_status_t st = validate_desc(desc);
  if (st != OWQ_OK) return st;
  owq_layer_info_t g;
  compute_geometry(desc->d_out, desc->d_in, desc->bits, desc->group_size, desc->k, desc->layout, &g);
  if (bytes < g.total_bytes) return OWQ_ERR_BUFFER;
  pack_blob(desc, g, static_cast<uint8_t *>(host_buf));
  return OWQ_OK;
}

owq_status_t owq_unpack_codes(const void *host_packed, const owq_layer_info_t *info, uint8_t *codes) {
  if (!host_packed || !info || !codes) return OWQ_ERR_NULL;
  owq_layer_info_t g;
  owq_status_t st = compute_geometry(info->d_out, info->d_in, info->bits, info->group_size, info->k, info->layout, &g);
  if (st != OWQ_OK) return st;
  const uint32_t *dwords = reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(host_packed) + g.off_codes);
  const uint32_t *wmeta = reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(host_packed) + g.off_wmask);
  for (int32_t row = 0; row < g.d_out; ++row) {
    const int32_t rt = row / g.r, rloc = row % g.r;
    for (int32_t jin = 0; jin < g.d_in; ++jin) {
      int32_t j = jin;             // stored column
      if (g.layout == OWQ_LAYOUT_COMPACT) {
        const uint32_t meta = wmeta[jin >> 3], m = meta & 0xffu;
        if ((m >> (jin & 7)) & 1u) {          // weak columns are not stored: code 0
          codes[(int64_t)row * g.d_in + jin] = 0;
          continue;
        }
        j = jin - (int32_t)((meta >> 8) + (uint32_t)__builtin_popcount(m & ((1u << (jin & 7)) - 1u)));
      }
      int32_t cin, lane;
      int64_t tile;
      if (g.layout == OWQ_LAYOUT_TILE) {
        const int32_t c256 = j % 256, c128 = c256 % 128, c16 = c128 % 16;
        cin = 64 * (c256 / 128) + 8 * (c128 / 16) + c16 % 8;
        lane = (c16 / 8) * kTileRows + rloc;
        tile = (int64_t)rt * g.nbp + j / 256;
      } else {
        const int32_t blk = j / kBlockCols;
        cin = j % kBlockCols;
        tile = (int64_t)rt * g.nslab + blk / g.cw;
        lane = rloc * g.cw + blk % g.cw;
      }
      int v, bit;          // dword of the lane, bit inside its 16-bit half
      uint32_t code = 0;
      const int half = cin & 1;
      if (g.bits == 3) {
        const int u = cin / 32, t = (cin % 32) / 2;
        for (int b = 0; b < 3; ++b) {
          const int sb = 3 * t + b;
          v = 3 * u + sb / 16;
          bit = sb % 16 + 16 * half;
          const int64_t unit = (tile * g.chunks + v / 4) * g.nact + lane;
          code |= ((dwords[unit * 4 + (v & 3)] >> bit) & 1u) << b;
        }
      } else {
        v = cin / 8;
        bit = 4 * ((cin % 8) / 2) + 16 * half;
        const int64_t unit = (tile * g.chunks + v / 4) * g.nact + lane;
        code = (dwords[unit * 4 + (v & 3)] >> bit) & 15u;
      }
      codes[(int64_t)row * g.d_in + jin] = (uint8_t)code;
    }
  }
  return OWQ_OK;
}

}  // extern "C"
