// GEMV kernel of the OWQ mixed-precision linear layer for gfx950 (batch rows are
// independent launches in grid.y).
//
// Computes, per output row i (paper: storage paragraph of "Outlier-Aware Weight
// Quantization" and section "Acceleration on Real Device"):
//     y_i = sum_{j not weak} s_ig (q_ij - z_ig) x_j  +  sum_t Ww_it x_{idx_t}
// in ONE launch: the weak-column product rides along with the dense stream
// instead of being a second kernel.
//
// Work split.  A block is 128 consecutive columns of one row; one lane owns one
// (row, block) pair per step and keeps the 128 activations of its block in 64
// registers for all the rows it visits.  A wave covers a tile of r rows by cw
// blocks per step and walks down the rows of its workgroup.  Lanes write one
// fp32 partial per (row, block) to LDS; after a barrier 16-lane groups add the
// partials of a row in a fixed order (no atomics: results are reproducible).
//
// Unpack.  A pair of codes is masked out of a dword and OR-ed into the
// mantissas of two packed fp16 constants 2^(10-o), o = bit offset of the field
// inside its 16-bit half: the pair then reads (2^(10-o) + q) exactly, and one
// packed dot product with the activations does two multiply-adds in fp32.  The
// constant part, sum_j 2^(10-o_j) x_j, depends only on the block's activations
// and is subtracted once per (row, block), together with z * sum_j x_j.
#include <hip/hip_runtime.h>

#include "owq_gemv_device.h"

namespace owq {

// Template parameters: code width; tiles in flight per wave; whether the layer has
// weak columns; XN = how many 16-byte units of activations a thread fetches into
// registers ahead of the weight stream (needs x 16-byte aligned and d_in a multiple of
// 8; 0 = general path with scalar loads).  Units beyond XN per thread follow in a loop.
// With 8 tiles in flight a wave needs the register file of a whole SIMD: at most 4 waves
// per workgroup then.
// COMPACT: the layer stores only the columns that are not weak (storage-favoured layout): the
// staging moves their activations together and drops the weak ones into their own array.
// DIRECT = 16, 32 or 64: a tile row holds ALL blocks of a row (one slab of that many blocks) and
// no weak chunk lies beyond one per block: a wave then owns whole rows, adds the partials of a
// tile row across its lanes right after the tile and stores y itself; no partials in LDS, no
// second barrier, no reduction phase.  0: rows are shared by waves (several slabs) and added up
// through LDS after the main loop, one partial per (row, block).  128: rows of several slabs of 64
// blocks: a wave adds its tile row across the lanes as above and leaves one sum per (row, slab) in
// LDS; after the barrier only the slabs' sums are left to add.
template <int BITS, int DEPTH, bool HAS_WEAK, int XN, bool COMPACT = false, int DIRECT = 0>
__global__ __launch_bounds__(DEPTH == 8 ? 256 : 512) void owq_gemv_kernel(const GemvPacked packed) {
  const GemvArgs a = packed.unpack();
  constexpr int CH = BITS == 3 ? 3 : 4;
  constexpr bool FAST = XN > 0;
  constexpr int XCH = FAST ? XN : 1;
  extern __shared__ uint4 smem[];
  uint4 *xs = smem;                                             // [16][xpitch] units of 8 fp16
  _Float16 *xs_h = reinterpret_cast<_Float16 *>(smem);
  const int xw_units = (a.kp * 2 + 15) >> 4;
  uint4 *xw_u = smem + 16 * a.xpitch;                           // activations of the weak columns
  _Float16 *xw = reinterpret_cast<_Float16 *>(xw_u);
  float *part = reinterpret_cast<float *>(xw_u + xw_units);     // [rows of the workgroup][ppitch]
  // scales and weak weights of the workgroup's rows (contiguous in the layer, copied as they are)
  uint4 *lsz_u = xw_u + xw_units + ((a.rtw * a.r * a.ppitch + 3) >> 2);
  const u32 *lsz = reinterpret_cast<const u32 *>(lsz_u);
  uint4 *lwk_u = lsz_u + (((a.rtw * a.r * a.n_groups + 3) >> 2) + 1);

  const int tid = threadIdx.x, nthr = a.nthr;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
  const _Float16 *xn = a.x + (size_t)blockIdx.y * a.d_in;
  _Float16 *yn = a.y + (size_t)blockIdx.y * a.d_out;
  const int nunits = a.nblk * 16;

  const bool active = lane < a.nact;
  const int al = active ? lane : 0;
  const int rloc = (int)(((u32)al * a.cw_magic) >> 16), bloc = al - rloc * a.cw;
  const int rt0 = blockIdx.x * a.rtw;
  const int rt_end = min(a.n_rt, rt0 + a.rtw);
  const u32 tile_bytes = (u32)(CH * a.nact) * 16u;
  const u32 chunk_bytes = (u32)a.nact * 16u;
  const char *codes_b = reinterpret_cast<const char *>(a.codes);
  const char *sz_b = reinterpret_cast<const char *>(a.sz);
  // A pointer read from memory is a generic one to the compiler; it is marked as pointing to
  // global memory here so that the loads through it stay global loads with exact wait counts.
  typedef const __attribute__((address_space(1))) char *gptr_t;
  gptr_t wk_b = (gptr_t)reinterpret_cast<const char *>(a.weak_w);
  if (HAS_WEAK && a.task_id != nullptr) {          // same for the whole workgroup
    const int t = a.task_id[blockIdx.y];
    if ((u32)t < (u32)a.n_sets) wk_b = (gptr_t)static_cast<const char *>(a.weak_sets[t]);
  }

  // ---- (1) loads the set-up needs: activations and weak indices ------------------
  // Issued before the weight stream: loads complete in order, so waiting for
  // these does not wait for the weights behind them.  No branches: units past the
  // end re-read unit 0 and are dropped below, so that the number of loads in
  // flight is fixed and the waits can be exact.
  const u32 *wmeta = reinterpret_cast<const u32 *>(a.weak_idx);     // COMPACT only
  uint4 xv[XCH];
  u32 wmv[XCH];
  int idx0 = -1;
  if (FAST) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int i = tid + j * nthr;
      const int ic = (i * 8 < a.d_in) ? i : 0;
      xv[j] = *reinterpret_cast<const uint4 *>(xn + ic * 8);
      if (COMPACT) wmv[j] = wmeta[ic];
    }
  }
  if (HAS_WEAK && !COMPACT) idx0 = a.weak_idx[tid < a.kp ? tid : 0];
  // The scales and the weak weights of the workgroup's rows are two contiguous pieces of the
  // layer: fetched here with 16-byte loads and handed round through LDS, so that the weight
  // stream below is the only thing the steady state asks memory for (every load instruction in
  // flight takes one of a compute unit's few request slots, whatever its size).
  const int rows_wg = (rt_end - rt0) * a.r;
  const u32 sz0 = (u32)(rt0 * a.r * a.n_groups) * 4u, sz_al = sz0 & ~15u;
  const int sz_units = rows_wg > 0 ? (int)((sz0 - sz_al + (u32)(rows_wg * a.n_groups) * 4u + 15u) >> 4) : 0;
  const int wk_units = HAS_WEAK ? rows_wg * a.kchunks : 0;
  const u32 wk0 = (u32)(rt0 * a.r * a.kchunks) * 16u;
  constexpr int SU = 2;                       // units per thread fetched ahead; more follow in a loop
  u32x4 szv[SU], wkv[SU];
#pragma unroll
  for (int j = 0; j < SU; ++j) {
    const int i = tid + j * nthr;
    szv[j] = *reinterpret_cast<const u32x4 *>(sz_b + (sz_al + (u32)(i < sz_units ? i : 0) * 16u));
    if (HAS_WEAK)
      wkv[j] = *((const __attribute__((address_space(1))) u32x4 *)(wk_b + (wk0 + (u32)(i < wk_units ? i : 0) * 16u)));
  }

  // ---- (2) per-item state and the tile pipeline ---------------------------------
  u32x4 buf[DEPTH][CH];
  u32 szb[DEPTH];
  u32x4 wkb[DEPTH];
  int item = wave;
  int blk = 0, niter = 0, niter_r = 0;
  bool wk = false;
  u32 off_c = 0, off_s = 0, off_w = 0;       // next tile to fetch: byte offset of its codes, LDS indices of its scales and weak chunk
  u32 str_c = 0, str_s = 0, str_w = 0;       // their strides per tile
  int fetched = 0, sided = 0;                // tiles whose codes / whose scales have been fetched so far for this item
  int pidx = 0, pstr = 0;                    // LDS index of the partial (DIRECT: output row), stride per tile

  auto set_item = [&](int it_) {
    const int q = (int)(((u32)it_ * a.nslab_magic) >> 16), s = it_ - q * a.nslab;
    blk = s * a.cw + bloc;
    const int grp = a.blocks_per_group ? (int)(((u32)blk * a.bpg_magic) >> 16) : 0;
    const int span = rt_end - rt0 - q;
    niter = span > 0 ? (int)(((u32)(span + a.rsplit - 1) * a.rsplit_magic) >> 16) : 0;
    niter_r = (niter + DEPTH - 1) / DEPTH * DEPTH;
    wk = HAS_WEAK && active && blk < a.kchunks;
    const int rt = rt0 + q;
    const int row = rt * a.r + rloc;
    off_c = (u32)(rt * a.nslab + s) * tile_bytes + (u32)al * 16u;
    str_c = (u32)(a.rsplit * a.nslab) * tile_bytes;
    const int rowl = q * a.r + rloc;            // row within the workgroup
    off_s = ((sz0 - sz_al) >> 2) + (u32)(rowl * a.n_groups + grp);
    str_s = (u32)(a.rsplit * a.r * a.n_groups);
    off_w = wk ? (u32)(rowl * a.kchunks + blk) : 0u;
    str_w = wk ? (u32)(a.rsplit * a.r * a.kchunks) : 0u;
    fetched = 0; sided = 0;
    pidx = DIRECT == 128 ? (q * a.r + rloc) * a.nslab + s : DIRECT ? row : (q * a.r + rloc) * a.ppitch + blk;
    pstr = DIRECT == 128 ? a.rsplit * a.r * a.nslab : DIRECT ? a.rsplit * a.r : a.rsplit * a.r * a.ppitch;
  };
  // the lane of a tile row that stores its sum (DIRECT): the first of the last 16 lanes
  const bool storer = DIRECT && bloc == (DIRECT == 128 ? 64 : DIRECT) - 16;
  auto finish_tile = [&](float p, bool real) {
    if (DIRECT == 128) {
      const float s = tile_row_sum<64>(p);
      if (storer && real) part[pidx] = s;
    } else if (DIRECT) {
      const float s = tile_row_sum<DIRECT ? DIRECT : 16>(p);
      if (storer && real && pidx < a.d_out) yn[pidx] = (_Float16)s;
    } else if (active && real) {
      part[pidx] = p;
    }
    pidx += pstr;
  };
  // Fetch the next tile into slot d.  Past the last tile every lane reads byte 0
  // of its section instead (one cache line per load), so that the number of loads
  // in flight is the same on every path.
  auto issue = [&](int d) {
    const bool live = fetched < niter;        // uniform
    const u32 oc = live ? off_c : 0u, cs = live ? chunk_bytes : 0u;
#pragma unroll
    for (int c = 0; c < CH; ++c)
      buf[d][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(codes_b + (oc + (u32)c * cs)));
    off_c += str_c;
    ++fetched;
  };
  // The same for the item after the current one: its first DEPTH tiles go out behind the current item's last
  // ones, so that the pipeline does not drain where a wave changes slab.
  u32 nf_off = 0, nf_str = 0;
  int nf_n = 0, nf_done = 0;
  auto peek_item = [&](int it_) {
    const int q = (int)(((u32)it_ * a.nslab_magic) >> 16), s = it_ - q * a.nslab;
    const int span = rt_end - rt0 - q;
    nf_n = span > 0 ? (int)(((u32)(span + a.rsplit - 1) * a.rsplit_magic) >> 16) : 0;
    nf_off = (u32)((rt0 + q) * a.nslab + s) * tile_bytes + (u32)al * 16u;
    nf_str = (u32)(a.rsplit * a.nslab) * tile_bytes;
    nf_done = 0;
  };
  auto issue_next = [&](int d) {
    const bool live = nf_done < nf_n;         // uniform
    const u32 oc = live ? nf_off : 0u, cs = live ? chunk_bytes : 0u;
#pragma unroll
    for (int c = 0; c < CH; ++c)
      buf[d][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(codes_b + (oc + (u32)c * cs)));
    nf_off += nf_str;
    ++nf_done;
  };
  // The scales and the weak chunk of the same tile, from LDS (after the barrier that follows their staging).
  auto side = [&](int d) {
    const bool live = sided < niter;          // uniform
    szb[d] = lsz[live ? off_s : 0u];
    if (HAS_WEAK) {
      const uint4 t4 = lwk_u[live ? off_w : 0u];
      wkb[d] = (u32x4){t4.x, t4.y, t4.z, t4.w};
    }
    off_s += str_s; off_w += str_w;
    ++sided;
  };

  // Only the first two tiles go out ahead of the activations' arrival: more would
  // queue up in front of the set-up's own loads and delay it.
  constexpr int EARLY = DEPTH < 2 ? DEPTH : 2;
  set_item(item);                             // waves <= items: every wave has a first item
#pragma unroll
  for (int d = 0; d < EARLY; ++d) issue(d);

  // ---- (3) activations -> LDS, transposed to [unit-in-block][block] -------------
  if (COMPACT) {
    // Column j goes to stored column j - (weak columns before j), or, if weak, to element
    // (weak columns before j) of the weak activations.  Units without a weak column whose
    // shift is a multiple of 8 move whole.
    auto place = [&](int i, const uint4 &v, u32 meta) {
      const u32 m = meta & 0xffu;
      const int r = (int)(meta >> 8);
      if (m == 0u && (r & 7) == 0 && i * 8 + 8 <= a.d_in) {
        const int u = i - (r >> 3);
        xs[(u & 15) * a.xpitch + (u >> 4)] = v;
        return;
      }
      const u32 w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (i * 8 + e >= a.d_in) continue;
        const unsigned short h = (unsigned short)(w4[e >> 1] >> (16 * (e & 1)));
        const int rr = r + __builtin_popcount(m & ((1u << e) - 1u));
        unsigned short *dst;
        if ((m >> e) & 1u) {
          dst = reinterpret_cast<unsigned short *>(xw) + rr;
        } else {
          const int c = i * 8 + e - rr, u = c >> 3;
          dst = reinterpret_cast<unsigned short *>(xs_h) + (((u & 15) * a.xpitch + (u >> 4)) * 8 + (c & 7));
        }
        *dst = h;
      }
    };
    for (int c = a.d_in - a.k + tid; c < a.nblk * 128; c += nthr) {      // past the last stored column
      const int u = c >> 3;
      xs_h[((u & 15) * a.xpitch + (u >> 4)) * 8 + (c & 7)] = (_Float16)0;
    }
    for (int t = a.k + tid; t < a.kp; t += nthr) xw[t] = (_Float16)0;
    if (FAST) {
#pragma unroll
      for (int j = 0; j < XCH; ++j) {
        const int i = tid + j * nthr;
        if (i * 8 < a.d_in) place(i, xv[j], wmv[j]);
      }
      for (int i = tid + XCH * nthr; i * 8 < a.d_in; i += nthr)         // very wide layers only
        place(i, *reinterpret_cast<const uint4 *>(xn + i * 8), wmeta[i]);
    } else {
      const bool vec = ((reinterpret_cast<uintptr_t>(xn) & 15) == 0) && ((a.d_in & 7) == 0);
      for (int i = tid; i * 8 < a.d_in; i += nthr) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (vec) {
          v = *reinterpret_cast<const uint4 *>(xn + i * 8);
        } else {
          _Float16 e[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            const int j = i * 8 + t;
            e[t] = j < a.d_in ? xn[j] : (_Float16)0;
          }
          v = *reinterpret_cast<const uint4 *>(e);
        }
        place(i, v, wmeta[i]);
      }
    }
  } else if (FAST) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int i = tid + j * nthr;
      if (i < nunits) xs[(i & 15) * a.xpitch + (i >> 4)] = (i * 8 < a.d_in) ? xv[j] : make_uint4(0, 0, 0, 0);
    }
    for (int i = tid + XCH * nthr; i < nunits; i += nthr) {       // very wide layers only
      uint4 v = make_uint4(0, 0, 0, 0);
      if (i * 8 < a.d_in) v = *reinterpret_cast<const uint4 *>(xn + i * 8);
      xs[(i & 15) * a.xpitch + (i >> 4)] = v;
    }
  } else {
    const bool vec = ((reinterpret_cast<uintptr_t>(xn) & 15) == 0) && ((a.d_in & 7) == 0);
    for (int i = tid; i < nunits; i += nthr) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (vec) {
        if (i * 8 < a.d_in) v = *reinterpret_cast<const uint4 *>(xn + i * 8);
      } else {
        _Float16 e[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int j = i * 8 + t;
          e[t] = j < a.d_in ? xn[j] : (_Float16)0;
        }
        v = *reinterpret_cast<const uint4 *>(e);
      }
      xs[(i & 15) * a.xpitch + (i >> 4)] = v;
    }
  }
#pragma unroll
  for (int d = EARLY; d < DEPTH; ++d) issue(d);   // the activations have arrived: fill the pipeline
  __syncthreads();
  // Move the activations of the weak columns to their own array and clear them in
  // the staged copy: the dense path must contribute nothing there.  The index list
  // is the only layer data this waits for, and it is small.
  if (HAS_WEAK && !COMPACT) {
    auto gather = [&](int t, int j) {
      _Float16 v = (_Float16)0;
      if (j >= 0) {
        const int b = j >> 7, u = (j >> 3) & 15, e = j & 7;
        const int pos = (u * a.xpitch + b) * 8 + e;
        v = xs_h[pos];
        xs_h[pos] = (_Float16)0;
      }
      xw[t] = v;
    };
    if (tid < a.kp) gather(tid, idx0);
    for (int t = tid + nthr; t < a.kp; t += nthr) gather(t, a.weak_idx[t]);
    __syncthreads();
  }

  // ---- (4) main loop over the wave's (slab, row split) items ----------------------
  Magic M;
  M.init();
  bool side_staged = false;
  for (;;) {
    u32 xr[64];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const uint4 v = xs[u * a.xpitch + blk];
      xr[4 * u + 0] = v.x; xr[4 * u + 1] = v.y; xr[4 * u + 2] = v.z; xr[4 * u + 3] = v.w;
    }
    u32x4 xwr = {0u, 0u, 0u, 0u};
    if (HAS_WEAK) {
      const uint4 t4 = xw_u[wk ? blk : 0];
      if (wk) { xwr.x = t4.x; xwr.y = t4.y; xwr.z = t4.z; xwr.w = t4.w; }
    }
    float X, Bc;
    block_sums<BITS>(xr, X, Bc);
    if (!side_staged) {                       // first item only; same for the whole workgroup
#pragma unroll
      for (int j = 0; j < SU; ++j) {
        const int i = tid + j * nthr;
        if (i < sz_units) lsz_u[i] = make_uint4(szv[j].x, szv[j].y, szv[j].z, szv[j].w);
        if (HAS_WEAK && i < wk_units) lwk_u[i] = make_uint4(wkv[j].x, wkv[j].y, wkv[j].z, wkv[j].w);
      }
      for (int i = tid + SU * nthr; i < sz_units; i += nthr)          // many groups or rows only
        lsz_u[i] = *reinterpret_cast<const uint4 *>(sz_b + (sz_al + (u32)i * 16u));
      if (HAS_WEAK)
        for (int i = tid + SU * nthr; i < wk_units; i += nthr) {
          const u32x4 v = *((const __attribute__((address_space(1))) u32x4 *)(wk_b + (wk0 + (u32)i * 16u)));
          lwk_u[i] = make_uint4(v.x, v.y, v.z, v.w);
        }
      __syncthreads();
      side_staged = true;
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) side(d);

    int it0 = 0;
    // steady state: every tile of the trip is real; fetch DEPTH tiles ahead
    for (; it0 + DEPTH < niter_r; it0 += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        finish_tile(tile_partial<BITS, HAS_WEAK>(buf[d], szb[d], wkb[d], xwr, xr, M, X, Bc), true);
        issue(d);
        side(d);
      }
    }
    // last trip of the item: tiles past its end are computed on filler and dropped; behind each tile goes a
    // tile of the wave's next item, if it has one
    const bool more = item + nwaves < a.items;
    const bool ahead = more && niter_r > 0;
    if (ahead) {
      peek_item(item + nwaves);
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        finish_tile(tile_partial<BITS, HAS_WEAK>(buf[d], szb[d], wkb[d], xwr, xr, M, X, Bc), it0 + d < niter);
        issue_next(d);
      }
    } else if (niter_r > 0) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        finish_tile(tile_partial<BITS, HAS_WEAK>(buf[d], szb[d], wkb[d], xwr, xr, M, X, Bc), it0 + d < niter);
      }
    }
    if (!more) break;
    item += nwaves;
    set_item(item);
    if (ahead) {
      off_c = nf_off;                          // DEPTH tiles of this item are in flight already
      fetched = DEPTH;
    } else {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) issue(d);
    }
  }
  if (DIRECT && DIRECT != 128) return;
  __syncthreads();
  if (DIRECT == 128) {
    // the sums of a row's slabs, in slab order
    for (int rs = tid; rs < (rt_end - rt0) * a.r; rs += nthr) {
      float sum = 0.f;
      for (int s = 0; s < a.nslab; ++s) sum += part[rs * a.nslab + s];
      const int row = rt0 * a.r + rs;
      if (row < a.d_out) yn[row] = (_Float16)sum;
    }
    return;
  }

  // ---- (5) add the partials of each row; weak chunks beyond one per block -------
  // A group of 16 lanes takes up to four rows at a time: their LDS reads go out together
  // and the four reductions overlap.  Reads past the end of a row are clamped and dropped by
  // select.
  const int rows_here = (rt_end - rt0) * a.r;
  const int l16 = tid & 15, groups = nthr >> 4;
  for (int rs0 = tid >> 4; rs0 < rows_here; rs0 += 4 * groups) {
    float sum[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int rs = rs0 + j * groups;
      const float *pr = part + rs * a.ppitch;
      float acc = 0.f;
      if (rs < rows_here)
      for (int b0 = l16; b0 < a.nblk; b0 += 64) {
        float v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int b = b0 + 16 * t;
          v[t] = pr[b < a.nblk ? b : a.nblk - 1];
          v[t] = b < a.nblk ? v[t] : 0.f;
        }
        acc += (v[0] + v[1]) + (v[2] + v[3]);
      }
      sum[j] = acc;
    }
    if (HAS_WEAK && a.kchunks > a.nblk) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int rs = rs0 + j * groups;
        const int row = rt0 * a.r + rs;
        if (rs < rows_here)
        for (int c = a.nblk + l16; c < a.kchunks; c += 16) {
          const u32x4 wv = ((const __attribute__((address_space(1))) u32x4 *)wk_b)[row * a.kchunks + c];
          const uint4 xv4 = xw_u[c];
          sum[j] = dot2(wv.x, xv4.x, sum[j]);
          sum[j] = dot2(wv.y, xv4.y, sum[j]);
          sum[j] = dot2(wv.z, xv4.z, sum[j]);
          sum[j] = dot2(wv.w, xv4.w, sum[j]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) sum[j] = row16_sum(sum[j]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int rs = rs0 + j * groups, row = rt0 * a.r + rs;
      if (l16 == 0 && rs < rows_here && row < a.d_out) yn[row] = (_Float16)sum[j];
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

typedef void (*kernel_fn)(const GemvPacked);

template <int BITS, int DEPTH, bool WEAK, bool COMPACT>
static kernel_fn pick3(int xn, int direct) {
  if constexpr (!COMPACT && DEPTH <= 4) {         // the shapes a wave can own whole rows of: 2048, 4096, 8192 columns
    if (xn == 4) {
      if (direct == 16) return owq_gemv_kernel<BITS, DEPTH, WEAK, 4, false, 16>;
      if (direct == 32) return owq_gemv_kernel<BITS, DEPTH, WEAK, 4, false, 32>;
      if (direct == 64) return owq_gemv_kernel<BITS, DEPTH, WEAK, 4, false, 64>;
    }
    if (xn == 8 && direct == 128) return owq_gemv_kernel<BITS, DEPTH, WEAK, 8, false, 128>;
  }
  if (xn == 4) return owq_gemv_kernel<BITS, DEPTH, WEAK, 4, COMPACT>;
  if (xn == 8) return owq_gemv_kernel<BITS, DEPTH, WEAK, 8, COMPACT>;
  return owq_gemv_kernel<BITS, DEPTH, WEAK, 0, COMPACT>;
}

// The storage-favoured layout always runs the variant with weak columns (k = 0 stores the same
// bytes as the other layout and takes the same kernel as it).
template <int BITS>
static kernel_fn pick2(int depth, bool weak, int xn, bool compact, int direct) {
  if (compact) {
    if (depth == 2) return pick3<BITS, 2, true, true>(xn, 0);
    if (depth == 3) return pick3<BITS, 3, true, true>(xn, 0);
    if (depth == 4) return pick3<BITS, 4, true, true>(xn, 0);
    return pick3<BITS, 8, true, true>(xn, 0);
  }
  if (depth == 2) return weak ? pick3<BITS, 2, true, false>(xn, direct) : pick3<BITS, 2, false, false>(xn, direct);
  if (depth == 3) return weak ? pick3<BITS, 3, true, false>(xn, direct) : pick3<BITS, 3, false, false>(xn, direct);
  if (depth == 4) return weak ? pick3<BITS, 4, true, false>(xn, direct) : pick3<BITS, 4, false, false>(xn, direct);
  return weak ? pick3<BITS, 8, true, false>(xn, 0) : pick3<BITS, 8, false, false>(xn, 0);
}

static kernel_fn pick(int bits, int depth, bool weak, int xn, bool compact = false, int direct = 0) {
  return bits == 3 ? pick2<3>(depth, weak, xn, compact, direct) : pick2<4>(depth, weak, xn, compact, direct);
}

int prepare_kernels(int32_t lds) {
  if (lds <= 64 * 1024) return (int)hipSuccess;
  for (int bits = 3; bits <= 4; ++bits)
    for (int depth : {2, 3, 4, 8})
      for (int w = 0; w < 3; ++w)            // without weak columns, with, storage-favoured
        for (int xn = 0; xn <= 8; xn += 4)
          for (int direct = 0; direct <= 128; direct = direct ? direct * 2 : 16) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick(bits, depth, w != 0, xn, w == 2, direct)),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return (int)e;
          }
  return (int)hipSuccess;
}

int device_lds_limit(int32_t *bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  int v = 0;
  e = hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) return (int)e;
  *bytes = v;
  return (int)hipSuccess;
}

int launch_gemv(const owq_layer_info_t &g, const LaunchShape &s, const DeviceLayer &dev, const TaskSets &tasks,
                const void *x, void *y, int32_t batch, int32_t lds_limit, void *stream) {
  if (batch >= 2 && tasks.task_id == nullptr) {     // two tokens per pass over the weights, where that fits
    const int r = launch_gemv_multi(g, s, dev, lds_limit, x, y, batch, stream);
    if (r > 0) return r;
    if (r == 0) {                                   // pairs done; an odd last token goes through the code below
      if ((batch & 1) == 0) return 0;
      x = static_cast<const _Float16 *>(x) + (size_t)(batch - 1) * g.d_in;
      y = static_cast<_Float16 *>(y) + (size_t)(batch - 1) * g.d_out;
      batch = 1;
    }
  }
  GemvPacked a;
  a.weak_sets = tasks.weak_sets; a.task_id = tasks.task_id; a.n_sets = tasks.n_sets;
  a.codes = static_cast<const u32x4 *>(dev.codes);
  a.sz = static_cast<const u32 *>(dev.sz);
  a.weak_w = static_cast<const u32x4 *>(dev.weak_w);
  a.weak_idx = static_cast<const int *>(dev.weak_idx);
  a.x = static_cast<const _Float16 *>(x);
  a.y = static_cast<_Float16 *>(y);
  a.d_in = g.d_in; a.d_out = g.d_out; a.nblk = g.nblk; a.nslab = g.nslab; a.n_rt = g.n_rt;
  a.n_groups = g.n_groups;
  a.blocks_per_group = g.group_size ? g.group_size / kBlockCols : 0;
  a.k = g.k;
  if (g.cw > 0xff || g.r > 0xff || s.rtw > 0xffff || s.rsplit > 0xffff) return (int)hipErrorInvalidValue;
  a.cw_r = (u32)g.cw | ((u32)g.r << 8) | ((u32)s.waves << 16);
  a.rtw_rsplit = (u32)s.rtw | ((u32)s.rsplit << 16);
  a.xpitch = s.xpitch;
  const int nthr = s.waves * 64;
  const bool compact = g.layout == OWQ_LAYOUT_COMPACT && g.kp > 0;
  if (compact) a.weak_idx = static_cast<const int *>(dev.wmeta);
  // units a thread stages: the stored blocks, or (storage-favoured) the wider input row
  const int units = compact && (g.d_in + 7) / 8 > g.nblk * 16 ? (g.d_in + 7) / 8 : g.nblk * 16;
  const int xper = (units + nthr - 1) / nthr;
  a.cw_magic = s.cw_magic; a.nslab_magic = s.nslab_magic; a.rsplit_magic = s.rsplit_magic;
  a.bpg_magic = s.bpg_magic;
  // 16-byte staging from registers needs aligned rows
  const bool aligned = (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (g.d_in % 8 == 0);
  const int xn = !aligned ? 0 : (xper <= 4 ? 4 : 8);
  const dim3 grid((unsigned)s.nwg, (unsigned)batch, 1), block((unsigned)nthr, 1, 1);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // a wave owns whole rows when one tile row spans the row and every weak chunk rides with a block
  // (several slabs of 64 blocks: the waves still add their tile rows themselves, 128)
  const int direct = (compact || g.kp / 8 > g.nblk) ? 0
                     : (g.nslab == 1 && (g.cw == 16 || g.cw == 32 || g.cw == 64)) ? g.cw
                     : (g.nslab > 1 && g.cw == 64) ? 128 : 0;
  kernel_fn fn = pick(g.bits, s.depth, g.kp > 0, xn, compact, direct);
  hipLaunchKernelGGL(fn, grid, block, s.lds_bytes, st, a);
  return (int)hipGetLastError();
}

}  // namespace owq
