// The single-token layout for two tokens at a time (gfx950).
//
//     y[n,i] = sum_{j not weak} s_ig (q_ij - z_ig) x[n,j]  +  sum_t Ww_it x[n, idx_t]
// (paper: storage paragraph of "Outlier-Aware Weight Quantization", section "Acceleration on Real
// Device").  The single-token kernel runs one wave per SIMD and is bound by the weight stream and
// its own start, so most of the register file idles.  Here a lane keeps the 128 activations of
// its block for NTOK = 2 tokens (64 registers each), unpacks every pair of codes once and multiplies
// it with both: a pair of tokens reads the layer once instead of twice (LLaMA-13B-like layers: 11.7
// instead of 17.8 us per call at batch 2).  Four tokens were built and measured too: 256 registers
// of activations leave the vector instructions nothing but the accumulation registers to work in,
// which they cannot address, and the copies made four tokens as slow as two passes of two.  Same packed bytes, same tiles, same launch shape as owq_gemv_kernel; per token the
// arithmetic and the order of additions are those of the single-token kernel's variant with partial
// sums through LDS (fixed order, no atomics: results are reproducible).
//
// Conditions (the launcher falls back to one launch row per token otherwise): rows of x 16-byte
// aligned, d_in a multiple of 8 with at most 8 units of 8 columns per thread and token, at most
// four waves per workgroup, no weak chunk beyond one per block, one task, not the
// storage-favoured layout, LDS room for NTOK staged rows.
#include <hip/hip_runtime.h>

#include "owq_gemv_device.h"

namespace owq {

// the 16 pairs of a quad of 32 3-bit codes (three dwords), each against NTOK tokens
template <int NTOK>
__device__ __forceinline__ void mac_quad3_n(u32 d0, u32 d1, u32 d2, const u32 (*xr)[64], int u, const Magic &M,
                                            float (*acc)[4]) {
  const u32 w1 = __builtin_amdgcn_perm(d1, d0, 0x06030401u);
  const u32 w3 = __builtin_amdgcn_perm(d2, d1, 0x06030401u);
  const u32 w5 = d2 >> 6;
  const u32 f[16] = {andor(d0, field(3, 0), M.m[0]), andor(d0, field(3, 3), M.m[3]), andor(d0, field(3, 6), M.m[6]),
                     andor(w1, field(3, 1), M.m[1]), andor(w1, field(3, 4), M.m[4]), andor(w1, field(3, 7), M.m[7]),
                     andor(d1, field(3, 2), M.m[2]), andor(d1, field(3, 5), M.m[5]), andor(w3, field(3, 0), M.m[0]),
                     andor(w3, field(3, 3), M.m[3]), andor(w3, field(3, 6), M.m[6]), andor(d2, field(3, 1), M.m[1]),
                     andor(d2, field(3, 4), M.m[4]), andor(d2, field(3, 7), M.m[7]), andor(w5, field(3, 4), M.m[4]),
                     andor(w5, field(3, 7), M.m[7])};
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int t = 0; t < NTOK; ++t) acc[t][i & 3] = dot2(f[i], xr[t][16 * u + i], acc[t][i & 3]);
}

// the four pairs of a dword of eight 4-bit codes, each against NTOK tokens
template <int NTOK>
__device__ __forceinline__ void mac_dword4_n(u32 d, const u32 (*xr)[64], int v, const Magic &M, float (*acc)[4]) {
  const u32 w = d >> 6;
  const u32 f[4] = {andor(d, field(4, 0), M.m[0]), andor(d, field(4, 4), M.m[4]), andor(w, field(4, 2), M.m[2]),
                    andor(w, field(4, 6), M.m[6])};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int t = 0; t < NTOK; ++t) acc[t][i] = dot2(f[i], xr[t][4 * v + i], acc[t][i]);
}

// One tile of one lane against NTOK tokens: p[t] = s (acc_t - Bc_t - z X_t) + weak chunk, as tile_partial does
// for one.
template <int BITS, bool HAS_WEAK, int NTOK>
__device__ __forceinline__ void tile_partial_n(const u32x4 *cb, u32 szw, const u32x4 &wkv, const u32x4 *xwr,
                                               const u32 (*xr)[64], const Magic &M, const float *X, const float *Bc,
                                               float *p) {
  float acc[NTOK][4];
#pragma unroll
  for (int t = 0; t < NTOK; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[t][i] = 0.f;
  if (BITS == 3) {
    u32 w[12];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      w[4 * c] = cb[c].x; w[4 * c + 1] = cb[c].y; w[4 * c + 2] = cb[c].z; w[4 * c + 3] = cb[c].w;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) mac_quad3_n<NTOK>(w[3 * u], w[3 * u + 1], w[3 * u + 2], xr, u, M, acc);
  } else {
    u32 w[16];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      w[4 * c] = cb[c].x; w[4 * c + 1] = cb[c].y; w[4 * c + 2] = cb[c].z; w[4 * c + 3] = cb[c].w;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) mac_dword4_n<NTOK>(w[v], xr, v, M, acc);
  }
  const float sc = half_lo(szw), zp = half_hi(szw);
#pragma unroll
  for (int t = 0; t < NTOK; ++t) {
    float q = ((acc[t][0] + acc[t][1]) + (acc[t][2] + acc[t][3])) - Bc[t];
    q = __builtin_fmaf(-zp, X[t], q);
    q *= sc;
    if (HAS_WEAK) {
      q = dot2(wkv.x, xwr[t].x, q);
      q = dot2(wkv.y, xwr[t].y, q);
      q = dot2(wkv.z, xwr[t].z, q);
      q = dot2(wkv.w, xwr[t].w, q);
    }
    p[t] = q;
  }
}

// grid (workgroups as in the single-token launch, groups of NTOK tokens).  LDS, in 16-byte units: per token
// [16][xpitch] staged activations then the activations at the weak columns; then the partial sums
// [NTOK][rows of the workgroup][ppitch] floats, the scale words and the weak weights of the workgroup's rows.
template <int BITS, int DEPTH, bool HAS_WEAK, int XN, int NTOK>
__global__ __launch_bounds__(256) void owq_gemv_multi_kernel(const GemvPacked packed, int batch) {
  const GemvArgs a = packed.unpack();
  constexpr int CH = BITS == 3 ? 3 : 4;
  extern __shared__ uint4 smem[];
  const int xw_units = (a.kp * 2 + 15) >> 4;
  const int tok_units = 16 * a.xpitch + xw_units;                 // LDS units of one token
  const int part_rows = a.rtw * a.r;
  float *part = reinterpret_cast<float *>(smem + NTOK * tok_units);     // [NTOK][part_rows][ppitch]
  const int part_tok = part_rows * a.ppitch;
  uint4 *lsz_u = smem + NTOK * tok_units + ((NTOK * part_tok + 3) >> 2);
  const u32 *lsz = reinterpret_cast<const u32 *>(lsz_u);
  uint4 *lwk_u = lsz_u + (((part_rows * a.n_groups + 3) >> 2) + 1);

  const int tid = threadIdx.x, nthr = a.nthr;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
  const int n0 = blockIdx.y * NTOK;
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
  const char *wk_b = reinterpret_cast<const char *>(a.weak_w);

  // ---- (1) loads of the set-up: activations of the NTOK tokens, weak indices, scales and weak weights of
  // the workgroup's rows; tokens past the batch re-read its last one and are dropped at the end ----------
  uint4 xv[NTOK][XN];
#pragma unroll
  for (int t = 0; t < NTOK; ++t) {
    const _Float16 *xn = a.x + (size_t)min(n0 + t, batch - 1) * a.d_in;
#pragma unroll
    for (int j = 0; j < XN; ++j) {
      const int i = tid + j * nthr;
      const int ic = (i * 8 < a.d_in) ? i : 0;
      xv[t][j] = *reinterpret_cast<const uint4 *>(xn + ic * 8);
    }
  }
  int idx0 = -1;
  if (HAS_WEAK) idx0 = a.weak_idx[tid < a.kp ? tid : 0];
  const int rows_wg = (rt_end - rt0) * a.r;
  const u32 sz0 = (u32)(rt0 * a.r * a.n_groups) * 4u, sz_al = sz0 & ~15u;
  const int sz_units = rows_wg > 0 ? (int)((sz0 - sz_al + (u32)(rows_wg * a.n_groups) * 4u + 15u) >> 4) : 0;
  const int wk_units = HAS_WEAK ? rows_wg * a.kchunks : 0;
  const u32 wk0 = (u32)(rt0 * a.r * a.kchunks) * 16u;
  constexpr int SU = 2;
  u32x4 szv[SU], wkv[SU];
#pragma unroll
  for (int j = 0; j < SU; ++j) {
    const int i = tid + j * nthr;
    szv[j] = *reinterpret_cast<const u32x4 *>(sz_b + (sz_al + (u32)(i < sz_units ? i : 0) * 16u));
    if (HAS_WEAK) wkv[j] = *reinterpret_cast<const u32x4 *>(wk_b + (wk0 + (u32)(i < wk_units ? i : 0) * 16u));
  }

  // ---- (2) per-item state and the tile pipeline (as in the single-token kernel) -------------------------
  u32x4 buf[DEPTH][CH];
  u32 szb[DEPTH];
  u32x4 wkb[DEPTH];
  int item = wave;
  int blk = 0, niter = 0, niter_r = 0;
  bool wk = false;
  u32 off_c = 0, off_s = 0, off_w = 0;
  u32 str_c = 0, str_s = 0, str_w = 0;
  int fetched = 0, sided = 0;
  int pidx = 0, pstr = 0;
  auto set_item = [&](int it_) {
    const int q = (int)(((u32)it_ * a.nslab_magic) >> 16), s = it_ - q * a.nslab;
    blk = s * a.cw + bloc;
    const int grp = a.blocks_per_group ? (int)(((u32)blk * a.bpg_magic) >> 16) : 0;
    const int span = rt_end - rt0 - q;
    niter = span > 0 ? (int)(((u32)(span + a.rsplit - 1) * a.rsplit_magic) >> 16) : 0;
    niter_r = (niter + DEPTH - 1) / DEPTH * DEPTH;
    wk = HAS_WEAK && active && blk < a.kchunks;
    off_c = (u32)((rt0 + q) * a.nslab + s) * tile_bytes + (u32)al * 16u;
    str_c = (u32)(a.rsplit * a.nslab) * tile_bytes;
    const int rowl = q * a.r + rloc;
    off_s = ((sz0 - sz_al) >> 2) + (u32)(rowl * a.n_groups + grp);
    str_s = (u32)(a.rsplit * a.r * a.n_groups);
    off_w = wk ? (u32)(rowl * a.kchunks + blk) : 0u;
    str_w = wk ? (u32)(a.rsplit * a.r * a.kchunks) : 0u;
    fetched = 0; sided = 0;
    pidx = rowl * a.ppitch + blk;
    pstr = a.rsplit * a.r * a.ppitch;
  };
  auto issue = [&](int d) {
    const bool live = fetched < niter;        // uniform
    const u32 oc = live ? off_c : 0u, cs = live ? chunk_bytes : 0u;
#pragma unroll
    for (int c = 0; c < CH; ++c)
      buf[d][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(codes_b + (oc + (u32)c * cs)));
    off_c += str_c;
    ++fetched;
  };
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
  constexpr int EARLY = DEPTH < 2 ? DEPTH : 2;
  set_item(item);
#pragma unroll
  for (int d = 0; d < EARLY; ++d) issue(d);

  // ---- (3) activations -> LDS, transposed to [unit-in-block][block], token after token ----------------------
#pragma unroll
  for (int t = 0; t < NTOK; ++t) {
    uint4 *xs = smem + t * tok_units;
#pragma unroll
    for (int j = 0; j < XN; ++j) {
      const int i = tid + j * nthr;
      if (i < nunits) xs[(i & 15) * a.xpitch + (i >> 4)] = (i * 8 < a.d_in) ? xv[t][j] : make_uint4(0, 0, 0, 0);
    }
  }
#pragma unroll
  for (int d = EARLY; d < DEPTH; ++d) issue(d);
  __syncthreads();
  if (HAS_WEAK) {
    // the activations at the weak columns move to their own array and are cleared in the staged copy
    for (int t0 = tid; t0 < a.kp; t0 += nthr) {
      const int j = t0 == tid ? idx0 : a.weak_idx[t0];
#pragma unroll
      for (int t = 0; t < NTOK; ++t) {
        _Float16 *xs_h = reinterpret_cast<_Float16 *>(smem + t * tok_units);
        _Float16 *xw = reinterpret_cast<_Float16 *>(smem + t * tok_units + 16 * a.xpitch);
        _Float16 v = (_Float16)0;
        if (j >= 0) {
          const int b = j >> 7, u = (j >> 3) & 15, e = j & 7;
          const int pos = (u * a.xpitch + b) * 8 + e;
          v = xs_h[pos];
          xs_h[pos] = (_Float16)0;
        }
        xw[t0] = v;
      }
    }
    __syncthreads();
  }

  // ---- (4) main loop over the wave's (slab, row split) items ---------------------------------------------
  Magic M;
  M.init();
  bool side_staged = false;
  for (;;) {
    u32 xr[NTOK][64];
    u32x4 xwr[NTOK];
    float X[NTOK], Bc[NTOK];
#pragma unroll
    for (int t = 0; t < NTOK; ++t) {
      const uint4 *xs = smem + t * tok_units;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const uint4 v = xs[u * a.xpitch + blk];
        xr[t][4 * u + 0] = v.x; xr[t][4 * u + 1] = v.y; xr[t][4 * u + 2] = v.z; xr[t][4 * u + 3] = v.w;
      }
      xwr[t] = (u32x4){0u, 0u, 0u, 0u};
      if (HAS_WEAK) {
        const uint4 t4 = xs[16 * a.xpitch + (wk ? blk : 0)];
        if (wk) { xwr[t].x = t4.x; xwr[t].y = t4.y; xwr[t].z = t4.z; xwr[t].w = t4.w; }
      }
      block_sums<BITS>(xr[t], X[t], Bc[t]);
    }
    if (!side_staged) {                       // first item only; same for the whole workgroup
#pragma unroll
      for (int j = 0; j < SU; ++j) {
        const int i = tid + j * nthr;
        if (i < sz_units) lsz_u[i] = make_uint4(szv[j].x, szv[j].y, szv[j].z, szv[j].w);
        if (HAS_WEAK && i < wk_units) lwk_u[i] = make_uint4(wkv[j].x, wkv[j].y, wkv[j].z, wkv[j].w);
      }
      for (int i = tid + SU * nthr; i < sz_units; i += nthr)
        lsz_u[i] = *reinterpret_cast<const uint4 *>(sz_b + (sz_al + (u32)i * 16u));
      if (HAS_WEAK)
        for (int i = tid + SU * nthr; i < wk_units; i += nthr)
          lwk_u[i] = *reinterpret_cast<const uint4 *>(wk_b + (wk0 + (u32)i * 16u));
      __syncthreads();
      side_staged = true;
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) side(d);

    int it0 = 0;
    for (; it0 + DEPTH < niter_r; it0 += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        float p[NTOK];
        tile_partial_n<BITS, HAS_WEAK, NTOK>(buf[d], szb[d], wkb[d], xwr, xr, M, X, Bc, p);
        if (active) {
#pragma unroll
          for (int t = 0; t < NTOK; ++t) part[t * part_tok + pidx] = p[t];
        }
        pidx += pstr;
        issue(d);
        side(d);
      }
    }
    if (niter_r > 0) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        float p[NTOK];
        tile_partial_n<BITS, HAS_WEAK, NTOK>(buf[d], szb[d], wkb[d], xwr, xr, M, X, Bc, p);
        if (active && it0 + d < niter) {
#pragma unroll
          for (int t = 0; t < NTOK; ++t) part[t * part_tok + pidx] = p[t];
        }
        pidx += pstr;
      }
    }
    item += nwaves;
    if (item >= a.items) break;
    set_item(item);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(d);
  }
  __syncthreads();

  // ---- (5) add the partials of each row in the single-token kernel's order, token after token ------------
  const int rows_here = (rt_end - rt0) * a.r;
  const int l16 = tid & 15, groups = nthr >> 4;
  for (int t = 0; t < NTOK; ++t) {
    if (n0 + t >= batch) break;               // same for the whole workgroup
    _Float16 *yn = a.y + (size_t)(n0 + t) * a.d_out;
    const float *pt = part + t * part_tok;
    for (int rs0 = tid >> 4; rs0 < rows_here; rs0 += 4 * groups) {
      float sum[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int rs = rs0 + j * groups;
        const float *pr = pt + rs * a.ppitch;
        float acc = 0.f;
        if (rs < rows_here)
          for (int b0 = l16; b0 < a.nblk; b0 += 64) {
            float v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int b = b0 + 16 * q;
              v[q] = pr[b < a.nblk ? b : a.nblk - 1];
              v[q] = b < a.nblk ? v[q] : 0.f;
            }
            acc += (v[0] + v[1]) + (v[2] + v[3]);
          }
        sum[j] = acc;
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
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
typedef void (*multi_fn)(const GemvPacked, int);

template <int BITS, int DEPTH, bool WEAK, int XN>
static multi_fn pick_tok(int) {
  return owq_gemv_multi_kernel<BITS, DEPTH, WEAK, XN, 2>;
}

template <int BITS, int DEPTH, bool WEAK>
static multi_fn pick_xn(int xn, int ntok) {
  return xn == 4 ? pick_tok<BITS, DEPTH, WEAK, 4>(ntok) : pick_tok<BITS, DEPTH, WEAK, 8>(ntok);
}

template <int BITS>
static multi_fn pick_depth(int depth, bool weak, int xn, int ntok) {
  if (depth == 2) return weak ? pick_xn<BITS, 2, true>(xn, ntok) : pick_xn<BITS, 2, false>(xn, ntok);
  if (depth == 3) return weak ? pick_xn<BITS, 3, true>(xn, ntok) : pick_xn<BITS, 3, false>(xn, ntok);
  return weak ? pick_xn<BITS, 4, true>(xn, ntok) : pick_xn<BITS, 4, false>(xn, ntok);
}

static multi_fn pick_multi(int bits, int depth, bool weak, int xn, int ntok) {
  return bits == 3 ? pick_depth<3>(depth, weak, xn, ntok) : pick_depth<4>(depth, weak, xn, ntok);
}

int prepare_multi_kernels(int32_t lds) {
  if (lds <= 64 * 1024) return (int)hipSuccess;
  for (int bits = 3; bits <= 4; ++bits)
    for (int depth = 2; depth <= 4; ++depth)
      for (int w = 0; w < 2; ++w)
        for (int xn = 4; xn <= 8; xn += 4) {
          const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_multi(bits, depth, w != 0, xn, 2)),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
          if (e != hipSuccess) return (int)e;
        }
  return (int)hipSuccess;
}

// LDS bytes of the kernel for ntok tokens at a time
static int64_t multi_lds_bytes(const owq_layer_info_t &g, int32_t rtw, int ntok, int32_t *xpitch) {
  const int32_t pitch = (g.nblk & 1) ? g.nblk : g.nblk + 1;
  *xpitch = pitch;
  const int64_t xs = (int64_t)16 * pitch * 16;
  const int64_t xw = ((int64_t)g.kp * 2 + 15) / 16 * 16;
  const int64_t part = ((int64_t)ntok * rtw * g.r * g.nblk * 4 + 15) / 16 * 16;
  const int64_t sz = (((int64_t)rtw * g.r * g.n_groups + 3) / 4 + 1) * 16;
  const int64_t wk = (int64_t)rtw * g.r * (g.kp / 8) * 16;
  return ntok * (xs + xw) + part + sz + wk;
}

// Returns a hipError_t as int, or -1 when the layer, the shape or x does not fit this kernel (the caller then
// launches one row of workgroups per token).  On success the first batch & ~1 tokens have been enqueued: an
// odd last token is left to the caller.
int launch_gemv_multi(const owq_layer_info_t &g, const LaunchShape &s, const DeviceLayer &dev, int32_t lds_limit,
                      const void *x, void *y, int32_t batch, void *stream) {
  if (batch < 2 || g.layout != OWQ_LAYOUT_GEMV) return -1;
  if (s.waves > 4 || s.depth > 4 || g.kp / 8 > g.nblk) return -1;
  if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || g.d_in % 8 != 0) return -1;
  const int nthr = s.waves * 64;
  const int xper = (g.nblk * 16 + nthr - 1) / nthr;
  if (xper > 8) return -1;
  int32_t xpitch = 0;
  const int ntok = 2;
  const int64_t lds = multi_lds_bytes(g, s.rtw, ntok, &xpitch);
  if (lds > lds_limit) return -1;
  GemvPacked a;
  a.weak_sets = nullptr; a.task_id = nullptr; a.n_sets = 0;
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
  a.xpitch = xpitch;
  a.cw_magic = s.cw_magic; a.nslab_magic = s.nslab_magic; a.rsplit_magic = s.rsplit_magic;
  a.bpg_magic = s.bpg_magic;
  const multi_fn fn = pick_multi(g.bits, s.depth, g.kp > 0, xper <= 4 ? 4 : 8, ntok);
  const dim3 grid((unsigned)s.nwg, (unsigned)(batch / ntok), 1), block((unsigned)nthr, 1, 1);
  hipLaunchKernelGGL(fn, grid, block, (size_t)lds, static_cast<hipStream_t>(stream), a, batch & ~1);
  return (int)hipGetLastError();
}

}  // namespace owq
