// Device-side pieces shared by the single-token kernels (one layer per launch, and a chain of
// dependent layers in one launch): the kernel arguments, the unpack-and-multiply of a lane's
// block of codes, and the per-block sums of the activations.
#pragma once
#include <hip/hip_runtime.h>

#include "owq_device.h"
#include "owq_internal.h"

namespace owq {

// What the kernel works with.  The launcher passes the packed form below: the kernel's
// arguments then fit two 64-byte lines, and every further line a kernel reads at its start
// costs about a quarter of a microsecond per launch here.
struct GemvArgs {
  const u32x4 *codes;
  const u32 *sz;
  const u32x4 *weak_w;
  // storage-favoured layout: not the indices but, per 8 input columns, weak mask | weak columns before << 8
  const int *weak_idx;
  const _Float16 *x;
  _Float16 *y;
  int d_in, d_out, nblk, cw, nact, nslab, n_rt, r, n_groups, blocks_per_group;
  int k, kp, kchunks;
  // several tasks (weak-column tuning): batch row n uses weak_sets[task_id[n]] if that index
  // is in [0, n_sets), else the layer's own weak columns; task_id == nullptr: always its own
  const void *const *weak_sets;
  const int *task_id;
  int n_sets;
  // host-made reciprocals: n / d == (n * magic) >> 16 for the small n that occur (checked on the host)
  u32 cw_magic, nslab_magic, rsplit_magic, bpg_magic;
  int rtw, rsplit, items, xpitch, ppitch;
  int nthr;     // threads per workgroup (from here, not from the launch's hidden arguments: one line less to read)
};

struct GemvPacked {                 // 128 bytes
  const u32x4 *codes;
  const u32 *sz;
  const u32x4 *weak_w;
  const int *weak_idx;
  const _Float16 *x;
  _Float16 *y;
  const void *const *weak_sets;
  const int *task_id;
  int d_in, d_out, nblk, nslab, n_rt, n_groups, blocks_per_group, k, n_sets, xpitch;
  u32 cw_r, rtw_rsplit;             // cw | r << 8 | waves per workgroup << 16; rtw | rsplit << 16
  u32 cw_magic, nslab_magic, rsplit_magic, bpg_magic;

  __device__ __forceinline__ GemvArgs unpack() const {
    GemvArgs a;
    a.codes = codes; a.sz = sz; a.weak_w = weak_w; a.weak_idx = weak_idx; a.x = x; a.y = y;
    a.weak_sets = weak_sets; a.task_id = task_id; a.n_sets = n_sets;
    a.d_in = d_in; a.d_out = d_out; a.nblk = nblk; a.nslab = nslab; a.n_rt = n_rt;
    a.n_groups = n_groups; a.blocks_per_group = blocks_per_group;
    a.cw = (int)(cw_r & 0xffu); a.r = (int)((cw_r >> 8) & 0xffu); a.nact = a.cw * a.r;
    a.nthr = (int)(cw_r >> 16) * 64;
    a.k = k; a.kp = (k + 7) & ~7; a.kchunks = a.kp >> 3;
    a.rtw = (int)(rtw_rsplit & 0xffffu); a.rsplit = (int)(rtw_rsplit >> 16);
    a.items = nslab * a.rsplit; a.xpitch = xpitch; a.ppitch = nblk;
    a.cw_magic = cw_magic; a.nslab_magic = nslab_magic; a.rsplit_magic = rsplit_magic; a.bpg_magic = bpg_magic;
    return a;
  }
};
static_assert(sizeof(GemvPacked) == 128, "two lines of kernel arguments");

// ---- 3-bit: 32 codes in three dwords --------------------------------------
// Even columns form a 48-bit stream in the low halves of the three dwords, odd
// columns one in the high halves; pair t sits at stream bits [3t, 3t+3).
// Six 16-bit windows per half expose every field at an offset <= 7:
//   d0 (bits 0..15), bytes 1..2 (8..23), d1 (16..31), bytes 3..4 (24..39),
//   d2 (32..47), d2 >> 6.
__device__ __forceinline__ void mac_quad3(u32 d0, u32 d1, u32 d2, const u32 *xq, const Magic &M, float *acc) {
  const u32 w1 = __builtin_amdgcn_perm(d1, d0, 0x06030401u);   // (d0.b1, d1.b0, d0.b3, d1.b2)
  const u32 w3 = __builtin_amdgcn_perm(d2, d1, 0x06030401u);
  const u32 w5 = d2 >> 6;
  acc[0] = dot2(andor(d0, field(3, 0), M.m[0]), xq[0], acc[0]);
  acc[1] = dot2(andor(d0, field(3, 3), M.m[3]), xq[1], acc[1]);
  acc[2] = dot2(andor(d0, field(3, 6), M.m[6]), xq[2], acc[2]);
  acc[3] = dot2(andor(w1, field(3, 1), M.m[1]), xq[3], acc[3]);
  acc[0] = dot2(andor(w1, field(3, 4), M.m[4]), xq[4], acc[0]);
  acc[1] = dot2(andor(w1, field(3, 7), M.m[7]), xq[5], acc[1]);
  acc[2] = dot2(andor(d1, field(3, 2), M.m[2]), xq[6], acc[2]);
  acc[3] = dot2(andor(d1, field(3, 5), M.m[5]), xq[7], acc[3]);
  acc[0] = dot2(andor(w3, field(3, 0), M.m[0]), xq[8], acc[0]);
  acc[1] = dot2(andor(w3, field(3, 3), M.m[3]), xq[9], acc[1]);
  acc[2] = dot2(andor(w3, field(3, 6), M.m[6]), xq[10], acc[2]);
  acc[3] = dot2(andor(d2, field(3, 1), M.m[1]), xq[11], acc[3]);
  acc[0] = dot2(andor(d2, field(3, 4), M.m[4]), xq[12], acc[0]);
  acc[1] = dot2(andor(d2, field(3, 7), M.m[7]), xq[13], acc[1]);
  acc[2] = dot2(andor(w5, field(3, 4), M.m[4]), xq[14], acc[2]);
  acc[3] = dot2(andor(w5, field(3, 7), M.m[7]), xq[15], acc[3]);
}

// ---- 4-bit: 8 codes in one dword -------------------------------------------
// Even columns in the low half, odd ones in the high half, pair t at bits [4t, 4t+4).
__device__ __forceinline__ void mac_dword4(u32 d, const u32 *xq, const Magic &M, float *acc) {
  const u32 w = d >> 6;
  acc[0] = dot2(andor(d, field(4, 0), M.m[0]), xq[0], acc[0]);
  acc[1] = dot2(andor(d, field(4, 4), M.m[4]), xq[1], acc[1]);
  acc[2] = dot2(andor(w, field(4, 2), M.m[2]), xq[2], acc[2]);
  acc[3] = dot2(andor(w, field(4, 6), M.m[6]), xq[3], acc[3]);
}

// Per block and lane: X = sum of the block's activations, Bc = sum_j 2^(10-o_j) x_j.
template <int BITS>
__device__ __forceinline__ void block_sums(const u32 *xr, float &X, float &Bc) {
  float c[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (BITS == 3) {
    constexpr int off[16] = {0, 3, 6, 1, 4, 7, 2, 5, 0, 3, 6, 1, 4, 7, 4, 7};
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int t = 0; t < 16; ++t) c[off[t]] = dot2(xr[16 * u + t], kOnes, c[off[t]]);
  } else {
    constexpr int off[4] = {0, 4, 2, 6};
#pragma unroll
    for (int v = 0; v < 16; ++v)
#pragma unroll
      for (int t = 0; t < 4; ++t) c[off[t]] = dot2(xr[4 * v + t], kOnes, c[off[t]]);
  }
  X = ((c[0] + c[1]) + (c[2] + c[3])) + ((c[4] + c[5]) + (c[6] + c[7]));
  float b = 0.f;
#pragma unroll
  for (int o = 0; o < 8; ++o) b = __builtin_fmaf(c[o], (float)(1 << (10 - o)), b);
  Bc = b;
}

// One tile of one lane: 128 codes against the block's activations, then the
// per-(row, block) epilogue  p = s * (acc - Bc - z * X) + weak chunk.
template <int BITS, bool HAS_WEAK>
__device__ __forceinline__ float tile_partial(const u32x4 *cb, u32 szw, const u32x4 &wkv, const u32x4 &xwr,
                                              const u32 *xr, const Magic &M, float X, float Bc) {
  float acc[4] = {0.f, 0.f, 0.f, 0.f};       // four chains of dependent multiply-adds: a lone wave on a SIMD issues them back to back
  if (BITS == 3) {
    u32 w[12];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      w[4 * c] = cb[c].x; w[4 * c + 1] = cb[c].y; w[4 * c + 2] = cb[c].z; w[4 * c + 3] = cb[c].w;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) mac_quad3(w[3 * u], w[3 * u + 1], w[3 * u + 2], &xr[16 * u], M, acc);
  } else {
    u32 w[16];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      w[4 * c] = cb[c].x; w[4 * c + 1] = cb[c].y; w[4 * c + 2] = cb[c].z; w[4 * c + 3] = cb[c].w;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) mac_dword4(w[v], &xr[4 * v], M, acc);
  }
  const float sc = half_lo(szw), zp = half_hi(szw);
  float p = ((acc[0] + acc[1]) + (acc[2] + acc[3])) - Bc;
  p = __builtin_fmaf(-zp, X, p);
  p *= sc;
  if (HAS_WEAK) {
    p = dot2(wkv.x, xwr.x, p);
    p = dot2(wkv.y, xwr.y, p);
    p = dot2(wkv.z, xwr.z, p);
    p = dot2(wkv.w, xwr.w, p);
  }
  return p;
}

}  // namespace owq
