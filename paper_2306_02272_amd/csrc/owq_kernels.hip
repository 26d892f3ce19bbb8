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

#include "owq_internal.h"

namespace owq {

typedef unsigned int u32;
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));   // native vector: 16-byte loads

struct GemvArgs {
  const u32x4 *codes;
  const u32 *sz;
  const u32x4 *weak_w;
  const int *weak_idx;
  const _Float16 *x;
  _Float16 *y;
  int d_in, d_out, nblk, cw, nact, nslab, n_rt, r, n_groups, blocks_per_group;
  int kp, kchunks;
  int rtw, rsplit, items, xpitch, ppitch;
};

__device__ __forceinline__ float dot2(u32 a, u32 b, float c) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2_t, a), __builtin_bit_cast(h2_t, b), c, false);
}

// fp16 bit pattern of 2^(10-o) in both halves
__device__ __forceinline__ constexpr u32 magic(int o) {
  return (u32)((25 - o) << 10) * 0x00010001u;
}
__device__ __forceinline__ constexpr u32 field(int width, int o) {
  return (u32)(((1 << width) - 1) << o) * 0x00010001u;
}
__device__ __forceinline__ u32 andor(u32 w, u32 m, u32 c) { return (w & m) | c; }

// The eight constants 2^(10-o) live in vector registers the compiler cannot see
// through: (w & mask) | magic then has one scalar operand only and maps onto a
// single v_and_or_b32 (a VALU instruction here reads at most one scalar source).
struct Magic {
  u32 m[8];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int o = 0; o < 8; ++o) asm("v_mov_b32 %0, %1" : "=v"(m[o]) : "s"(magic(o)));
  }
};

constexpr u32 kOnes = 0x3C003C00u;   // (1.0h, 1.0h)

// ---- 3-bit: 32 codes in three dwords --------------------------------------
// Even columns form a 48-bit stream in the low halves of the three dwords, odd
// columns one in the high halves; pair t sits at stream bits [3t, 3t+3).
// Six 16-bit windows per half expose every field at an offset <= 7:
//   d0 (bits 0..15), bytes 1..2 (8..23), d1 (16..31), bytes 3..4 (24..39),
//   d2 (32..47), d2 >> 6.
__device__ __forceinline__ void mac_quad3(u32 d0, u32 d1, u32 d2, const u32 *xq, const Magic &M, float &a0, float &a1) {
  const u32 w1 = __builtin_amdgcn_perm(d1, d0, 0x06030401u);   // (d0.b1, d1.b0, d0.b3, d1.b2)
  const u32 w3 = __builtin_amdgcn_perm(d2, d1, 0x06030401u);
  const u32 w5 = d2 >> 6;
  a0 = dot2(andor(d0, field(3, 0), M.m[0]), xq[0], a0);
  a1 = dot2(andor(d0, field(3, 3), M.m[3]), xq[1], a1);
  a0 = dot2(andor(d0, field(3, 6), M.m[6]), xq[2], a0);
  a1 = dot2(andor(w1, field(3, 1), M.m[1]), xq[3], a1);
  a0 = dot2(andor(w1, field(3, 4), M.m[4]), xq[4], a0);
  a1 = dot2(andor(w1, field(3, 7), M.m[7]), xq[5], a1);
  a0 = dot2(andor(d1, field(3, 2), M.m[2]), xq[6], a0);
  a1 = dot2(andor(d1, field(3, 5), M.m[5]), xq[7], a1);
  a0 = dot2(andor(w3, field(3, 0), M.m[0]), xq[8], a0);
  a1 = dot2(andor(w3, field(3, 3), M.m[3]), xq[9], a1);
  a0 = dot2(andor(w3, field(3, 6), M.m[6]), xq[10], a0);
  a1 = dot2(andor(d2, field(3, 1), M.m[1]), xq[11], a1);
  a0 = dot2(andor(d2, field(3, 4), M.m[4]), xq[12], a0);
  a1 = dot2(andor(d2, field(3, 7), M.m[7]), xq[13], a1);
  a0 = dot2(andor(w5, field(3, 4), M.m[4]), xq[14], a0);
  a1 = dot2(andor(w5, field(3, 7), M.m[7]), xq[15], a1);
}

// ---- 4-bit: 8 codes in one dword -------------------------------------------
// Even columns in the low half, odd ones in the high half, pair t at bits [4t, 4t+4).
__device__ __forceinline__ void mac_dword4(u32 d, const u32 *xq, const Magic &M, float &a0, float &a1) {
  const u32 w = d >> 6;
  a0 = dot2(andor(d, field(4, 0), M.m[0]), xq[0], a0);
  a1 = dot2(andor(d, field(4, 4), M.m[4]), xq[1], a1);
  a0 = dot2(andor(w, field(4, 2), M.m[2]), xq[2], a0);
  a1 = dot2(andor(w, field(4, 6), M.m[6]), xq[3], a1);
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

__device__ __forceinline__ float half_lo(u32 w) {
  return (float)__builtin_bit_cast(h2_t, w)[0];
}
__device__ __forceinline__ float half_hi(u32 w) {
  return (float)__builtin_bit_cast(h2_t, w)[1];
}

template <int BITS, int DEPTH>
__global__ __launch_bounds__(512) void owq_gemv_kernel(const GemvArgs a) {
  constexpr int CH = BITS == 3 ? 3 : 4;
  constexpr int XCH = 12;   // 16-byte activation units a thread stages from registers
  extern __shared__ uint4 smem[];
  uint4 *xs = smem;                                             // [16][xpitch] units of 8 fp16
  _Float16 *xs_h = reinterpret_cast<_Float16 *>(smem);
  const int xw_units = (a.kp * 2 + 15) >> 4;
  uint4 *xw_u = smem + 16 * a.xpitch;                           // gathered weak activations
  _Float16 *xw = reinterpret_cast<_Float16 *>(xw_u);
  float *part = reinterpret_cast<float *>(xw_u + xw_units);     // [rows of the workgroup][ppitch]

  const int tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
  const _Float16 *xn = a.x + (size_t)blockIdx.y * a.d_in;
  _Float16 *yn = a.y + (size_t)blockIdx.y * a.d_out;
  const int nunits = a.nblk * 16;
  const bool fast_x = ((reinterpret_cast<uintptr_t>(xn) & 15) == 0) && ((a.d_in & 7) == 0);

  const bool active = lane < a.nact;
  const int al = active ? lane : 0;
  const int rloc = al / a.cw, bloc = al - rloc * a.cw;
  const int rt0 = blockIdx.x * a.rtw;
  const int rt_end = min(a.n_rt, rt0 + a.rtw);
  const int tile_units = CH * a.nact;

  // ---- activations: global -> registers (first XCH units per thread) --------
  uint4 xv[XCH];
  if (fast_x) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int i = tid + j * nthr;
      xv[j] = make_uint4(0, 0, 0, 0);
      if (i < nunits && i * 8 < a.d_in) xv[j] = *reinterpret_cast<const uint4 *>(xn + i * 8);
    }
  }

  // ---- per-item state and the tile pipeline ---------------------------------
  u32x4 buf[DEPTH][CH];
  u32 szb[DEPTH];
  u32x4 wkb[DEPTH];
  int item = wave;
  int s = 0, q = 0, blk = 0, grp = 0, niter = 0;
  bool wk = false;

  auto set_item = [&](int it_) {
    s = it_ % a.nslab;
    q = it_ / a.nslab;
    blk = s * a.cw + bloc;
    grp = a.blocks_per_group ? blk / a.blocks_per_group : 0;
    const int span = rt_end - rt0 - q;
    niter = span > 0 ? (span + a.rsplit - 1) / a.rsplit : 0;
    wk = active && blk < a.kchunks;
  };
  auto issue = [&](int d, int it) {
    // Tiles past the end read unit 0 (always valid) so that the number of loads
    // in flight never depends on data.
    const bool live = it < niter;
    const int rt = rt0 + q + it * a.rsplit;
    const int base = live ? (rt * a.nslab + s) * tile_units + al : 0;
    const int step = live ? a.nact : 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) buf[d][c] = __builtin_nontemporal_load(a.codes + base + c * step);
    const int row = rt * a.r + rloc;
    szb[d] = a.sz[live ? row * a.n_groups + grp : 0];
    if (a.kchunks) wkb[d] = __builtin_nontemporal_load(a.weak_w + ((live && wk) ? row * a.kchunks + blk : 0));
  };

  if (item < a.items) {
    set_item(item);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(d, d);
  }

  // ---- activations: registers -> LDS, transposed to [unit-in-block][block] ---
  if (fast_x) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int i = tid + j * nthr;
      if (i < nunits) xs[(i & 15) * a.xpitch + (i >> 4)] = xv[j];
    }
    for (int i = tid + XCH * nthr; i < nunits; i += nthr) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (i * 8 < a.d_in) v = *reinterpret_cast<const uint4 *>(xn + i * 8);
      xs[(i & 15) * a.xpitch + (i >> 4)] = v;
    }
  } else {
    for (int i = tid; i < nunits; i += nthr) {
      _Float16 e[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int j = i * 8 + t;
        e[t] = j < a.d_in ? xn[j] : (_Float16)0;
      }
      xs[(i & 15) * a.xpitch + (i >> 4)] = *reinterpret_cast<const uint4 *>(e);
    }
  }
  __syncthreads();
  // Gather the activations of the weak columns, then clear them in the staged
  // copy: the dense path must contribute nothing there.
  for (int t = tid; t < a.kp; t += nthr) {
    const int j = a.weak_idx[t];
    _Float16 v = (_Float16)0;
    if (j >= 0) {
      const int b = j >> 7, u = (j >> 3) & 15, e = j & 7;
      const int pos = (u * a.xpitch + b) * 8 + e;
      v = xs_h[pos];
      xs_h[pos] = (_Float16)0;
    }
    xw[t] = v;
  }
  __syncthreads();

  // ---- main loop over the wave's (slab, row split) items ----------------------
  Magic M;
  M.init();
  for (; item < a.items; item += nwaves) {
    if (item != wave) {
      set_item(item);
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) issue(d, d);
    }
    u32 xr[64];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const uint4 v = xs[u * a.xpitch + blk];
      xr[4 * u + 0] = v.x; xr[4 * u + 1] = v.y; xr[4 * u + 2] = v.z; xr[4 * u + 3] = v.w;
    }
    float X, Bc;
    block_sums<BITS>(xr, X, Bc);
    uint4 xwr = make_uint4(0, 0, 0, 0);
    if (wk) xwr = xw_u[blk];

    for (int it0 = 0; it0 < niter; it0 += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        const int it = it0 + d;
        if (it < niter) {
          float a0 = 0.f, a1 = 0.f;
          if (BITS == 3) {
            u32 w[12];
#pragma unroll
            for (int c = 0; c < 3; ++c) {
              w[4 * c] = buf[d][c].x; w[4 * c + 1] = buf[d][c].y; w[4 * c + 2] = buf[d][c].z; w[4 * c + 3] = buf[d][c].w;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) mac_quad3(w[3 * u], w[3 * u + 1], w[3 * u + 2], &xr[16 * u], M, a0, a1);
          } else {
            u32 w[16];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              w[4 * c] = buf[d][c].x; w[4 * c + 1] = buf[d][c].y; w[4 * c + 2] = buf[d][c].z; w[4 * c + 3] = buf[d][c].w;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) mac_dword4(w[v], &xr[4 * v], M, a0, a1);
          }
          const float sc = half_lo(szb[d]), zp = half_hi(szb[d]);
          float p = (a0 + a1) - Bc;
          p = __builtin_fmaf(-zp, X, p);
          p *= sc;
          if (a.kchunks) {
            p = dot2(wkb[d].x, xwr.x, p);
            p = dot2(wkb[d].y, xwr.y, p);
            p = dot2(wkb[d].z, xwr.z, p);
            p = dot2(wkb[d].w, xwr.w, p);
          }
          const int rt = rt0 + q + it * a.rsplit;
          if (active) part[((rt - rt0) * a.r + rloc) * a.ppitch + blk] = p;
          issue(d, it + DEPTH);
        }
      }
    }
  }
  __syncthreads();

  // ---- add the partials of each row; weak chunks beyond one per block -------
  const int rows_here = (rt_end - rt0) * a.r;
  const int l16 = tid & 15;
  for (int rs = tid >> 4; rs < rows_here; rs += nthr >> 4) {
    const int row = rt0 * a.r + rs;
    float sum = 0.f;
    for (int b = l16; b < a.nblk; b += 16) sum += part[rs * a.ppitch + b];
    for (int c = a.nblk + l16; c < a.kchunks; c += 16) {
      const u32x4 wv = a.weak_w[row * a.kchunks + c];
      const uint4 xv4 = xw_u[c];
      sum = dot2(wv.x, xv4.x, sum);
      sum = dot2(wv.y, xv4.y, sum);
      sum = dot2(wv.z, xv4.z, sum);
      sum = dot2(wv.w, xv4.w, sum);
    }
    sum += __shfl_xor(sum, 1, 16);
    sum += __shfl_xor(sum, 2, 16);
    sum += __shfl_xor(sum, 4, 16);
    sum += __shfl_xor(sum, 8, 16);
    if (l16 == 0 && row < a.d_out) yn[row] = (_Float16)sum;
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

template <int BITS, int DEPTH>
static hipError_t launch_one(const GemvArgs &args, dim3 grid, dim3 block, int lds, hipStream_t st) {
  hipLaunchKernelGGL((owq_gemv_kernel<BITS, DEPTH>), grid, block, lds, st, args);
  return hipGetLastError();
}

template <int BITS, int DEPTH>
static hipError_t raise_lds(int lds) {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&owq_gemv_kernel<BITS, DEPTH>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

int prepare_kernels(int32_t lds) {
  if (lds <= 64 * 1024) return (int)hipSuccess;
  hipError_t e;
  if ((e = raise_lds<3, 1>(lds)) != hipSuccess) return (int)e;
  if ((e = raise_lds<3, 2>(lds)) != hipSuccess) return (int)e;
  if ((e = raise_lds<3, 4>(lds)) != hipSuccess) return (int)e;
  if ((e = raise_lds<4, 1>(lds)) != hipSuccess) return (int)e;
  if ((e = raise_lds<4, 2>(lds)) != hipSuccess) return (int)e;
  if ((e = raise_lds<4, 4>(lds)) != hipSuccess) return (int)e;
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

int launch_gemv(const owq_layer_info_t &g, const LaunchShape &s, const DeviceLayer &dev,
                const void *x, void *y, int32_t batch, void *stream) {
  GemvArgs a;
  a.codes = static_cast<const u32x4 *>(dev.codes);
  a.sz = static_cast<const u32 *>(dev.sz);
  a.weak_w = static_cast<const u32x4 *>(dev.weak_w);
  a.weak_idx = static_cast<const int *>(dev.weak_idx);
  a.x = static_cast<const _Float16 *>(x);
  a.y = static_cast<_Float16 *>(y);
  a.d_in = g.d_in; a.d_out = g.d_out; a.nblk = g.nblk; a.cw = g.cw; a.nact = g.nact;
  a.nslab = g.nslab; a.n_rt = g.n_rt; a.r = g.r; a.n_groups = g.n_groups;
  a.blocks_per_group = g.group_size ? g.group_size / kBlockCols : 0;
  a.kp = g.kp; a.kchunks = g.kp / 8;
  a.rtw = s.rtw; a.rsplit = s.rsplit; a.items = g.nslab * s.rsplit;
  a.xpitch = s.xpitch;
  a.ppitch = g.nblk;
  const dim3 grid((unsigned)s.nwg, (unsigned)batch, 1), block((unsigned)s.waves * 64, 1, 1);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipErrorInvalidValue;
  if (g.bits == 3) {
    if (s.depth == 1) e = launch_one<3, 1>(a, grid, block, s.lds_bytes, st);
    else if (s.depth == 2) e = launch_one<3, 2>(a, grid, block, s.lds_bytes, st);
    else if (s.depth == 4) e = launch_one<3, 4>(a, grid, block, s.lds_bytes, st);
  } else {
    if (s.depth == 1) e = launch_one<4, 1>(a, grid, block, s.lds_bytes, st);
    else if (s.depth == 2) e = launch_one<4, 2>(a, grid, block, s.lds_bytes, st);
    else if (s.depth == 4) e = launch_one<4, 4>(a, grid, block, s.lds_bytes, st);
  }
  return (int)e;
}

}  // namespace owq
