// Backward of the OWQ layer for weak-column tuning (paper, section "PEFT with Weak Column
// Tuning") on gfx950, from the packed tiles of the tile layout:
//
//     dx[n, j]           = sum_i dy[n, i] s[i, g(j)] (q[i, j] - z[i, g(j)])     j not weak
//     dx[n, weak_idx[t]] = sum_i dy[n, i] Ww[i, t]
//     dww[i, t]          = sum_n dy[n, i] x[n, weak_idx[t]]
//
// The dense part contracts over the rows i, while a lane of a packed tile holds eight
// consecutive COLUMNS of one row, which is what the forward product wants as a matrix-core
// operand and the wrong way round here.  The codes are therefore sent through the matrix core
// twice.  First as the A operand against a selection matrix (ones on a diagonal): the result
// is the same 32 x 32 block of codes, but in the accumulator layout, where a lane holds one
// column and sixteen rows; starting the accumulator at minus the unpack constant 2^(10-o) of
// the lane's column leaves the bare integer codes.  Converted to fp16 they are the B operand
// of the real product, whose A operand is dy times the step size, staged in operand order.
// No LDS and no shuffles are needed for the turn.  The zero-point term sum_i a[n, i] z[i] is
// summed on the vector units beside the matrix instructions and taken off at the end.
//
// Four launches per pass of up to 128 tokens (stage dy, product into fp32 partial results per
// range of rows, sum of the partial results into fp16 dx, the weak columns of dx), one more
// for dww over the whole batch.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "owq_internal.h"
#include "owq_tile_device.h"

namespace owq {
namespace {

constexpr int kPassTokens = 128;     // tokens per pass: four accumulator tiles of 32 per wave
constexpr int kBwdWaves = 4;         // one per quarter of a tile's 256 columns
constexpr int kSplitMax = 16;        // most ranges of rows per block pair

// bit offset of the pair of codes that column c (0..15) of K-step t holds, as in the packer
__device__ const signed char kPairOffset3[4][4] = {{0, 3, 6, 1}, {4, 7, 2, 5}, {0, 3, 6, 1}, {4, 7, 4, 7}};
__device__ const signed char kPairOffset4[4] = {0, 4, 2, 6};

struct StageArgs {
  const _Float16 *dy;   // [batch][d_out]
  u32x4 *a_st;          // [n_rt][2][4 token tiles][64 lanes] units of 8 fp16
  int d_out, n_rt, n0, batch;
};

// One thread per unit: token 32 m + lane % 32 of the pass, rows 32 rt + 16 s + 4 h + {0..3} and
// the same + 8 (h = lane / 32): the order in which the turned codes hold their rows.
__global__ __launch_bounds__(256) void owq_bwd_stage(const StageArgs a) {
  const long long u = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long total = (long long)a.n_rt * 2 * 4 * 64;
  if (u >= total) return;
  const int l = (int)(u & 63), m = (int)((u >> 6) & 3), s = (int)((u >> 8) & 1), rt = (int)(u >> 9);
  const int n = a.n0 + 32 * m + (l & 31), h = l >> 5;
  h8_t v;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int i = 32 * rt + 16 * s + 4 * h + (e & 3) + 8 * (e >> 2);
    v[e] = (n < a.batch && i < a.d_out) ? a.dy[(size_t)n * a.d_out + i] : (_Float16)0.f;
  }
  a.a_st[u] = __builtin_bit_cast(u32x4, v);
}

struct ProdArgs {
  const u32 *codes;     // dwords of the packed tiles
  const u32 *sz;        // [G][d_out_pad] step size | zero point << 16
  const u32x4 *a_st;
  float *part;          // [split][128][d_in_pad]
  int n_rt, nbp, chunks, d_out_pad, d_in_pad, blocks_per_group, n_groups, split, rt_per_split;
};

template <int BITS>
__global__ __launch_bounds__(kBwdWaves * 64) void owq_bwd_product(const ProdArgs a) {
  __shared__ float zbuf[kBwdWaves][4][32];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, n32 = lane & 31;
  const int bp = blockIdx.x % a.nbp, sp = blockIdx.x / a.nbp;
  const int rt0 = sp * a.rt_per_split;
  const int rt1 = rt0 + a.rt_per_split < a.n_rt ? rt0 + a.rt_per_split : a.n_rt;
  Magic M;
  M.init();
  // this wave's 64 columns lie in one block (128 columns), hence in one group
  const int blk = 2 * bp + (w >> 1);
  int g = blk / a.blocks_per_group;
  g = g < a.n_groups ? g : a.n_groups - 1;                          // columns past d_in: any group, their codes are 0
  const u32 *sz = a.sz + (size_t)g * a.d_out_pad;
  // selection matrices: K-step t of the forward numbering holds columns 16 t .. 16 t + 15 of the
  // block; two of them side by side make a 32-column tile
  h8_t sel0, sel1;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sel0[e] = (n32 == 8 * h + e) ? (_Float16)1.f : (_Float16)0.f;
    sel1[e] = (n32 == 16 + 8 * h + e) ? (_Float16)1.f : (_Float16)0.f;
  }
  // minus the unpack constant of this lane's column in either column tile of the wave
  float cneg[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int t = 2 * c + (n32 >> 4), i = (n32 & 7) >> 1;            // t & 3 of the K-step, pair in its octet
    const int o = BITS == 3 ? kPairOffset3[t][i] : kPairOffset4[i];
    cneg[c] = -(float)(1 << (10 - o));
  }
  f16_t acc[4][2];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][c][r] = 0.f;
  float zacc[4] = {0.f, 0.f, 0.f, 0.f};
  constexpr int kDw = BITS == 3 ? 3 : 4;                              // dwords of the lane that hold this wave's columns
  for (int rt = rt0; rt < rt1; ++rt) {
    // codes of K-steps 4 w .. 4 w + 3 of the lane: dwords kDw w .. kDw w + kDw - 1 of its 12 or 16
    const size_t tile = (size_t)rt * a.nbp + bp;
    u32 cw[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int v = 0; v < kDw; ++v) {
      const int dwi = kDw * w + v;
      cw[v] = a.codes[((tile * a.chunks + (dwi >> 2)) * 64 + lane) * 4 + (dwi & 3)];
    }
    // turned codes of the two column tiles: B operands for both halves of the 32 rows
    h8_t wb[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      f16_t t;
#pragma unroll
      for (int r = 0; r < 16; ++r) t[r] = cneg[c];
      if (c == 0) {
        t = mma(a_operand<BITS, 0>(cw, M), sel0, t);
        t = mma(a_operand<BITS, 1>(cw, M), sel1, t);
      } else {
        t = mma(a_operand<BITS, 2>(cw, M), sel0, t);
        t = mma(a_operand<BITS, 3>(cw, M), sel1, t);
      }
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) wb[c][s][e] = (_Float16)t[8 * s + e];
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      // step sizes and zero points of the lane's eight rows of this half
      const int i0 = 32 * rt + 16 * s + 4 * h;
      const u32x4 q0 = *reinterpret_cast<const u32x4 *>(sz + i0), q1 = *reinterpret_cast<const u32x4 *>(sz + i0 + 8);
      const u32 d[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
      u32 sp2[4], zp2[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        sp2[p] = __builtin_amdgcn_perm(d[2 * p + 1], d[2 * p], 0x05040100u);   // (lo of even, lo of odd)
        zp2[p] = __builtin_amdgcn_perm(d[2 * p + 1], d[2 * p], 0x07060302u);   // (hi of even, hi of odd)
      }
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const u32x4 raw = a.a_st[(((size_t)rt * 2 + s) * 4 + m) * 64 + lane];
        const u32 r[4] = {raw.x, raw.y, raw.z, raw.w};
        u32 ap[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const h2_t prod = __builtin_bit_cast(h2_t, r[p]) * __builtin_bit_cast(h2_t, sp2[p]);   // one rounding to fp16
          ap[p] = __builtin_bit_cast(u32, prod);
          zacc[m] = dot2(ap[p], zp2[p], zacc[m]);
        }
        const u32x4 av = {ap[0], ap[1], ap[2], ap[3]};
        const h8_t aop = __builtin_bit_cast(h8_t, av);
        acc[m][0] = mma(aop, wb[0][s], acc[m][0]);
        acc[m][1] = mma(aop, wb[1][s], acc[m][1]);
      }
    }
  }
  // zero-point term of every token: both halves of the rows, then from the operand layout
  // (token = lane % 32) to the accumulator layout (tokens along the registers)
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const float z = zacc[m] + __shfl_xor(zacc[m], 32);
    if (h == 0) zbuf[w][m][n32] = z;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  float *part = a.part + (size_t)sp * kPassTokens * a.d_in_pad;
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int j = 256 * bp + 64 * w + 32 * c + n32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int nl = 8 * (r >> 2) + 4 * h + (r & 3);              // token of the tile that register r holds
        part[(size_t)(32 * m + nl) * a.d_in_pad + j] = acc[m][c][r] - zbuf[w][m][nl];
      }
    }
}

struct SumArgs {
  const float *part;    // [split][128][d_in_pad]
  const uint8_t *wmask; // bit j = column j is weak
  _Float16 *dx;         // [batch][d_in]
  int d_in, d_in_pad, split, n0, ntok;
};

// dx of the columns that are not weak: the partial results added in a fixed order.
__global__ __launch_bounds__(256) void owq_bwd_sum(const SumArgs a) {
  const int j = blockIdx.x * 256 + threadIdx.x, nl = blockIdx.y;
  if (j >= a.d_in || nl >= a.ntok) return;
  if ((a.wmask[j >> 3] >> (j & 7)) & 1) return;
  float v = 0.f;
  for (int s = 0; s < a.split; ++s) v += a.part[((size_t)s * kPassTokens + nl) * a.d_in_pad + j];
  a.dx[(size_t)(a.n0 + nl) * a.d_in + j] = (_Float16)v;
}

struct WeakArgs {
  const _Float16 *dy;        // [batch][d_out]
  const _Float16 *weak_w;    // [d_out_pad][kp]
  const int *weak_idx;       // [kp], -1 = padding
  _Float16 *dx;
  int d_out, d_in, kp, n0, ntok;
};

// dx at the weak columns: 8 tokens x 8 weak columns per workgroup, rows dealt to the threads.
__global__ __launch_bounds__(256) void owq_bwd_weak(const WeakArgs a) {
  __shared__ float red[4][64];
  const int t0 = blockIdx.x * 8, nb = blockIdx.y * 8;
  float acc[8][8];
#pragma unroll
  for (int n = 0; n < 8; ++n)
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[n][t] = 0.f;
  for (int i = threadIdx.x; i < a.d_out; i += 256) {
    const h8_t wv = *reinterpret_cast<const h8_t *>(a.weak_w + (size_t)i * a.kp + t0);
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int nl = nb + n < a.ntok ? nb + n : a.ntok - 1;         // past the end: the last token again, dropped below
      const float d = (float)a.dy[(size_t)(a.n0 + nl) * a.d_out + i];
#pragma unroll
      for (int t = 0; t < 8; ++t) acc[n][t] = __builtin_fmaf(d, (float)wv[t], acc[n][t]);
    }
  }
  // sum over the 256 threads: inside the waves, then the four waves through LDS
  const int lane = threadIdx.x & 63, wv_id = threadIdx.x >> 6;
#pragma unroll
  for (int n = 0; n < 8; ++n)
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float v = acc[n][t];
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) v += __shfl_xor(v, d);
      if (lane == 0) red[wv_id][n * 8 + t] = v;
    }
  __syncthreads();
  if (threadIdx.x < 64) {
    const int n = threadIdx.x >> 3, t = threadIdx.x & 7;
    const float v = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
    const int col = a.weak_idx[t0 + t];
    if (nb + n < a.ntok && (unsigned)col < (unsigned)a.d_in) a.dx[(size_t)(a.n0 + nb + n) * a.d_in + col] = (_Float16)v;
  }
}

struct DwwArgs {
  const _Float16 *dy, *x;
  const int *weak_idx;
  float *dww;                // [d_out][k]
  int d_out, d_in, k, batch;
};

// dww: one thread per row, 8 weak columns per workgroup, the whole batch in order.
__global__ __launch_bounds__(256) void owq_bwd_dww(const DwwArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x, t0 = blockIdx.y * 8;
  int col[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int c = t0 + t < a.k ? a.weak_idx[t0 + t] : 0;
    col[t] = (unsigned)c < (unsigned)a.d_in ? c : 0;
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int ii = i < a.d_out ? i : a.d_out - 1;
  for (int n = 0; n < a.batch; ++n) {
    const float d = (float)a.dy[(size_t)n * a.d_out + ii];
    const _Float16 *xr = a.x + (size_t)n * a.d_in;
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = __builtin_fmaf(d, (float)xr[col[t]], acc[t]);
  }
  if (i < a.d_out)
#pragma unroll
    for (int t = 0; t < 8; ++t)
      if (t0 + t < a.k) a.dww[(size_t)i * a.k + t0 + t] = acc[t];
}

struct BwdPlan {
  int split, rt_per_split;
  size_t a_st_bytes, part_bytes, total;
};

BwdPlan plan(const owq_layer_info_t &g) {
  BwdPlan p;
  // enough workgroups for the chip, few enough ranges that the partial results stay small
  int split = (512 + g.nbp - 1) / g.nbp;
  if (split > kSplitMax) split = kSplitMax;
  if (split > g.n_rt) split = g.n_rt;
  if (split < 1) split = 1;
  p.rt_per_split = (g.n_rt + split - 1) / split;
  p.split = (g.n_rt + p.rt_per_split - 1) / p.rt_per_split;
  p.a_st_bytes = (size_t)g.n_rt * 2 * 4 * 64 * 16;
  p.part_bytes = (size_t)p.split * kPassTokens * ((size_t)g.nbp * 256) * 4;
  p.total = p.a_st_bytes + p.part_bytes;
  return p;
}

bool live(owq_handle_t h) { return h && h->magic == kMagic; }

}  // namespace
}  // namespace owq

extern "C" owq_status_t owq_backward_workspace_bytes(owq_handle_t h, int32_t batch, size_t *bytes) {
  using namespace owq;
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (h->info.layout != OWQ_LAYOUT_TILE) return OWQ_ERR_LAYOUT;
  if (!bytes) return OWQ_ERR_NULL;
  if (batch < 0 || batch > OWQ_MAX_BATCH) return OWQ_ERR_BATCH;
  *bytes = plan(h->info).total;
  return OWQ_OK;
}

extern "C" owq_status_t owq_linear_backward(owq_handle_t h, const void *dy, const void *x, void *dx, float *dww,
                                            int32_t batch, void *workspace, size_t workspace_bytes, void *stream) {
  using namespace owq;
  if (!live(h)) return OWQ_ERR_HANDLE;
  const owq_layer_info_t &g = h->info;
  if (g.layout != OWQ_LAYOUT_TILE) return OWQ_ERR_LAYOUT;
  if (batch < 0 || batch > OWQ_MAX_BATCH) return OWQ_ERR_BATCH;
  if (batch == 0 || (!dx && !dww)) return OWQ_OK;
  if (!dy || (dww && g.k > 0 && !x) || (dx && !workspace)) return OWQ_ERR_NULL;
  const BwdPlan p = plan(g);
  if (dx && workspace_bytes < p.total) return OWQ_ERR_BUFFER;
  if (((uintptr_t)dy | (uintptr_t)x | (uintptr_t)dx | (uintptr_t)dww) & 15u) return OWQ_ERR_BUFFER;
  if (dx && ((uintptr_t)workspace & 255u)) return OWQ_ERR_BUFFER;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint8_t *blob = static_cast<const uint8_t *>(h->dev_buf);
  hipError_t err = hipSuccess;
  if (dx) {
    u32x4 *a_st = static_cast<u32x4 *>(workspace);
    float *part = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + p.a_st_bytes);
    for (int n0 = 0; n0 < batch && err == hipSuccess; n0 += kPassTokens) {
      const int ntok = batch - n0 < kPassTokens ? batch - n0 : kPassTokens;
      StageArgs sa = {static_cast<const _Float16 *>(dy), a_st, g.d_out, g.n_rt, n0, batch};
      const long long units = (long long)g.n_rt * 512;
      hipLaunchKernelGGL(owq_bwd_stage, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st, sa);
      ProdArgs pa;
      pa.codes = reinterpret_cast<const u32 *>(blob + g.off_codes);
      pa.sz = reinterpret_cast<const u32 *>(blob + g.off_sz);
      pa.a_st = a_st;
      pa.part = part;
      pa.n_rt = g.n_rt;
      pa.nbp = g.nbp;
      pa.chunks = g.chunks;
      pa.d_out_pad = g.d_out_pad;
      pa.d_in_pad = g.nbp * 256;
      pa.blocks_per_group = g.group_size == 0 ? 0x40000000 : g.group_size / kBlockCols;
      pa.n_groups = g.n_groups;
      pa.split = p.split;
      pa.rt_per_split = p.rt_per_split;
      const dim3 grid((unsigned)(g.nbp * p.split));
      if (g.bits == 3) hipLaunchKernelGGL(owq_bwd_product<3>, grid, dim3(kBwdWaves * 64), 0, st, pa);
      else hipLaunchKernelGGL(owq_bwd_product<4>, grid, dim3(kBwdWaves * 64), 0, st, pa);
      SumArgs su = {part, blob + g.off_wmask, static_cast<_Float16 *>(dx), g.d_in, g.nbp * 256, p.split, n0, ntok};
      hipLaunchKernelGGL(owq_bwd_sum, dim3((unsigned)((g.d_in + 255) / 256), (unsigned)ntok), dim3(256), 0, st, su);
      if (g.k > 0) {
        WeakArgs wa = {static_cast<const _Float16 *>(dy), reinterpret_cast<const _Float16 *>(blob + g.off_weak_w),
                       reinterpret_cast<const int *>(blob + g.off_weak_idx), static_cast<_Float16 *>(dx),
                       g.d_out, g.d_in, g.kp, n0, ntok};
        hipLaunchKernelGGL(owq_bwd_weak, dim3((unsigned)(g.kp / 8), (unsigned)((ntok + 7) / 8)), dim3(256), 0, st, wa);
      }
      err = hipGetLastError();
    }
  }
  if (dww && g.k > 0 && err == hipSuccess) {
    DwwArgs da = {static_cast<const _Float16 *>(dy), static_cast<const _Float16 *>(x),
                  reinterpret_cast<const int *>(blob + g.off_weak_idx), dww, g.d_out, g.d_in, g.k, batch};
    hipLaunchKernelGGL(owq_bwd_dww, dim3((unsigned)((g.d_out + 255) / 256), (unsigned)((g.k + 7) / 8)), dim3(256), 0, st, da);
    err = hipGetLastError();
  }
  if (err != hipSuccess) {
    h->info.last_hip_error = (int32_t)err;
    return OWQ_ERR_HIP;
  }
  return OWQ_OK;
}
