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
// Three launches per group of up to four passes of 128 tokens (staging: dy into operand order,
// on the first group also the weak columns and the activations at the weak columns; product into
// fp32 partial results per range of rows, the weak columns of dx riding along as one more tile of
// columns per workgroup; sum of the partial results into fp16 dx), one more for dww over the whole
// batch (a product with the tokens on the contraction axis).  A layer with more tiles of weak
// columns than block pairs takes a plain kernel for the weak columns of dx instead.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "owq_internal.h"
#include "owq_tile_device.h"

namespace owq {
namespace {

constexpr int kPassTokens = 128;     // tokens per pass: four accumulator tiles of 32 per wave
constexpr int kBwdWaves = 4;         // one per quarter of a tile's 256 columns
constexpr int kSplitMax = 16;        // most ranges of rows per block pair
constexpr int kLaunchPasses = 4;     // passes (of 128 tokens) that one set of launches takes
constexpr size_t kScanBytes = 2048;  // end of the workspace: the magnitude scan's 256 words, then the exponent

// bit offset of the pair of codes that column c (0..15) of K-step t holds, as in the packer
__device__ const signed char kPairOffset3[4][4] = {{0, 3, 6, 1}, {4, 7, 2, 5}, {0, 3, 6, 1}, {4, 7, 4, 7}};
__device__ const signed char kPairOffset4[4] = {0, 4, 2, 6};

// N 2-byte loads whose results get a use of their own after all of them have been issued, so
// that the compiler cannot move a load under the branch of a later select (loads under branches
// are waited for one by one).  Every address must be valid whatever the selects decide.
template <int N>
__device__ __forceinline__ void load_h(const _Float16 *const (&p)[N], _Float16 (&out)[N]) {
  u32 r[N];
#pragma unroll
  for (int e = 0; e < N; ++e) r[e] = __builtin_bit_cast(unsigned short, *p[e]);
#pragma unroll
  for (int e = 0; e < N; ++e) asm volatile("" : "+v"(r[e]));
#pragma unroll
  for (int e = 0; e < N; ++e) out[e] = __builtin_bit_cast(_Float16, (unsigned short)r[e]);
}

constexpr int kMaxBlocks = 256;      // workgroups of the magnitude scan = entries of its result

// Largest magnitude of dy, as fp16 bit patterns without sign (Inf and NaN count as the largest
// finite number): one entry per workgroup, no atomics.  The product forms dy * s in fp16; with
// gradients of 1e-3 and step sizes of 1e-3 that product is a subnormal number and loses most of
// its bits, so dy is first scaled by a power of two (exact) that brings its largest magnitude
// into [512, 1024), and the sums are scaled back at the end (also exact).
__global__ __launch_bounds__(256) void owq_bwd_absmax(const u32x4 *dy, size_t n16, size_t n_halves, const unsigned short *dy_h,
                                                      u32 *out) {
  __shared__ u32 red[4];
  u32 m = 0;
  auto take = [&](u32 w) {
    const u32 lo = w & 0x7fffu, hi = (w >> 16) & 0x7fffu;
    m = max(m, max(lo, hi));
  };
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)kMaxBlocks * 256) {
    const u32x4 v = dy[i];
    take(v.x); take(v.y); take(v.z); take(v.w);
  }
  for (size_t i = n16 * 8 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n_halves; i += (size_t)kMaxBlocks * 256)
    take(dy_h[i]);
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m = max(m, (u32)__shfl_xor((int)m, d));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) out[blockIdx.x] = min(max(max(red[0], red[1]), max(red[2], red[3])), 0x7bffu);
}

// The power of two dy is scaled by: 2^k brings the largest magnitude into [2^9, 2^10).
__device__ __forceinline__ int scale_exponent(u32 max_bits) { return 24 - (int)(max_bits >> 10); }

struct StageArgs {
  const _Float16 *dy;   // [batch][d_out]
  u32x4 *a_st;          // [pass][n_rt][2][4 token tiles][64 lanes] units of 8 fp16
  int d_out, n_rt, n0, batch, passes;
  const u32 *maxima;    // [kMaxBlocks] from owq_bwd_absmax
  int *kword;           // the exponent, for the kernel that scales the sums back
};

// One thread per unit: token 32 m + lane % 32 of the pass, rows 32 rt + 16 s + 4 h + {0..3} and
// the same + 8 (h = lane / 32): the order in which the turned codes hold their rows.  Block b of
// the staging takes one tile of 32 tokens and two row tiles: the 64 rows x 2 bytes that its four
// waves read of a token are one 128-byte line, fetched by this block only.
__device__ __forceinline__ void stage_dy(const StageArgs &a, unsigned b, int t) {
  // the scale: every workgroup reduces the scan's 256 entries again (cheaper than one more launch)
  __shared__ u32 red[4];
  u32 mx = a.maxima[t];
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) mx = max(mx, (u32)__shfl_xor((int)mx, d));
  if ((t & 63) == 0) red[t >> 6] = mx;
  __syncthreads();
  const int kexp = scale_exponent(max(max(red[0], red[1]), max(red[2], red[3])));
  const float scale = __builtin_ldexpf(1.0f, kexp);
  if (b == 0 && t == 0) *a.kword = kexp;
  const int pairs = (a.n_rt + 1) >> 1;
  const int m = (int)(b & 3), pr = (int)((b >> 2) % (unsigned)pairs), pass = (int)((b >> 2) / (unsigned)pairs);
  const int l = t & 63, s = (t >> 6) & 1, rt = 2 * pr + (t >> 7);
  if (pass >= a.passes || rt >= a.n_rt) return;
  const long long u = (long long)pass * a.n_rt * 512 + (((long long)rt * 2 + s) * 4 + m) * 64 + l;
  const int n = a.n0 + kPassTokens * pass + 32 * m + (l & 31), h = l >> 5;
  h8_t v;
  const int ia = 32 * rt + 16 * s + 4 * h;          // rows ia .. ia + 3 and ia + 8 .. ia + 11
  if (n < a.batch && ia + 11 < a.d_out && (a.d_out & 3) == 0) {
    // both runs of four rows inside the matrix and 8-byte aligned (dy is 16-byte aligned)
    typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
    const _Float16 *row = a.dy + (size_t)n * a.d_out + ia;
    const h4_t lo = *reinterpret_cast<const h4_t *>(row), hi = *reinterpret_cast<const h4_t *>(row + 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = lo[e];
      v[4 + e] = hi[e];
    }
  } else {
    const _Float16 *p[8];
    _Float16 x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = ia + (e & 3) + 8 * (e >> 2);
      p[e] = a.dy + (size_t)(n < a.batch ? n : a.batch - 1) * a.d_out + (i < a.d_out ? i : a.d_out - 1);
    }
    load_h<8>(p, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = ia + (e & 3) + 8 * (e >> 2);
      v[e] = (n < a.batch && i < a.d_out) ? x[e] : (_Float16)0.f;
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (_Float16)((float)v[e] * scale);      // a power of two, below 1024 afterwards: exact
  a.a_st[u] = __builtin_bit_cast(u32x4, v);
}

struct StageWeakArgs {
  const _Float16 *weak_w;   // [d_out_pad][kp]
  u32x4 *wst;               // [n_rt][2][kp32][64 lanes] units of 8 fp16
  int kp, kp32, n_rt;
};

// The weak columns in the same operand order: lane % 32 = weak column of the tile, rows as above.
__device__ __forceinline__ void stage_weak(const StageWeakArgs &a, long long u) {
  const long long total = (long long)a.n_rt * 2 * a.kp32 * 64;
  if (u >= total) return;
  const int l = (int)(u & 63);
  const long long q = u >> 6;
  const int tt = (int)(q % a.kp32), s = (int)((q / a.kp32) & 1), rt = (int)(q / a.kp32 / 2);
  const int t = 32 * tt + (l & 31), h = l >> 5;
  h8_t v;
  const _Float16 *p[8];
  _Float16 x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int i = 32 * rt + 16 * s + 4 * h + (e & 3) + 8 * (e >> 2);     // below d_out_pad; padded rows hold 0
    p[e] = a.weak_w + (size_t)i * a.kp + (t < a.kp ? t : a.kp - 1);
  }
  load_h<8>(p, x);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = t < a.kp ? x[e] : (_Float16)0.f;
  a.wst[u] = __builtin_bit_cast(u32x4, v);
}

struct ProdArgs {
  const u32 *codes;     // dwords of the packed tiles
  const u32 *sz;        // [G][d_out_pad] step size | zero point << 16
  const u32x4 *a_st;
  float *part;          // [split][128][d_in_pad]
  const u32x4 *wst;     // staged weak columns, or nullptr: the weak columns of dx are not made here
  float *pw;            // [split][128][32 kp32]: their partial results
  int n_rt, nbp, chunks, d_out_pad, d_in_pad, blocks_per_group, n_groups, split, rt_per_split, kp32;
};

// HAS_W: the weak columns of dx ride along (every workgroup does the matrix instruction, those
// without a tile of weak columns on a tile they do not store: a branch around it costs more).
template <int BITS, bool HAS_W>
__global__ __launch_bounds__(kBwdWaves * 64) void owq_bwd_product(const ProdArgs a) {
  __shared__ float zbuf[kBwdWaves][4][32];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, n32 = lane & 31;
  // Workgroups go to the eight dies (each with its own L2) in turn.  The workgroups that read the
  // same rows of the staged dy (same pass, same range of rows, different block pairs) are given
  // ids that land on one die: die d takes a contiguous eighth of the (pass, range, block pair) order.
  int id = blockIdx.x;
  const int total = gridDim.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int bp = id % a.nbp, sp = (id / a.nbp) % a.split, pass = id / (a.nbp * a.split);
  const u32x4 *a_st = a.a_st + (size_t)pass * a.n_rt * 512;
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
  // Weak columns of dx: the workgroup of block pair bp also takes tile bp of the weak columns
  // (32 of them), each of its waves one tile of 32 tokens, from the same staged dy, unscaled.
  const bool has_w = HAS_W && bp < a.kp32;
  const int wtile = HAS_W ? (bp < a.kp32 ? bp : 0) : 0;
  f16_t wacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) wacc[r] = 0.f;
  constexpr int kDw = BITS == 3 ? 3 : 4;                              // dwords of the lane that hold this wave's columns
  // What one row tile needs from memory besides its codes; fetched one tile ahead.
  struct Fetched {
    u32x4 q[2][2];      // step sizes and zero points of the lane's eight rows of either half
    u32x4 raw[2][4];    // staged dy of the four token tiles
    u32x4 wsu[2];       // staged weak columns
    u32x4 raww[2];      // staged dy of token tile w once more (unscaled operand of the weak product)
  };
  // codes of K-steps 4 w .. 4 w + 3 of the lane: dwords kDw w .. of its 12 or 16; fetched two tiles ahead
  struct Codes {
    u32 cw[4];
  };
  auto fetch_codes = [&](Codes &c, int rt) __attribute__((always_inline)) {
    const size_t tile = (size_t)rt * a.nbp + bp;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int dwi = kDw * w + (v < kDw ? v : 0);
      c.cw[v] = a.codes[((tile * a.chunks + (dwi >> 2)) * 64 + lane) * 4 + (dwi & 3)];
    }
  };
  auto fetch = [&](Fetched &f, int rt) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int i0 = 32 * rt + 16 * s + 4 * h;
      f.q[s][0] = *reinterpret_cast<const u32x4 *>(sz + i0);
      f.q[s][1] = *reinterpret_cast<const u32x4 *>(sz + i0 + 8);
#pragma unroll
      for (int m = 0; m < 4; ++m) f.raw[s][m] = a_st[(((size_t)rt * 2 + s) * 4 + m) * 64 + lane];
      if (HAS_W) {
        f.wsu[s] = a.wst[(((size_t)rt * 2 + s) * a.kp32 + wtile) * 64 + lane];
        f.raww[s] = a_st[(((size_t)rt * 2 + s) * 4 + w) * 64 + lane];
      }
    }
  };
  // turned codes of the two column tiles: B operands for both halves of the 32 rows
  struct Turned {
    u32x4 wb[2][2];
  };
  auto turn = [&](const Codes &cd, Turned &o) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      f16_t t;
#pragma unroll
      for (int r = 0; r < 16; ++r) t[r] = cneg[c];    // start from minus the unpack constant
      if (c == 0) {
        t = mma(a_operand<BITS, 0>(cd.cw, M), sel0, t);
        t = mma(a_operand<BITS, 1>(cd.cw, M), sel1, t);
      } else {
        t = mma(a_operand<BITS, 2>(cd.cw, M), sel0, t);
        t = mma(a_operand<BITS, 3>(cd.cw, M), sel1, t);
      }
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        u32 pk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)       // small integers: exact whatever the rounding
          pk[e] = __builtin_bit_cast(u32, __builtin_amdgcn_cvt_pkrtz(t[8 * s + 2 * e], t[8 * s + 2 * e + 1]));
        o.wb[c][s] = (u32x4){pk[0], pk[1], pk[2], pk[3]};
      }
    }
  };
  auto product = [&](const Fetched &f, const Turned &tw) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const u32x4 q0 = f.q[s][0], q1 = f.q[s][1];
      const u32 d[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
      u32 sp2[4], zp2[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        sp2[p] = __builtin_amdgcn_perm(d[2 * p + 1], d[2 * p], 0x05040100u);   // (lo of even, lo of odd)
        zp2[p] = __builtin_amdgcn_perm(d[2 * p + 1], d[2 * p], 0x07060302u);   // (hi of even, hi of odd)
      }
      if (HAS_W)
        wacc = mma(__builtin_bit_cast(h8_t, f.raww[s]), __builtin_bit_cast(h8_t, f.wsu[s]), wacc);
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const u32x4 raw = f.raw[s][m];
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
        acc[m][0] = mma(aop, __builtin_bit_cast(h8_t, tw.wb[0][s]), acc[m][0]);
        acc[m][1] = mma(aop, __builtin_bit_cast(h8_t, tw.wb[1][s]), acc[m][1]);
      }
    }
  };
  // Tile t's product runs while tile t + 1's codes are turned (its vector work under the product's
  // matrix instructions), tile t + 1's operands are in flight and tile t + 2's codes are fetched.
  const int last = rt1 - 1;
  Fetched cur, nxt;
  Codes c1, c2;
  Turned tw, tn;
  fetch_codes(c1, rt0);
  fetch(cur, rt0);
  fetch_codes(c2, rt0 + 1 < rt1 ? rt0 + 1 : last);
  turn(c1, tw);
  for (int rt = rt0; rt < rt1; ++rt) {
    fetch(nxt, rt + 1 < rt1 ? rt + 1 : last);        // past the range: the last tile again, unused
    c1 = c2;
    fetch_codes(c2, rt + 2 < rt1 ? rt + 2 : last);
    __builtin_amdgcn_sched_barrier(0);               // the loads above go out before the work below
    product(cur, tw);
    turn(c1, tn);
    cur = nxt;
    tw = tn;
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
  float *part = a.part + ((size_t)pass * a.split + sp) * kPassTokens * a.d_in_pad;
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
  if (has_w) {
    float *pw = a.pw + ((size_t)pass * a.split + sp) * kPassTokens * (32 * a.kp32);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int nl = 8 * (r >> 2) + 4 * h + (r & 3);
      pw[(size_t)(32 * w + nl) * (32 * a.kp32) + 32 * bp + n32] = wacc[r];
    }
  }
}

struct SumArgs {
  const float *part;    // [pass][split][128][d_in_pad]
  const float *pw;      // [pass][split][128][32 kp32], or nullptr
  const uint8_t *wmask; // bit j = column j is weak
  const int *weak_idx;
  _Float16 *dx;         // [batch][d_in]
  int d_in, d_in_pad, split, n0, ntok, k, kp32, dense_blocks;
  const int *kword;     // dy was scaled by 2^*kword
};

// dx: the partial results added in a fixed order.  Blocks below dense_blocks take 1024 columns
// each and skip the weak ones; the blocks after them take 256 weak columns each.
__global__ __launch_bounds__(256) void owq_bwd_sum(const SumArgs a) {
  if ((int)blockIdx.y >= a.ntok) return;
  const int pass = blockIdx.y / kPassTokens, nl = blockIdx.y % kPassTokens;
  const size_t base = (size_t)pass * a.split * kPassTokens;           // first (range, token) row of this pass
  const float back = __builtin_ldexpf(1.0f, -*a.kword);                // undo the scaling of dy
  if ((int)blockIdx.x < a.dense_blocks) {
    const int j = (blockIdx.x * 256 + threadIdx.x) * 4;            // four columns per thread (d_in_pad is a multiple of 256)
    if (j >= a.d_in) return;
    f4_t v = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < a.split; ++s)
      v += *reinterpret_cast<const f4_t *>(a.part + (base + (size_t)s * kPassTokens + nl) * a.d_in_pad + j);
    const u32 weak = (a.wmask[j >> 3] >> (j & 7)) & 15u;          // j is a multiple of 4: the four bits sit in one byte
    _Float16 *out = a.dx + (size_t)(a.n0 + blockIdx.y) * a.d_in + j;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (j + e < a.d_in && !((weak >> e) & 1u)) out[e] = (_Float16)(v[e] * back);
  } else {
    const int t = ((int)blockIdx.x - a.dense_blocks) * 256 + threadIdx.x;
    if (a.pw == nullptr || t >= a.k) return;
    const int col = a.weak_idx[t];
    if ((unsigned)col >= (unsigned)a.d_in) return;
    float v = 0.f;
    for (int s = 0; s < a.split; ++s) v += a.pw[(base + (size_t)s * kPassTokens + nl) * (32 * a.kp32) + t];
    a.dx[(size_t)(a.n0 + blockIdx.y) * a.d_in + col] = (_Float16)(v * back);
  }
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

struct StageXArgs {
  const _Float16 *x;         // [batch][d_in]
  const int *weak_idx;
  u32x4 *xw_st;              // [token steps of 16][kp32][64 lanes] units of 8 fp16
  int d_in, k, kp32, batch, steps;
};

// The activations at the weak columns as A operands with the tokens on the contraction axis:
// lane % 32 = weak column of the tile, eight consecutive tokens per lane.
__device__ __forceinline__ void stage_x(const StageXArgs &a, long long u) {
  if (u >= (long long)a.steps * a.kp32 * 64) return;
  const int l = (int)(u & 63);
  const long long q = u >> 6;
  const int tt = (int)(q % a.kp32), ks = (int)(q / a.kp32);
  const int t = 32 * tt + (l & 31), h = l >> 5;
  int col = t < a.k ? a.weak_idx[t] : -1;
  if ((unsigned)col >= (unsigned)a.d_in) col = -1;
  h8_t v;
  const _Float16 *p[8];
  _Float16 xv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int n = 16 * ks + 8 * h + e;
    p[e] = a.x + (size_t)(n < a.batch ? n : a.batch - 1) * a.d_in + (col >= 0 ? col : 0);
  }
  load_h<8>(p, xv);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (col >= 0 && 16 * ks + 8 * h + e < a.batch) ? xv[e] : (_Float16)0.f;
  a.xw_st[u] = __builtin_bit_cast(u32x4, v);
}

struct StageAllArgs {
  StageArgs dy;
  StageWeakArgs weak;
  StageXArgs x;
  unsigned dy_blocks, weak_blocks;   // blocks [0, dy_blocks) stage dy, the next weak_blocks the weak columns, the rest x
};

// All staging of a call in one launch: the three parts are independent of each other.
__global__ __launch_bounds__(256) void owq_bwd_stage_all(const StageAllArgs a) {
  const unsigned b = blockIdx.x;
  if (b < a.dy_blocks) stage_dy(a.dy, b, (int)threadIdx.x);
  else if (b < a.dy_blocks + a.weak_blocks) stage_weak(a.weak, (long long)(b - a.dy_blocks) * 256 + threadIdx.x);
  else stage_x(a.x, (long long)(b - a.dy_blocks - a.weak_blocks) * 256 + threadIdx.x);
}

struct DwwArgs {
  const _Float16 *dy;        // [batch][d_out]
  const u32x4 *xw_st;
  float *dww;                // [d_out][k]
  int d_out, k, kp32, batch, steps;
};

// dww[i, t] = sum_n x[n, idx[t]] dy[n, i] on the matrix cores: a workgroup owns 32 rows i and NTT
// tiles of 32 weak columns; its four waves deal the token steps among them and add their results
// through LDS in a fixed order.  The work is tiny and all latency: a wave sends out the loads of
// eight of its token steps at once.
template <int NTT>
__global__ __launch_bounds__(256) void owq_bwd_dww(const DwwArgs a) {
  __shared__ float red[4][16][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5;
  const int i = blockIdx.x * 32 + (lane & 31), tt0 = blockIdx.y * NTT;
  const int ntt = a.kp32 - tt0 < NTT ? a.kp32 - tt0 : NTT;
  const int ic = i < a.d_out ? i : a.d_out - 1;
  f16_t acc[NTT];
#pragma unroll
  for (int c = 0; c < NTT; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  constexpr int kSteps = 8;                          // token steps of a wave in flight together
  for (int ks = w; ks < a.steps; ks += 4 * kSteps) {
    h8_t b[kSteps];
    u32x4 xa[kSteps][NTT];
    const _Float16 *p[8 * kSteps];
    _Float16 v[8 * kSteps];
#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
      const int k2 = ks + 4 * u;                     // k2 >= steps: tokens past the batch, zeros
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int n = 16 * k2 + 8 * h + e;
        p[8 * u + e] = a.dy + (size_t)(n < a.batch ? n : a.batch - 1) * a.d_out + ic;
      }
      const int kc = k2 < a.steps ? k2 : a.steps - 1;
#pragma unroll
      for (int c = 0; c < NTT; ++c) xa[u][c] = a.xw_st[((size_t)kc * a.kp32 + (c < ntt ? tt0 + c : tt0)) * 64 + lane];
    }
    load_h<8 * kSteps>(p, v);
#pragma unroll
    for (int u = 0; u < kSteps; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        b[u][e] = (16 * (ks + 4 * u) + 8 * h + e < a.batch && i < a.d_out) ? v[8 * u + e] : (_Float16)0.f;
#pragma unroll
    for (int u = 0; u < kSteps; ++u)
#pragma unroll
      for (int c = 0; c < NTT; ++c) acc[c] = mma(__builtin_bit_cast(h8_t, xa[u][c]), b[u], acc[c]);
  }
#pragma unroll
  for (int c = 0; c < NTT; ++c) {
    __syncthreads();                                 // every thread, every round: the trip count is fixed
#pragma unroll
    for (int r = 0; r < 16; ++r) red[w][r][lane] = acc[c][r];
    __syncthreads();
    if (c < ntt) {
      // this thread's share of the 16 x 64 results: registers 4 w .. 4 w + 3 = four consecutive weak columns
      f4_t v;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r = 4 * w + q;
        v[q] = (red[0][r][lane] + red[1][r][lane]) + (red[2][r][lane] + red[3][r][lane]);
      }
      const int t = 32 * (tt0 + c) + 8 * w + 4 * h;
      if (i < a.d_out) {
        float *out = a.dww + (size_t)i * a.k + t;
        if ((a.k & 3) == 0 && t + 3 < a.k) {
          *reinterpret_cast<f4_t *>(out) = v;        // 16-byte aligned: dww is, and k is a multiple of 4
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (t + q < a.k) out[q] = v[q];
        }
      }
    }
  }
}

struct BwdPlan {
  int passes;                    // passes per set of launches
  int split, rt_per_split, kp32;
  bool weak_in_product;          // every tile of 32 weak columns finds a block pair's workgroup
  int x_steps;                   // steps of 16 tokens of the whole batch
  size_t a_st_bytes, part_bytes, wst_bytes, pw_bytes, xw_bytes, total;
};

BwdPlan plan(const owq_layer_info_t &g, int batch) {
  BwdPlan p;
  const int all_passes = (batch + kPassTokens - 1) / kPassTokens;
  p.passes = all_passes < kLaunchPasses ? (all_passes < 1 ? 1 : all_passes) : kLaunchPasses;
  // Ranges of rows per block pair.  A compute unit holds one workgroup at a time (its registers), so
  // the product takes rounds of 256 workgroups, each as long as a workgroup's row tiles (plus a fixed
  // part: set-up and the store of its partial results); every further range costs the sum kernel about
  // one row tile's time.  Cost in row tiles, fitted to measurements on MI355X.
  int split = 1;
  double best = 1e30;
  for (int sp = 1; sp <= kSplitMax && sp <= g.n_rt; ++sp) {
    const long long wgs = (long long)g.nbp * sp * p.passes;
    const double rounds = (double)((wgs + 255) / 256);
    const double cost = rounds * ((g.n_rt + sp - 1) / sp + 6.0) + 1.1 * sp;
    if (cost < best) {
      best = cost;
      split = sp;
    }
  }
  p.rt_per_split = (g.n_rt + split - 1) / split;
  p.split = (g.n_rt + p.rt_per_split - 1) / p.rt_per_split;
  p.a_st_bytes = (size_t)p.passes * g.n_rt * 2 * 4 * 64 * 16;
  p.part_bytes = (size_t)p.passes * p.split * kPassTokens * ((size_t)g.nbp * 256) * 4;
  p.kp32 = (g.kp + 31) / 32;
  p.weak_in_product = g.k > 0 && p.kp32 <= g.nbp;
  p.wst_bytes = p.weak_in_product ? (size_t)g.n_rt * 2 * p.kp32 * 64 * 16 : 0;
  p.pw_bytes = p.weak_in_product ? (size_t)p.passes * p.split * kPassTokens * 32 * p.kp32 * 4 : 0;
  p.x_steps = (batch + 15) / 16;
  p.xw_bytes = g.k > 0 ? (size_t)p.x_steps * p.kp32 * 64 * 16 : 0;
  p.total = p.a_st_bytes + p.part_bytes + p.wst_bytes + p.pw_bytes + p.xw_bytes + kScanBytes;
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
  *bytes = plan(h->info, batch).total;
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
  if (!dy || (dww && g.k > 0 && !x) || !workspace) return OWQ_ERR_NULL;
  const BwdPlan p = plan(g, batch);
  if (workspace_bytes < p.total) return OWQ_ERR_BUFFER;
  if (((uintptr_t)dy | (uintptr_t)x | (uintptr_t)dx | (uintptr_t)dww) & 15u) return OWQ_ERR_BUFFER;
  if ((uintptr_t)workspace & 255u) return OWQ_ERR_BUFFER;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint8_t *blob = static_cast<const uint8_t *>(h->dev_buf);
  uint8_t *ws = static_cast<uint8_t *>(workspace);
  hipError_t err = hipSuccess;
  u32x4 *a_st = reinterpret_cast<u32x4 *>(ws);
  float *part = reinterpret_cast<float *>(ws + p.a_st_bytes);
  u32x4 *wst = p.weak_in_product ? reinterpret_cast<u32x4 *>(ws + p.a_st_bytes + p.part_bytes) : nullptr;
  float *pw = p.weak_in_product ? reinterpret_cast<float *>(ws + p.a_st_bytes + p.part_bytes + p.wst_bytes) : nullptr;
  u32x4 *xw_st = reinterpret_cast<u32x4 *>(ws + p.a_st_bytes + p.part_bytes + p.wst_bytes + p.pw_bytes);
  u32 *maxima = reinterpret_cast<u32 *>(ws + p.total - kScanBytes);
  int *kword = reinterpret_cast<int *>(maxima + kMaxBlocks);
  const bool want_dww = dww && g.k > 0;
  const int per_launch = p.passes * kPassTokens;
  if (dx) {
    const size_t halves = (size_t)batch * g.d_out;
    hipLaunchKernelGGL(owq_bwd_absmax, dim3(kMaxBlocks), dim3(256), 0, st, static_cast<const u32x4 *>(dy), halves / 8, halves,
                       static_cast<const unsigned short *>(dy), maxima);
  }
  // The first launch stages everything the call needs; later groups of passes stage their dy only.
  for (int n0 = 0; n0 < batch && err == hipSuccess && (dx || n0 == 0); n0 += per_launch) {
    const int ntok = batch - n0 < per_launch ? batch - n0 : per_launch;
    const int passes = (ntok + kPassTokens - 1) / kPassTokens;
    StageAllArgs sa = {};
    sa.dy = {static_cast<const _Float16 *>(dy), a_st, g.d_out, g.n_rt, n0, batch, passes, maxima, kword};
    sa.weak = {reinterpret_cast<const _Float16 *>(blob + g.off_weak_w), wst, g.kp, p.kp32, g.n_rt};
    sa.x = {static_cast<const _Float16 *>(x), reinterpret_cast<const int *>(blob + g.off_weak_idx), xw_st,
            g.d_in, g.k, p.kp32, batch, p.x_steps};
    sa.dy_blocks = dx ? (unsigned)(((g.n_rt + 1) / 2) * 4 * passes) : 0u;
    sa.weak_blocks = dx && n0 == 0 && p.weak_in_product ? (unsigned)(((long long)g.n_rt * 2 * p.kp32 * 64 + 255) / 256) : 0u;
    const unsigned x_blocks = want_dww && n0 == 0 ? (unsigned)(((long long)p.x_steps * p.kp32 * 64 + 255) / 256) : 0u;
    if (sa.dy_blocks + sa.weak_blocks + x_blocks > 0)
      hipLaunchKernelGGL(owq_bwd_stage_all, dim3(sa.dy_blocks + sa.weak_blocks + x_blocks), dim3(256), 0, st, sa);
    if (dx) {
      ProdArgs pa;
      pa.codes = reinterpret_cast<const u32 *>(blob + g.off_codes);
      pa.sz = reinterpret_cast<const u32 *>(blob + g.off_sz);
      pa.a_st = a_st;
      pa.part = part;
      pa.wst = wst;
      pa.pw = pw;
      pa.kp32 = p.kp32;
      pa.n_rt = g.n_rt;
      pa.nbp = g.nbp;
      pa.chunks = g.chunks;
      pa.d_out_pad = g.d_out_pad;
      pa.d_in_pad = g.nbp * 256;
      pa.blocks_per_group = g.group_size == 0 ? 0x40000000 : g.group_size / kBlockCols;
      pa.n_groups = g.n_groups;
      pa.split = p.split;
      pa.rt_per_split = p.rt_per_split;
      const dim3 grid((unsigned)(g.nbp * p.split * passes));
      const dim3 block(kBwdWaves * 64);
      if (g.bits == 3 && p.weak_in_product) hipLaunchKernelGGL((owq_bwd_product<3, true>), grid, block, 0, st, pa);
      else if (g.bits == 3) hipLaunchKernelGGL((owq_bwd_product<3, false>), grid, block, 0, st, pa);
      else if (p.weak_in_product) hipLaunchKernelGGL((owq_bwd_product<4, true>), grid, block, 0, st, pa);
      else hipLaunchKernelGGL((owq_bwd_product<4, false>), grid, block, 0, st, pa);
      const int dense_blocks = (g.d_in + 1023) / 1024, weak_blocks = p.weak_in_product ? (g.k + 255) / 256 : 0;
      SumArgs su = {part, pw, blob + g.off_wmask, reinterpret_cast<const int *>(blob + g.off_weak_idx),
                    static_cast<_Float16 *>(dx), g.d_in, g.nbp * 256, p.split, n0, ntok, g.k, p.kp32, dense_blocks, kword};
      hipLaunchKernelGGL(owq_bwd_sum, dim3((unsigned)(dense_blocks + weak_blocks), (unsigned)ntok), dim3(256), 0, st, su);
      if (g.k > 0 && !p.weak_in_product) {
        WeakArgs wa = {static_cast<const _Float16 *>(dy), reinterpret_cast<const _Float16 *>(blob + g.off_weak_w),
                       reinterpret_cast<const int *>(blob + g.off_weak_idx), static_cast<_Float16 *>(dx),
                       g.d_out, g.d_in, g.kp, n0, ntok};
        hipLaunchKernelGGL(owq_bwd_weak, dim3((unsigned)(g.kp / 8), (unsigned)((ntok + 7) / 8)), dim3(256), 0, st, wa);
      }
    }
    err = hipGetLastError();
  }
  if (want_dww && err == hipSuccess) {
    DwwArgs da = {static_cast<const _Float16 *>(dy), xw_st, dww, g.d_out, g.k, p.kp32, batch, p.x_steps};
    const unsigned rows32 = (unsigned)((g.d_out + 31) / 32);
    if (p.kp32 == 1) hipLaunchKernelGGL(owq_bwd_dww<1>, dim3(rows32, 1), dim3(256), 0, st, da);
    else if (p.kp32 == 2) hipLaunchKernelGGL(owq_bwd_dww<2>, dim3(rows32, 1), dim3(256), 0, st, da);
    else hipLaunchKernelGGL(owq_bwd_dww<4>, dim3(rows32, (unsigned)((p.kp32 + 3) / 4)), dim3(256), 0, st, da);
    err = hipGetLastError();
  }
  if (err != hipSuccess) {
    h->info.last_hip_error = (int32_t)err;
    return OWQ_ERR_HIP;
  }
  return OWQ_OK;
}
