// Batched path of the OWQ mixed-precision linear layer on the matrix cores of gfx950
// (tile layout: 32 rows x 256 columns per tile, 64 tokens per pass over the weights).
//
// Same result as the single-token kernel (paper: storage paragraph of "Outlier-Aware
// Weight Quantization", section "Acceleration on Real Device"):
//     y[n,i] = sum_{j not weak} s_ig (q_ij - z_ig) x[n,j]  +  sum_t Ww_it x[n, idx_t]
// computed as a dense contraction.  The paper measures single tokens only; this path is
// this library's own extension for prompts.
//
// Three launches per pass of up to 64 tokens:
//   stage   copies x into the order the matrix instruction reads it, clears the weak
//           columns (by select), gathers x at the weak indices and sums, per token and
//           block, x and c*x (c = the constant each code is OR-ed into, see below);
//           one workgroup per 256 columns and 32 tokens;
//   mma     every wave owns 64 rows x 64 tokens of fp32 accumulators and walks along the
//           columns: codes go from registers straight into the A operand (a pair of codes
//           is masked out of a dword and OR-ed into the mantissas of 2^(10-o), giving
//           2^(10-o)+q exactly), tokens come from LDS as the B operand.  The flattened
//           (row group, column step) sequence is cut into equal ranges, one per workgroup,
//           so that all compute units stay busy whatever the shape; a workgroup writes one
//           partial result per row group it touches.  While their first loads are in
//           flight the first 64 workgroups add up the block sums of one token each;
//   finish  adds the partial results of a row group in a fixed order, removes the constant
//           part and the zero point, scales, adds the product of the fp16 weak columns
//           (a few more K-steps on the matrix cores), rounds to fp16.
// No atomics: results are reproducible.
#include <hip/hip_runtime.h>

#include <mutex>

#include <type_traits>

#include "owq_internal.h"
#include "owq_tile_device.h"

namespace owq {

// ---------------------------------------------------------------------------
// stage
// ---------------------------------------------------------------------------
struct StageArgs {
  const _Float16 *x;           // [ntok][d_in] of this pass
  const unsigned char *wmask;  // bit e of byte i: column 8i+e is weak
  const int *weak_idx;         // [kp], padding -1
  u32x4 *xs;                   // [nbp][16][2][64] units
  f2_t *bsum;                  // [nblk][64]
  _Float16 *xw;                // [64][kp]
  int d_in, ntok, nblk, kp;
};

// grid (block pair, token tile of 32); thread = (token, octets oo, oo+8, oo+16, oo+24 of the pair).
template <int BITS>
__global__ __launch_bounds__(256) void owq_tile_stage(const StageArgs a) {
  __shared__ f2_t red[8][2][32];
  const int tid = threadIdx.x, nl = tid & 31, oo = tid >> 5;
  const int bp = blockIdx.x, nt = blockIdx.y;
  const int n = nt * 32 + nl;
  const bool valid = n < a.ntok;
  const _Float16 *xr = a.x + (size_t)(valid ? n : 0) * a.d_in;
  const bool vec = ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0) && ((a.d_in & 7) == 0);
  // octet o = 8*trip + oo of the pair: k-step (o >> 1) & 7, whose place in its quad is (oo >> 1) & 3
  float cst[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (((oo >> 1) & 3) == q) v = (float)(1 << (10 - pair_offset(BITS, q, i)));
    cst[i] = v;
  }
  u32 w[4][4];
  u32 m[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int o = it * 8 + oo;
    const int j0 = bp * 256 + o * 8;
    w[it][0] = w[it][1] = w[it][2] = w[it][3] = 0u;
    if (valid && j0 < a.d_in) {
      if (vec) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(xr + j0);
        w[it][0] = v.x; w[it][1] = v.y; w[it][2] = v.z; w[it][3] = v.w;
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int j = j0 + t;
          const u32 h = j < a.d_in ? (u32)__builtin_bit_cast(unsigned short, xr[j]) : 0u;
          w[it][t >> 1] |= h << (16 * (t & 1));
        }
      }
    }
    m[it] = a.wmask[bp * 32 + o];
  }
  float X[2] = {0.f, 0.f}, Bc[2] = {0.f, 0.f};
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int o = it * 8 + oo;
#pragma unroll
    for (int i = 0; i < 4; ++i) {        // weak columns contribute nothing to the dense term
      if (m[it] & (1u << (2 * i))) w[it][i] &= 0xffff0000u;
      if (m[it] & (2u << (2 * i))) w[it][i] &= 0x0000ffffu;
    }
    if (valid) {
      const u32x4 v = {w[it][0], w[it][1], w[it][2], w[it][3]};
      a.xs[((size_t)(bp * 16 + (o >> 1)) * 2 + nt) * 64 + (o & 1) * 32 + nl] = v;
    }
    float sx = 0.f, sb = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float pr = dot2(w[it][i], kOnes, 0.f);
      sx += pr;
      sb = __builtin_fmaf(pr, cst[i], sb);
    }
    X[it >> 1] += sx;
    Bc[it >> 1] += sb;
  }
  red[oo][0][nl] = (f2_t){X[0], Bc[0]};
  red[oo][1][nl] = (f2_t){X[1], Bc[1]};
  __syncthreads();
  if (tid < 64 && valid) {
    const int b = tid >> 5;
    float sx = 0.f, sb = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const f2_t r = red[q][b][nl];
      sx += r.x;
      sb += r.y;
    }
    a.bsum[(size_t)(2 * bp + b) * 64 + n] = (f2_t){sx, sb};
  }
  // activations at the weak columns: the workgroups of a token tile share its 32 x kp elements
  for (int e = bp * 256 + tid; e < 32 * a.kp; e += (int)gridDim.x * 256) {
    const int ln = e / a.kp, t = e - ln * a.kp, nn = nt * 32 + ln;
    if (nn < a.ntok) {
      const int j = a.weak_idx[t];
      a.xw[nn * a.kp + t] = j >= 0 ? a.x[(size_t)nn * a.d_in + j] : (_Float16)0;
    }
  }
}

// ---------------------------------------------------------------------------
// mma
// ---------------------------------------------------------------------------
struct TileArgs {
  const u32x4 *codes;
  const u32 *sz;         // [n_groups][d_out_pad]: fp16 scale | fp16 zero << 16
  const u32x4 *xs;
  const f2_t *bsum;
  f2_t *tsum;            // [64]: per token, sum over all blocks of (x, c*x)
  f4_t *slots;
  int nbp, n_rt, n_groups, bpg, nblk, d_out_pad;
  int steps;             // row groups x column steps
  int split;             // > 0: every row group is cut into `split` ranges (grid = row groups x split);
                         // 0: the whole flattened sequence is cut into gridDim.x equal ranges
};

template <int S> struct KStep {};   // tag: k-step S of a column step
template <int S> __device__ std::integral_constant<int, S> kstep_index(KStep<S>);

// k-steps S..15 of one column step: wd0/wd1 = the dwords of the wave's two row tiles.
// between(KStep<S>) runs after the matrix instructions of k-step S have been issued: the
// caller spreads its global loads over the k-steps there, so that the memory pipeline of
// the compute unit works on them while the matrix cores run.
// GROUPED: the first k-step of a 128-column block (k-steps 0 and 8) starts the four tiles from `zero`.
template <int BITS, int NT, bool GROUPED, int S>
struct KSteps {
  template <typename Between>
  static __device__ __forceinline__ void run(const u32 *wd0, const u32 *wd1, const u32x4 *xb, int lane,
                                             const Magic &M, f16_t *acc, const f16_t &zero, Between &between) {
    constexpr bool kFirst = GROUPED && (S & 7) == 0;
    const h8_t a0 = a_operand<BITS, S>(wd0, M), a1 = a_operand<BITS, S>(wd1, M);
    const h8_t b0 = __builtin_bit_cast(h8_t, xb[(S * 2 + 0) * 64 + lane]);
    acc[0] = mma(a0, b0, kFirst ? zero : acc[0]);
    acc[2] = mma(a1, b0, kFirst ? zero : acc[2]);
    if (NT == 2) {
      const h8_t b1 = __builtin_bit_cast(h8_t, xb[(S * 2 + 1) * 64 + lane]);
      acc[1] = mma(a0, b1, kFirst ? zero : acc[1]);
      acc[3] = mma(a1, b1, kFirst ? zero : acc[3]);
    }
    between(KStep<S>{});
    KSteps<BITS, NT, GROUPED, S + 1>::run(wd0, wd1, xb, lane, M, acc, zero, between);
  }
};
template <int BITS, int NT, bool GROUPED>
struct KSteps<BITS, NT, GROUPED, 16> {
  template <typename Between>
  static __device__ __forceinline__ void run(const u32 *, const u32 *, const u32x4 *, int, const Magic &, f16_t *, const f16_t &,
                                             Between &) {}
};

template <int J> struct Slot {};   // tag: code buffer J of the three
template <int J> __device__ std::integral_constant<int, J> slot_index(Slot<J>);

// One workgroup = WAVES waves = WAVES*64 rows (a row group); wave w owns row tiles 2w, 2w+1
// of it.  Two waves share a SIMD (two workgroups of 4 waves, or one of 8, per compute unit;
// at most 256 registers each) so that one computes while the other waits at its barrier.
template <int BITS, int NT, bool GROUPED, int WAVES>
__global__ __launch_bounds__(WAVES * 64, GROUPED ? 1 : 2) void owq_tile_mma(const TileArgs a) {
  constexpr int CH = BITS == 3 ? 3 : 4;
  constexpr int THREADS = WAVES * 64;
  constexpr int XU = (NT == 2 ? 2048 : 1024) / THREADS;   // activation units a thread stages per step
  constexpr int RTG = 2 * WAVES;                           // row tiles per row group
  constexpr int SLOT_UNITS = WAVES * 16 * 64;              // 16-byte units of one partial result
  constexpr int ROWS = WAVES * 64;
  // LDS buffer of a step: the activation tile; for grouped layers also, per block of the step, the scales of
  // the rows and their zero-points as floats (two planes of ROWS), and per block and token the two
  // 16-byte units that hold sum c*x and sum x as the token operand of the correcting matrix instruction
  constexpr int SZ_UNITS = GROUPED ? ROWS : 0, BS_UNITS = GROUPED ? 256 : 0;
  constexpr int BUF_UNITS = kUnitsPerTile + SZ_UNITS + BS_UNITS;
  static_assert(XU >= 1 && XU <= 8 && 8 + 2 * CH <= 16, "loads must fit the 16 k-steps");
  static_assert(THREADS >= ROWS / 2 + 64, "one thread per staged unit of scales and sums");
  extern __shared__ u32x4 lds[];                // two buffers
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int P = gridDim.x, p = blockIdx.x;
  int lo, hi;
  if (a.split > 0) {         // ranges aligned to row groups: workgroups of one range move in step
    const int g0 = p / a.split, sp = p - g0 * a.split;
    lo = g0 * a.nbp + (int)((long long)sp * a.nbp / a.split);
    hi = g0 * a.nbp + (int)((long long)(sp + 1) * a.nbp / a.split);
  } else {
    lo = (int)((long long)p * a.steps / P);
    hi = (int)((long long)(p + 1) * a.steps / P);
  }
  if (lo >= hi) return;
  int rg = lo / a.nbp, bp = lo - rg * a.nbp;    // the step being computed
  int st = lo;

  // ---- fetch cursors: codes two steps ahead, activations one step ahead -------------
  // Past the last step of the workgroup the cursors stay on it: the loads still go out
  // (their number in flight is the same on every path) and their data is dropped.
  u32x4 cb[3][2][CH];
  int c_st = lo, c_rg = rg, c_bp = bp;
  auto fetch_code = [&](int slot, int rtl, int c) {
    const int rt = min(c_rg * RTG + 2 * w + rtl, a.n_rt - 1);
    const u32x4 *src = a.codes + ((size_t)(rt * a.nbp + c_bp) * CH + c) * 64 + lane;
    cb[slot][rtl][c] = __builtin_nontemporal_load(src);
  };
  auto advance_codes = [&]() {
    const bool more = c_st + 1 < hi, wrap = more && c_bp + 1 == a.nbp;
    c_st += more ? 1 : 0;
    c_rg += wrap ? 1 : 0;
    c_bp = wrap ? 0 : c_bp + (more ? 1 : 0);
  };
  // Staging registers.  8 waves (4 or fewer units per thread): three sets rotating with the code
  // buffers, the tile of step st + 2 is fetched during step st and goes to LDS at the end of
  // step st + 1, when it has long arrived.  4 waves: one set, one step ahead.
  constexpr int XSETS = WAVES == 8 ? 3 : 1;
  u32x4 xg[XSETS][XU];
  u32x4 auxg[XSETS];
#pragma unroll
  for (int i = 0; i < XSETS; ++i) auxg[i] = (u32x4){0u, 0u, 0u, 0u};
  int x_st = lo, x_bp = bp, x_rg = rg;
  auto unit_of = [&](int j) {
    const int i = tid + THREADS * j;
    return NT == 2 ? i : ((i >> 6) * 128 + (i & 63));
  };
  auto fetch_x = [&](int set, int j) { xg[set][j] = a.xs[(size_t)x_bp * kUnitsPerTile + unit_of(j)]; };
  // grouped layers: thread t < ROWS/2 stages (scale, zero) of 4 rows of one block of the step,
  // the next 64 threads stage the sums of 2 tokens of one block
  auto fetch_aux = [&](int set) {
    if constexpr (GROUPED) {
      const u32x4 *src = reinterpret_cast<const u32x4 *>(a.sz);
      if (tid < ROWS / 2) {
        const int h = tid / (ROWS / 4), r4 = tid - h * (ROWS / 4);
        int g = (2 * x_bp + h) / a.bpg;
        if (g > a.n_groups - 1) g = a.n_groups - 1;
        int row = x_rg * ROWS + r4 * 4;
        if (row > a.d_out_pad - 4) row = a.d_out_pad - 4;
        src = reinterpret_cast<const u32x4 *>(a.sz + (size_t)g * a.d_out_pad + row);
      } else if (tid < ROWS / 2 + 64) {
        const int u = tid - ROWS / 2;
        src = reinterpret_cast<const u32x4 *>(a.bsum + (size_t)(2 * x_bp + (u >> 5)) * 64 + (u & 31) * 2);
      }
      auxg[set] = *src;
    }
  };
  auto advance_x = [&]() {
    const bool more = x_st + 1 < hi, wrap = more && x_bp + 1 == a.nbp;
    x_st += more ? 1 : 0;
    x_rg += wrap ? 1 : 0;
    x_bp = wrap ? 0 : x_bp + (more ? 1 : 0);
  };
  auto store_x = [&](int set, int buf) {
#pragma unroll
    for (int j = 0; j < XU; ++j) lds[buf * BUF_UNITS + unit_of(j)] = xg[set][j];
    if constexpr (GROUPED) {
      if (tid < ROWS / 2) {
        // four rows of block h: scales to plane 2h, zero-points to plane 2h + 1
        const int h = tid / (ROWS / 4), r4 = tid - h * (ROWS / 4);
        const u32 d[4] = {auxg[set].x, auxg[set].y, auxg[set].z, auxg[set].w};
        float *pl = reinterpret_cast<float *>(lds + buf * BUF_UNITS + kUnitsPerTile) + 2 * h * ROWS + r4 * 4;
        *reinterpret_cast<f4_t *>(pl) = (f4_t){half_lo(d[0]), half_lo(d[1]), half_lo(d[2]), half_lo(d[3])};
        *reinterpret_cast<f4_t *>(pl + ROWS) = (f4_t){half_hi(d[0]), half_hi(d[1]), half_hi(d[2]), half_hi(d[3])};
      } else if (tid < ROWS / 2 + 64) {
        // two tokens of one block: C = sum c*x and X = sum x in three bf16 pieces each (the top 16 bits of what
        // is left, so the pieces add up to the float exactly), in the order the correcting instruction
        // multiplies them: k = 0..7: C_h C_m C_l X_h X_m X_l X_h X_m; k = 8: X_l
        const int u = tid - ROWS / 2;
        u32x4 *dst = lds + buf * BUF_UNITS + kUnitsPerTile + SZ_UNITS + ((u >> 5) * 64 + (u & 31) * 2) * 2;
        auto pieces = [&](u32 xbits, u32 cbits, u32x4 *out) __attribute__((always_inline)) {
          const float X = __builtin_bit_cast(float, xbits), Cs = __builtin_bit_cast(float, cbits);
          const u32 ch = cbits & 0xffff0000u;
          const float cr = Cs - __builtin_bit_cast(float, ch);
          const u32 cm = __builtin_bit_cast(u32, cr) & 0xffff0000u;
          const u32 cl = __builtin_bit_cast(u32, cr - __builtin_bit_cast(float, cm)) & 0xffff0000u;
          const u32 xh = xbits & 0xffff0000u;
          const float xr = X - __builtin_bit_cast(float, xh);
          const u32 xmid = __builtin_bit_cast(u32, xr) & 0xffff0000u;
          const u32 xl = __builtin_bit_cast(u32, xr - __builtin_bit_cast(float, xmid)) & 0xffff0000u;
          out[0] = (u32x4){(ch >> 16) | cm, (cl >> 16) | xh, (xmid >> 16) | xl, (xh >> 16) | xmid};
          out[1] = (u32x4){xl >> 16, 0u, 0u, 0u};
        };
        const u32x4 v = auxg[set];           // (sum x, sum c*x) of two tokens
        pieces(v.x, v.y, dst);
        pieces(v.z, v.w, dst + 2);
      }
    }
  };

#pragma unroll
  for (int j = 0; j < XU; ++j) fetch_x(0, j);
  fetch_aux(0);
  advance_x();
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) {
#pragma unroll
    for (int i = 0; i < 2 * CH; ++i) fetch_code(sl, i / CH, i % CH);
    advance_codes();
  }
  if (!GROUPED) {
    // While the first loads are in flight: the sums over all blocks of token n, for the
    // finish kernel (layers with one scale per row only).  Fixed order of additions.
    __shared__ f2_t tred[WAVES];
    for (int n = p; n < kScratchBatch; n += P) {
      float sx = 0.f, sb = 0.f;
      for (int b = tid; b < a.nblk; b += THREADS) {
        const f2_t v = a.bsum[(size_t)b * 64 + n];
        sx += v.x;
        sb += v.y;
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        sx += __shfl_xor(sx, d);
        sb += __shfl_xor(sb, d);
      }
      if (lane == 0) tred[w] = (f2_t){sx, sb};
      __syncthreads();
      if (tid == 0) {
        float tx = 0.f, tb = 0.f;
#pragma unroll
        for (int i = 0; i < WAVES; ++i) { tx += tred[i].x; tb += tred[i].y; }
        a.tsum[n] = (f2_t){tx, tb};
      }
      __syncthreads();
    }
  }
  store_x(0, 0);
  __syncthreads();
  if constexpr (XSETS == 3) {      // the tile of the second step
#pragma unroll
    for (int j = 0; j < XU; ++j) fetch_x(1, j);
    fetch_aux(1);
    advance_x();
  }

  Magic M;
  M.init();
  // one scale per row: four tiles of raw sums over all columns.  Grouped: the four tiles are started from zero
  // at every 128-column block, and `tot` holds the scaled sums.
  f16_t acc[4], tot[GROUPED ? 4 : 1];
  auto clear = [&](f16_t *v) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) v[i][r] = 0.f;
  };
  clear(acc);
  if constexpr (GROUPED) clear(tot);
  f16_t zero16;
#pragma unroll
  for (int r = 0; r < 16; ++r) zero16[r] = 0.f;
  auto flush = [&](const f16_t *v, int slot) {
    f4_t *dst = a.slots + (size_t)slot * SLOT_UNITS + (w * 16) * 64 + lane;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (NT == 1 && (i & 1)) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f4_t o = {v[i][4 * q], v[i][4 * q + 1], v[i][4 * q + 2], v[i][4 * q + 3]};
        dst[(i * 4 + q) * 64] = o;
      }
    }
  };
  // Grouped layers.  After the 8 k-steps of block h of a step one more matrix instruction per tile takes
  // sum c*x + z * sum x away: A = (-1 -1 -1 -zh -zh -zh -zl -zl | -zl 0 ...) of the lane's row in bf16
  // (zh + zl = z exactly, z being an fp16 number), B = the token's pieces staged with the step.  What is
  // left is sum (q - z) x of the block, and `tot += s * acc` (scale_in) follows: one fused multiply-add per
  // accumulator value.  (A second set of tiles, so that the scaling of one block could run under the matrix
  // instructions of the next, does not fit the registers: 512 and 61 to 88 spilled.)
  auto correct = [&](int h, int buf) __attribute__((always_inline)) {
    const float *zpl = reinterpret_cast<const float *>(lds + buf * BUF_UNITS + kUnitsPerTile) + (2 * h + 1) * ROWS;
    const u32x4 *bop = lds + buf * BUF_UNITS + kUnitsPerTile + SZ_UNITS + h * 128;
    const int kg = lane >> 5;
    u32x4 be[2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) be[nt] = bop[(nt * 32 + (lane & 31)) * 2 + kg];
#pragma unroll
    for (int rtl = 0; rtl < 2; ++rtl) {
      const float z = zpl[w * 64 + rtl * 32 + (lane & 31)];
      const u32 zh = __builtin_bit_cast(u32, z) & 0xffff0000u;
      const u32 zl = __builtin_bit_cast(u32, z - __builtin_bit_cast(float, zh)) & 0xffff0000u;
      const u32 nzh = zh ^ 0x80000000u, nzl = zl ^ 0x80000000u;
      const u32 m1 = 0xbf80u;                  // bf16 -1
      const u32x4 ae = kg == 0 ? (u32x4){m1 | (m1 << 16), m1 | nzh, (nzh >> 16) | nzh, (nzl >> 16) | nzl}
                               : (u32x4){nzl >> 16, 0u, 0u, 0u};
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[rtl * 2 + nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf8_t, ae), __builtin_bit_cast(bf8_t, be[nt]), acc[rtl * 2 + nt], 0, 0, 0);
    }
  };
  auto scale_in = [&](int h, int buf) __attribute__((always_inline)) {
    constexpr int kTot = GROUPED ? 1 : 0;
    const float *spl = reinterpret_cast<const float *>(lds + buf * BUF_UNITS + kUnitsPerTile) + 2 * h * ROWS;
#pragma unroll
    for (int rtl = 0; rtl < 2; ++rtl)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f4_t sc = *reinterpret_cast<const f4_t *>(spl + w * 64 + rtl * 32 + 8 * q + 4 * (lane >> 5));
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            tot[kTot * (rtl * 2 + nt)][4 * q + e] =
                __builtin_fmaf(sc[e], acc[rtl * 2 + nt][4 * q + e], tot[kTot * (rtl * 2 + nt)][4 * q + e]);
      }
  };

  int par = 0;
  // One column step out of code buffer J: 16 k-steps on the matrix cores with the loads of
  // the steps ahead spread between them, then the activations of the next step go to LDS.
  auto step = [&](auto slot_tag) __attribute__((always_inline)) {
    constexpr int J = decltype(slot_index(slot_tag))::value;
    u32 wd0[CH * 4], wd1[CH * 4];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      wd0[4 * c] = cb[J][0][c].x; wd0[4 * c + 1] = cb[J][0][c].y; wd0[4 * c + 2] = cb[J][0][c].z; wd0[4 * c + 3] = cb[J][0][c].w;
      wd1[4 * c] = cb[J][1][c].x; wd1[4 * c + 1] = cb[J][1][c].y; wd1[4 * c + 2] = cb[J][1][c].z; wd1[4 * c + 3] = cb[J][1][c].w;
    }
    auto between = [&](auto ks) __attribute__((always_inline)) {
      constexpr int S = decltype(kstep_index(ks))::value;
      constexpr int XF = XSETS == 3 ? (J + 2) % 3 : 0;         // set being fetched: step st + 2 or st + 1
      if constexpr (S < XU) fetch_x(XF, S);
      if constexpr (S >= 8 && S < 8 + 2 * CH) fetch_code((J + 2) % 3, (S - 8) / CH, (S - 8) % CH);   // codes of step st + 2
      if constexpr (S == 8 + 2 * CH - 1) advance_codes();
      if constexpr (S == XU - 1) { fetch_aux(XF); advance_x(); }
      if constexpr (GROUPED && (S == 7 || S == 15)) {
        correct(S >> 3, par);
        scale_in(S >> 3, par);
      }
    };
    KSteps<BITS, NT, GROUPED, 0>::run(wd0, wd1, lds + par * BUF_UNITS, lane, M, acc, zero16, between);
    const bool last_of_group = bp == a.nbp - 1;
    if (last_of_group || st == hi - 1) {
      if constexpr (GROUPED) {
        flush(tot, p + rg);
        clear(tot);
      } else {
        flush(acc, p + rg);
        clear(acc);
      }
    }
    // as selects of values: an `if` that increments one of the two gets turned into one increment through a
    // selected address, which puts both counters into scratch memory, and every wait for such a load is
    // a wait for all the loads of codes in flight
    rg += last_of_group ? 1 : 0;
    bp = last_of_group ? 0 : bp + 1;
    store_x(XSETS == 3 ? (J + 1) % 3 : 0, par ^ 1);
    __syncthreads();
    par ^= 1;
    ++st;
  };
  while (st + 3 <= hi) {
    step(Slot<0>{});
    step(Slot<1>{});
    step(Slot<2>{});
  }
  if (st < hi) step(Slot<0>{});
  if (st < hi) step(Slot<1>{});
}

// ---------------------------------------------------------------------------
// finish
// ---------------------------------------------------------------------------
struct FinishArgs {
  const f4_t *slots;
  const f2_t *tsum;      // [64]
  const u32 *sz;
  const u32x4 *weak_w;   // [d_out_pad][kp/8] units
  const u32x4 *xw;       // [64][kp/8] units
  _Float16 *y;           // [ntok][d_out] of this pass
  int nbp, d_out, d_out_pad, ntok, steps, grid, kp;
  int split;             // as in the main kernel
  int waves;             // waves per workgroup of the main kernel: a slot holds waves*64 rows
  // several tasks: token n uses weak_sets[task_id[n]] if that index is in [0, n_sets), else
  // the layer's own weak columns; task_id == nullptr: always its own
  const void *const *weak_sets;
  const int *task_id;    // of this pass
  int n_sets;
  int scaled;            // the partial results are already scaled (grouped layers)
};

// grid.x = row groups x waves of the main kernel: one workgroup per 64 rows (the part of a slot
// one wave of the main kernel wrote); wave i takes accumulator tile i = (row tile i >> 1,
// token tile i & 1).  grid.y = 2 (layers with few rows, more than 32 tokens): a workgroup per token
// tile as well, its waves sharing the row tiles as they do for 32 tokens or fewer.
__global__ __launch_bounds__(256) void owq_tile_finish(const FinishArgs a) {
  __shared__ _Float16 out[64][72];     // [token][row], padded pitch
  constexpr int kWeakPitch = 17;       // 16-byte units per staged row of a chunk of weak columns, odd
  __shared__ u32x4 wstage[2][64 * kWeakPitch];   // weak weights of the 64 rows, gathered activations of the 64 tokens
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = blockIdx.x / a.waves, w = blockIdx.x - rg * a.waves;
  const int row_base = (rg * a.waves + w) * 64;
  const size_t slot_units = (size_t)a.waves * 1024;
  // 64 tokens: wave = accumulator tile (row tile wv >> 1, token tile wv & 1), all four groups
  // of 8 rows; 32 tokens or fewer: two waves share a row tile, two groups of 8 rows each
  const bool per_tile = gridDim.y == 2;
  const bool two = a.ntok > 32 && !per_tile;
  const int i = two ? wv : (wv >> 1) * 2 + (per_tile ? (int)blockIdx.y : 0), nt = i & 1, rtl = i >> 1;
  const int q0 = two ? 0 : 2 * (wv & 1), qn = two ? 4 : 2;
  const int n = nt * 32 + (lane & 31);
  // product of the fp16 weak columns with the activations gathered at their indices
  f16_t wk;
#pragma unroll
  for (int r = 0; r < 16; ++r) wk[r] = 0.f;
  const int kunits = a.kp >> 3;
  if (kunits > 0) {
    int row = row_base + rtl * 32 + (lane & 31);
    if (row > a.d_out_pad - 1) row = a.d_out_pad - 1;
    const u32x4 *xsrc = a.xw + (size_t)n * kunits;
    const int kg = lane >> 5;
    // the set of weak columns of this lane's token: -1 = the layer's own, -2 = no token
    int mine = n < a.ntok ? -1 : -2;
    if (a.task_id != nullptr && n < a.ntok) {
      const int t = a.task_id[n];
      if ((u32)t < (u32)a.n_sets) mine = t;
    }
    typedef const __attribute__((address_space(1))) u32x4 *gptr_t;   // pointers read from memory: global
    constexpr int KS = 8;                            // K-steps whose loads are in flight together
    if (a.task_id == nullptr) {
      // One set, the layer's own.  A lane's operand is 16 bytes of its own row, so a wave reading operands
      // straight from memory touches 64 cache lines per load, and the address path takes a cycle for each
      // (4 of this kernel's 12 us).  Instead the workgroup copies the 64 rows x 16 units of a chunk of 8 K-steps
      // with loads that cover whole lines (a quarter wave per row), weights and gathered activations alike,
      // and the waves take their operands from LDS (odd pitch: no bank conflicts).
      const int cu = tid & 15, cr = tid >> 4;
      for (int s0 = 0; 2 * s0 < kunits; s0 += KS) {
        const int u = 2 * s0 + cu, uc = u < kunits ? u : 0;
        u32x4 ta[4], tb[4];
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          int r = row_base + cr + 16 * i4;
          if (r > a.d_out_pad - 1) r = a.d_out_pad - 1;
          ta[i4] = a.weak_w[(size_t)r * kunits + uc];
          tb[i4] = a.xw[(size_t)(cr + 16 * i4) * kunits + uc];
        }
        if (s0 > 0) __syncthreads();                 // the operands of the last chunk have been read
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const u32x4 zero = {0u, 0u, 0u, 0u};
          wstage[0][(cr + 16 * i4) * kWeakPitch + cu] = u < kunits ? ta[i4] : zero;
          wstage[1][(cr + 16 * i4) * kWeakPitch + cu] = (u < kunits && cr + 16 * i4 < a.ntok) ? tb[i4] : zero;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          if (2 * (s0 + j) >= kunits) continue;      // same for the whole workgroup
          const u32x4 av = wstage[0][(rtl * 32 + (lane & 31)) * kWeakPitch + 2 * j + kg];
          const u32x4 bw = wstage[1][n * kWeakPitch + 2 * j + kg];
          wk = mma(__builtin_bit_cast(h8_t, av), __builtin_bit_cast(h8_t, bw), wk);
        }
      }
    } else
    for (int s0 = 0; 2 * s0 < kunits; s0 += KS) {
      // the gathered activations of these K-steps are the same for every set: fetched once
      u32x4 bv[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        const int u = 2 * (s0 + j) + kg;
        bv[j] = xsrc[u < kunits ? u : 0];
        if (u >= kunits) bv[j] = (u32x4){0u, 0u, 0u, 0u};
      }
      // one pass per set that some token of the tile uses, in ascending order of the set index (at most
      // 33 passes however many sets the table holds): the least index still pending in the wave is next
      int pending = mine;
      for (;;) {
        int cand = pending >= -1 ? pending : 0x7fffffff;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) cand = min(cand, __shfl_xor(cand, d));
        const int t = __builtin_amdgcn_readfirstlane(cand);
        if (t == 0x7fffffff) break;
        if (pending == t) pending = -2;
        const gptr_t wbase = t < 0 ? (gptr_t)a.weak_w : (gptr_t)static_cast<const u32x4 *>(a.weak_sets[t]);
        const gptr_t wsrc = wbase + (size_t)row * kunits;
        const bool use = mine == t;
        u32x4 av[KS];
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          const int u = 2 * (s0 + j) + kg;
          av[j] = wsrc[u < kunits ? u : 0];
          if (u >= kunits) av[j] = (u32x4){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          if (2 * (s0 + j) >= kunits) continue;      // same for the whole wave
          const u32x4 zero = {0u, 0u, 0u, 0u};
          wk = mma(__builtin_bit_cast(h8_t, av[j]), __builtin_bit_cast(h8_t, use ? bv[j] : zero), wk);
        }
      }
    }
  }
  // owners of the first and the last step of this row group
  const long long st0 = (long long)rg * a.nbp, st1 = st0 + a.nbp - 1;
  int p_first, p_last;
  if (a.split > 0) {
    p_first = rg * a.split;
    p_last = p_first + a.split - 1;
  } else {
    p_first = (int)(((st0 + 1) * a.grid - 1) / a.steps);
    p_last = (int)(((st1 + 1) * a.grid - 1) / a.steps);
  }
  f2_t t = {0.f, 0.f};
  if (!a.scaled) t = a.tsum[n];
  f4_t sum[4];
#pragma unroll
  for (int qq = 0; qq < 4; ++qq) sum[qq] = (f4_t){0.f, 0.f, 0.f, 0.f};
  const f4_t *src = a.slots + (size_t)((w * 4 + i) * 4 + q0) * 64 + lane;
  constexpr int kInFlight = 4;                       // partial results fetched together (x up to 4 row groups)
  for (int p = p_first; p <= p_last; p += kInFlight) {     // fixed order of additions
    f4_t v[kInFlight][4];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      if (p + j > p_last) continue;                 // same for the whole workgroup
#pragma unroll
      for (int qq = 0; qq < 4; ++qq)
        if (qq < qn) v[j][qq] = src[(size_t)(p + j + rg) * slot_units + qq * 64];
    }
#pragma unroll
    for (int j = 0; j < kInFlight; ++j)
      if (p + j <= p_last) {
#pragma unroll
        for (int qq = 0; qq < 4; ++qq)
          if (qq < qn) sum[qq] += v[j][qq];
      }
  }
#pragma unroll
  for (int qq = 0; qq < 4; ++qq) {
    if (qq >= qn) continue;
    const int q = q0 + qq;
    const int r0 = rtl * 32 + 8 * q + 4 * (lane >> 5);      // row within the workgroup's 64
    f4_t sm = sum[qq];
    if (!a.scaled) {
      int row = row_base + r0;
      if (row > a.d_out_pad - 4) row = a.d_out_pad - 4;
      const u32x4 szw = *reinterpret_cast<const u32x4 *>(a.sz + row);
      const u32 s4[4] = {szw.x, szw.y, szw.z, szw.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float v = sm[e] - t.y;
        v = __builtin_fmaf(-half_hi(s4[e]), t.x, v);
        sm[e] = v * half_lo(s4[e]);
      }
    }
    // wk[4q + e] with q known only at run time: pick by comparison, no indexed register file access
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float wv4 = 0.f;
#pragma unroll
      for (int qs = 0; qs < 4; ++qs)
        if (qs == q) wv4 = wk[4 * qs + e];
      out[n][r0 + e] = (_Float16)(sm[e] + wv4);
    }
  }
  __syncthreads();
  const int n_lo = per_tile ? 32 * (int)blockIdx.y : 0, n_hi = per_tile ? min(a.ntok, n_lo + 32) : a.ntok;
  for (int e = tid; e < (n_hi - n_lo) * 64; e += 256) {
    const int nn = n_lo + (e >> 6), r = e & 63;
    if (row_base + r < a.d_out) a.y[(size_t)nn * a.d_out + row_base + r] = out[nn][r];
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
typedef void (*mma_fn)(const TileArgs);

template <int BITS, int WAVES>
static mma_fn pick_mma2(int nt, bool grouped) {
  if constexpr (WAVES == 4) {      // grouped layers: four waves only (their twelve accumulator tiles need a SIMD's registers)
    if (grouped) return nt == 2 ? owq_tile_mma<BITS, 2, true, 4> : owq_tile_mma<BITS, 1, true, 4>;
  } else {
    if (grouped) return nullptr;
  }
  return nt == 2 ? owq_tile_mma<BITS, 2, false, WAVES> : owq_tile_mma<BITS, 1, false, WAVES>;
}

static mma_fn pick_mma(int bits, int nt, bool grouped, int waves) {
  if (bits == 3) return waves == 8 ? pick_mma2<3, 8>(nt, grouped) : pick_mma2<3, 4>(nt, grouped);
  return waves == 8 ? pick_mma2<4, 8>(nt, grouped) : pick_mma2<4, 4>(nt, grouped);
}

static int32_t tile_lds_bytes(bool grouped, int waves) {
  return 2 * (kUnitsPerTile + (grouped ? waves * 64 + 256 : 0)) * 16;
}

// Grouped layers stage scales and sums next to the activations: more than the 64 KiB of LDS a
// kernel may use without asking.  Returns a hipError_t as int.
int prepare_tile_kernels(const owq_layer_info_t &g, int32_t lds_limit) {
  if (g.n_groups <= 1) return (int)hipSuccess;
  for (int waves = 4; waves <= 4; waves += 4) {
    const int32_t need = tile_lds_bytes(true, waves);
    if (need > lds_limit) return (int)hipErrorInvalidValue;
    for (int nt = 1; nt <= 2; ++nt) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_mma(g.bits, nt, true, waves)),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, need);
      if (e != hipSuccess) return (int)e;
    }
  }
  return (int)hipSuccess;
}

// Most workgroups the partial-result slots of the scratch area allow for `waves` per workgroup.
int32_t tile_grid_limit(const owq_layer_info_t &g, int32_t waves, uint64_t scratch_bytes) {
  const TileScratch ts = tile_scratch(g);
  const uint64_t total = scratch_bytes ? scratch_bytes : ts.total;
  if (total < ts.off_slots) return 0;
  const int64_t slot = (int64_t)waves * 16384;
  const int64_t n_rg = (g.n_rt + 2 * waves - 1) / (2 * waves);
  const int64_t room = (int64_t)(total - ts.off_slots) / slot - n_rg;
  const int64_t steps = n_rg * g.nbp;
  int64_t lim = room < steps ? room : steps;
  const int64_t cap = waves == 8 ? kTileGridMax / 2 : kTileGridMax;
  if (lim > cap) lim = cap;
  return lim < 0 ? 0 : (int32_t)lim;
}

// Default work split: ranges aligned to row groups (fewer partial results, and the workgroups
// of a range use the same activation tile at the same time, which keeps it in L2) unless that
// costs more than a tenth in steps per workgroup against equal ranges of the whole sequence.
void tile_default_shape(const owq_layer_info_t &g, int32_t waves, int32_t *grid, int32_t *split, uint64_t scratch_bytes) {
  const int32_t limit = tile_grid_limit(g, waves, scratch_bytes);
  // One workgroup per compute unit.  Two of four waves (which the registers allow for layers with one scale per
  // row) are no faster per step, as the matrix cores and the memory stream take turns rather than overlap on
  // this machine, and twice the workgroups write twice the partial results: 256 against 512 workgroups at 64
  // tokens measured 30.2 / 36.1 us on a 16384 x 4096 layer, 50.0 / 56.5 us on 28672 x 8192, 62.3 / 64.0 us on
  // 9216 x 36864.
  int32_t cap = kTileGridMax / 2;
  if (cap > limit) cap = limit;
  const int64_t n_rg = (g.n_rt + 2 * waves - 1) / (2 * waves);
  const int64_t steps = n_rg * g.nbp;
  *grid = cap;
  *split = 0;
  if (cap < 1) return;
  int64_t sa = cap / n_rg;
  if (sa > g.nbp) sa = g.nbp;
  if (sa >= 1) {
    const int64_t aligned = (g.nbp + sa - 1) / sa, equal = (steps + cap - 1) / cap;
    if (aligned * 10 <= equal * 11) {
      *grid = (int32_t)(n_rg * sa);
      *split = (int32_t)sa;
    }
  }
}

int launch_tile(const owq_layer_info_t &g, void *blob, void *scratch, uint64_t scratch_bytes, int32_t grid, int32_t split,
                int32_t waves, int32_t small_split, const TaskSets &tasks, const void *x, void *y, int32_t batch,
                void *stream) {
  const TileScratch ts = tile_scratch(g);
  uint8_t *base = static_cast<uint8_t *>(blob);
  uint8_t *scr = scratch ? static_cast<uint8_t *>(scratch) : base + g.off_scratch;
  const uint64_t scr_bytes = scratch ? scratch_bytes : ts.total;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool grouped = g.n_groups > 1;
  if (waves != 4 && waves != 8) return (int)hipErrorInvalidValue;
  if (grouped && waves != 4) return (int)hipErrorInvalidValue;
  if (grid < 1 || grid > tile_grid_limit(g, waves, scr_bytes)) return (int)hipErrorInvalidValue;
  const int n_rg = (g.n_rt + 2 * waves - 1) / (2 * waves);
  if (split < 0 || split > g.nbp || (split > 0 && grid != n_rg * split)) return (int)hipErrorInvalidValue;

  StageArgs sa;
  sa.wmask = base + g.off_wmask;
  sa.weak_idx = reinterpret_cast<const int *>(base + g.off_weak_idx);
  sa.xs = reinterpret_cast<u32x4 *>(scr + ts.off_xs);
  sa.bsum = reinterpret_cast<f2_t *>(scr + ts.off_bsum);
  sa.xw = reinterpret_cast<_Float16 *>(scr + ts.off_xw);
  sa.d_in = g.d_in; sa.nblk = g.nblk; sa.kp = g.kp;

  TileArgs ta;
  ta.codes = reinterpret_cast<const u32x4 *>(base + g.off_codes);
  ta.sz = reinterpret_cast<const u32 *>(base + g.off_sz);
  ta.xs = sa.xs;
  ta.bsum = sa.bsum;
  ta.tsum = reinterpret_cast<f2_t *>(scr + ts.off_tsum);
  ta.slots = reinterpret_cast<f4_t *>(scr + ts.off_slots);
  ta.nbp = g.nbp; ta.n_rt = g.n_rt; ta.n_groups = g.n_groups; ta.nblk = g.nblk; ta.d_out_pad = g.d_out_pad;
  ta.bpg = g.group_size ? g.group_size / kBlockCols : g.nblk;
  ta.steps = n_rg * g.nbp;
  ta.split = split;

  FinishArgs fa;
  fa.slots = ta.slots;
  fa.tsum = ta.tsum;
  fa.sz = ta.sz;
  fa.weak_w = reinterpret_cast<const u32x4 *>(base + g.off_weak_w);
  fa.xw = reinterpret_cast<const u32x4 *>(sa.xw);
  fa.nbp = g.nbp; fa.d_out = g.d_out; fa.d_out_pad = g.d_out_pad;
  fa.steps = ta.steps; fa.grid = grid; fa.kp = g.kp; fa.waves = waves; fa.split = split;
  fa.scaled = grouped ? 1 : 0;
  fa.weak_sets = tasks.weak_sets; fa.n_sets = tasks.n_sets;

  const _Float16 *xp = static_cast<const _Float16 *>(x);
  _Float16 *yp = static_cast<_Float16 *>(y);
  for (int32_t t0 = 0; t0 < batch; t0 += kScratchBatch) {
    const int ntok = batch - t0 < kScratchBatch ? batch - t0 : kScratchBatch;
    const int nt = ntok > 32 ? 2 : 1;
    if (ntok <= 32 && small_split >= 0 && tasks.task_id == nullptr) {   // few tokens, one task: one launch
      const int r = launch_tile_small(g, blob, scr + ts.off_slots, scr_bytes - ts.off_slots, small_split,
                                      xp + (size_t)t0 * g.d_in, yp + (size_t)t0 * g.d_out, ntok, stream);
      if (r > 0 || r == -2) return r;
      if (r == 0) continue;
    }
    sa.x = xp + (size_t)t0 * g.d_in;
    sa.ntok = ntok;
    if (g.bits == 3)
      hipLaunchKernelGGL(owq_tile_stage<3>, dim3((unsigned)g.nbp, (unsigned)nt, 1), dim3(256, 1, 1), 0, st, sa);
    else
      hipLaunchKernelGGL(owq_tile_stage<4>, dim3((unsigned)g.nbp, (unsigned)nt, 1), dim3(256, 1, 1), 0, st, sa);
    hipLaunchKernelGGL(pick_mma(g.bits, nt, grouped, waves), dim3((unsigned)grid, 1, 1), dim3((unsigned)(waves * 64), 1, 1),
                       tile_lds_bytes(grouped, waves), st, ta);
    fa.y = yp + (size_t)t0 * g.d_out;
    fa.ntok = ntok;
    fa.task_id = tasks.task_id ? tasks.task_id + t0 : nullptr;
    // few rows: one workgroup per (64 rows, token tile), so that the launch fills more of the chip
    const unsigned per_tile = (ntok > 32 && n_rg * waves <= 384) ? 2u : 1u;
    hipLaunchKernelGGL(owq_tile_finish, dim3((unsigned)(n_rg * waves), per_tile, 1), dim3(256, 1, 1), 0, st, fa);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return (int)hipSuccess;
}

// The library's own scratch memory for callers that can pass no workspace and whose blobs may
// not be written to: one array per GPU, held until the process ends.  The symbol below is a
// host-side stand-in; its device address is looked up once per device (hipGetSymbolAddress)
// and only that address is handed to kernels.
static __device__ __align__(256) unsigned char g_static_scratch[OWQ_STATIC_SCRATCH_BYTES];

int static_scratch(void **ptr) {
  constexpr int kMaxDevices = 64;
  static void *addr[kMaxDevices];
  static std::mutex lock;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(lock);
  if (!addr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return (int)hipSuccess;
}

}  // namespace owq
