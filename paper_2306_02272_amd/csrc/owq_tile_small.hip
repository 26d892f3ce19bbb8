// Tile layout, 32 tokens or fewer: the whole layer in one launch on the matrix cores of
// gfx950 (two when the columns of a row tile are split over several workgroups).
//
// Same result as the other kernels (paper: storage paragraph of "Outlier-Aware Weight
// Quantization", section "Acceleration on Real Device"):
//     y[n,i] = sum_{j not weak} s_ig (q_ij - z_ig) x[n,j]  +  sum_t Ww_it x[n, idx_t]
//
// With few tokens the layer is bound by its weight stream and by latency, so nothing is
// staged through memory first.  A workgroup of four waves owns one tile of 32 rows and a
// range of blocks of 128 columns; every wave takes a quarter of the range and streams it on
// its own: codes go from registers straight into the A operand (a pair of codes is masked out
// of a dword and OR-ed into the mantissas of 2^(10-o), giving 2^(10-o)+q exactly), the
// activations come straight from x as the B operand (lane = token, eight consecutive
// columns; the weak columns are cleared by select on the way).  A second matrix instruction
// per k-step, whose A operand holds a row of ones and a row of the constants 2^(10-o),
// yields per token sum x and sum 2^(10-o) x of the block in the same lanes as the
// products, so that  tot += s (acc - sum c x - z sum x)  can follow every block.  The product
// of the fp16 weak columns with the activations gathered at their indices is a few more
// k-steps into the same accumulators.  The four waves add their results through LDS in a
// fixed order; with more than one column range per row tile the sums go to memory and a
// second small kernel adds them, again in a fixed order.  No atomics.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "owq_internal.h"
#include "owq_tile_device.h"

namespace owq {

typedef u32 u32x2 __attribute__((ext_vector_type(2)));

struct SmallArgs {
  const u32x4 *codes;
  const u32 *sz;               // [n_groups][d_out_pad]: fp16 scale | fp16 zero << 16
  const unsigned char *wmask;  // bit e of byte i: column 8i+e is weak
  const int *weak_idx;         // [kp], padding -1
  const u32x4 *weak_w;         // [d_out_pad][kp/8] units
  const _Float16 *x;           // [ntok][d_in], 16-byte aligned, d_in a multiple of 128
  _Float16 *y;                 // [ntok][d_out]
  float *part;                 // split > 1: [split][32][d_out_pad]
  int d_in, d_out, d_out_pad, ntok, nbp, nblk, bpg, kp, split;
};

template <int J> struct Buf {};   // tag: register buffer J of the blocks in flight
template <int J> __device__ std::integral_constant<int, J> buf_index(Buf<J>);

constexpr int kSmallWaves = 4;
constexpr int kSmallSzUnits = 4;      // 16-byte units of scales a thread stages: 128 groups per workgroup
constexpr int kSmallRedUnits = 1024;  // LDS units of the waves' results: [4][16][64] floats

template <int BITS, bool GROUPED>
__global__ __launch_bounds__(256, 2) void owq_tile_small(const SmallArgs a) {
  constexpr int CH = BITS == 3 ? 3 : 4;
  constexpr int NB = 2;                   // blocks in flight per wave; refilled register by register as they are used
  constexpr int WK = GROUPED ? 2 : 3;     // k-steps of weak columns a wave fetches ahead of its blocks (registers decide)
  extern __shared__ u32x4 lds[];
  float *red = reinterpret_cast<float *>(lds);
  f2_t *szl = reinterpret_cast<f2_t *>(lds + kSmallRedUnits);   // [groups of the workgroup][32 rows] (scale, zero)

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, kg = lane >> 5;
  const int rt = blockIdx.x / a.split, sp = blockIdx.x - rt * a.split;
  const int b0 = (int)((long long)a.nblk * sp / a.split), b1 = (int)((long long)a.nblk * (sp + 1) / a.split);
  const int nbw = b1 - b0;                                      // >= 1: split <= nblk
  const int wb0 = b0 + nbw * w / kSmallWaves, wb1 = b0 + nbw * (w + 1) / kSmallWaves;
  const int g_lo = GROUPED ? b0 / a.bpg : 0;
  const int ng = GROUPED ? (b1 - 1) / a.bpg - g_lo + 1 : 1;
  u32x4 *wml = lds + kSmallRedUnits + ng * 16;                  // [blocks of the workgroup] 16 bytes of weak mask
  const int n_c = n < a.ntok ? n : 0;                           // lanes without a token re-read token 0; never stored
  const _Float16 *xrow = a.x + (size_t)n_c * a.d_in;

  // ---- (1) what the set-up needs: scales, weak masks, weak indices -------------------
  // Issued before the weight stream: loads complete in order, so waiting for these does not
  // wait for the weights behind them.  No branches: reads past the end are clamped and dropped.
  u32x4 szv[kSmallSzUnits];
#pragma unroll
  for (int j = 0; j < kSmallSzUnits; ++j) {
    const int i = tid + 256 * j, ic = i < ng * 8 ? i : 0;
    szv[j] = *reinterpret_cast<const u32x4 *>(a.sz + (size_t)(g_lo + (ic >> 3)) * a.d_out_pad + rt * 32 + (ic & 7) * 4);
  }
  const u32x4 wmv = *reinterpret_cast<const u32x4 *>(a.wmask + (size_t)(b0 + (tid < nbw ? tid : 0)) * 16);
  // weak columns: the k-steps are dealt out to all waves of the row tile's workgroups; the first
  // WK of a wave ride ahead of its blocks
  const int kunits = a.kp >> 3, ksteps = (kunits + 1) >> 1;
  const bool weak_here = kunits > 0;
  const int wslot = sp * kSmallWaves + w, wstride = a.split * kSmallWaves;
  int widx[WK][8];
#pragma unroll
  for (int i = 0; i < WK; ++i) {
    const int s = wslot + wstride * i;
    const int u = 2 * s + kg, uc = (weak_here && u < kunits) ? u : 0;
    const u32x4 *ip = reinterpret_cast<const u32x4 *>(a.weak_idx + 8 * uc);
    const u32x4 lo = ip[0], hi = ip[1];
    widx[i][0] = (int)lo.x; widx[i][1] = (int)lo.y; widx[i][2] = (int)lo.z; widx[i][3] = (int)lo.w;
    widx[i][4] = (int)hi.x; widx[i][5] = (int)hi.y; widx[i][6] = (int)hi.z; widx[i][7] = (int)hi.w;
  }

  // ---- (2) the weight stream: NB blocks in flight per wave ----------------------------
  u32x4 cA[NB];
  u32x4 cB[NB];      // 4-bit: second chunk; 3-bit: .xy = the block's half of the middle chunk
  u32x4 xb[NB][8];
  // Past the wave's range the loads still go out (to a block that exists) and are dropped: the
  // number of loads in flight is the same on every path.
  auto fetch_codes = [&](auto tag, int b) __attribute__((always_inline)) {
    constexpr int J = decltype(buf_index(tag))::value;
    const int bc = b < wb1 ? b : b0;
    const int bp = bc >> 1, h = bc & 1;
    const u32x4 *t = a.codes + (size_t)(rt * a.nbp + bp) * CH * 64 + lane;
    cA[J] = __builtin_nontemporal_load(t + 2 * h * 64);
    if (BITS == 4) {
      cB[J] = __builtin_nontemporal_load(t + (2 * h + 1) * 64);
    } else {
      const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(t + 64) + h);
      cB[J].x = v.x; cB[J].y = v.y;
    }
  };
  auto fetch_x = [&](auto tag, auto ks, int b) __attribute__((always_inline)) {
    constexpr int J = decltype(buf_index(tag))::value;
    constexpr int S = decltype(buf_index(ks))::value;
    const int bc = b < wb1 ? b : b0;
    xb[J][S] = *reinterpret_cast<const u32x4 *>(xrow + bc * 128 + 8 * kg + 16 * S);
  };
  auto fetch = [&](auto tag, int b) __attribute__((always_inline)) {
    fetch_x(tag, Buf<0>{}, b); fetch_x(tag, Buf<1>{}, b); fetch_x(tag, Buf<2>{}, b); fetch_x(tag, Buf<3>{}, b);
    fetch_x(tag, Buf<4>{}, b); fetch_x(tag, Buf<5>{}, b); fetch_x(tag, Buf<6>{}, b); fetch_x(tag, Buf<7>{}, b);
    fetch_codes(tag, b);
  };
  fetch(Buf<0>{}, wb0);
  fetch(Buf<1>{}, wb0 + 1);
  if constexpr (NB == 3) fetch(Buf<2>{}, wb0 + 2);

  // ---- (3) set-up data to LDS; gathers of the weak columns ------------------------------
#pragma unroll
  for (int j = 0; j < kSmallSzUnits; ++j) {
    const int i = tid + 256 * j;
    if (i < ng * 8) {
      const u32 d[4] = {szv[j].x, szv[j].y, szv[j].z, szv[j].w};
      f4_t *dst = reinterpret_cast<f4_t *>(szl + i * 4);
      dst[0] = (f4_t){half_lo(d[0]), half_hi(d[0]), half_lo(d[1]), half_hi(d[1])};
      dst[1] = (f4_t){half_lo(d[2]), half_hi(d[2]), half_lo(d[3]), half_hi(d[3])};
    }
  }
  if (tid < nbw) wml[tid] = wmv;
  u32x4 wa[WK];
  h8_t wg[WK];
  u32 wok[WK];       // bit e: element e of the k-step is a real weak column
#pragma unroll
  for (int i = 0; i < WK; ++i) {
    const int s = wslot + wstride * i;
    const int u = 2 * s + kg, uc = (weak_here && u < kunits) ? u : 0;
    wa[i] = a.weak_w[(size_t)(rt * 32 + n) * kunits + uc];
    wok[i] = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int j = widx[i][e];
      const bool ok = (u32)j < (u32)a.d_in;
      wg[i][e] = xrow[ok ? j : 0];
      wok[i] |= ok ? (1u << e) : 0u;
    }
  }
  __syncthreads();

  // ---- (4) the wave's blocks ------------------------------------------------------------
  Magic M;
  M.init();
  // A operand of the second instruction: rows 0 and 4 ones, rows 1 and 5 the constants
  u32 cxm[8];
#pragma unroll
  for (int o = 0; o < 8; ++o) {
    const int cls = n < 8 ? (n & 3) : 3;
    cxm[o] = cls == 0 ? kOnes : (cls == 1 ? M.m[o] : 0u);
  }
  f16_t acc, accx, tot;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[r] = 0.f; accx[r] = 0.f; tot[r] = 0.f; }
  const f16_t zero16 = tot;
  int b = wb0;
  int gi = GROUPED ? wb0 / a.bpg - g_lo : 0, gpos = GROUPED ? wb0 % a.bpg : 0;

  auto scale_in = [&](int g) __attribute__((always_inline)) {
    // tot += s * (acc - sum c*x - z * sum x) with the staged (scale, zero) of group g
    const float X = accx[0], Bc = accx[1];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f4_t *src = reinterpret_cast<const f4_t *>(szl + g * 32 + 8 * q + 4 * kg);
      const f4_t s01 = src[0], s23 = src[1];
      const float sc[4] = {s01[0], s01[2], s23[0], s23[2]}, zp[4] = {s01[1], s01[3], s23[1], s23[3]};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float v = acc[4 * q + e] - Bc;
        v = __builtin_fmaf(-zp[e], X, v);
        tot[4 * q + e] = __builtin_fmaf(sc[e], v, tot[4 * q + e]);
      }
    }
  };

  auto step = [&](auto tag) __attribute__((always_inline)) {
    constexpr int J = decltype(buf_index(tag))::value;
    u32 wd[8];
    if (BITS == 4) {
      wd[0] = cA[J].x; wd[1] = cA[J].y; wd[2] = cA[J].z; wd[3] = cA[J].w;
      wd[4] = cB[J].x; wd[5] = cB[J].y; wd[6] = cB[J].z; wd[7] = cB[J].w;
    } else {
      const bool h = b & 1;     // first half: chunk 0 then .xy of chunk 1; second half: .zw of chunk 1 then chunk 2
      wd[0] = h ? cB[J].x : cA[J].x; wd[1] = h ? cB[J].y : cA[J].y;
      wd[2] = h ? cA[J].x : cA[J].z; wd[3] = h ? cA[J].y : cA[J].w;
      wd[4] = h ? cA[J].z : cB[J].x; wd[5] = h ? cA[J].w : cB[J].y;
    }
    const u32x4 wm = wml[b - b0];
    const u32 wms[4] = {(u32)__builtin_amdgcn_readfirstlane((int)wm.x), (u32)__builtin_amdgcn_readfirstlane((int)wm.y),
                        (u32)__builtin_amdgcn_readfirstlane((int)wm.z), (u32)__builtin_amdgcn_readfirstlane((int)wm.w)};
    auto kstep = [&](auto ks) __attribute__((always_inline)) {
      constexpr int S = decltype(buf_index(ks))::value;
      u32x4 xv = xb[J][S];
      const u32 m16 = (wms[S >> 1] >> (16 * (S & 1))) & 0xffffu;     // same for the whole wave
      if (m16 != 0u) {
        const u32 m = (m16 >> (8 * kg)) & 0xffu;
        // weak columns contribute nothing to the dense term
        if (m & 0x01u) xv.x &= 0xffff0000u;
        if (m & 0x02u) xv.x &= 0x0000ffffu;
        if (m & 0x04u) xv.y &= 0xffff0000u;
        if (m & 0x08u) xv.y &= 0x0000ffffu;
        if (m & 0x10u) xv.z &= 0xffff0000u;
        if (m & 0x20u) xv.z &= 0x0000ffffu;
        if (m & 0x40u) xv.w &= 0xffff0000u;
        if (m & 0x80u) xv.w &= 0x0000ffffu;
      }
      const h8_t bo = __builtin_bit_cast(h8_t, xv);
      const h8_t ao = a_operand<BITS, S>(wd, M);
      const u32x4 cx = {cxm[pair_offset(BITS, S, 0)], cxm[pair_offset(BITS, S, 1)], cxm[pair_offset(BITS, S, 2)],
                        cxm[pair_offset(BITS, S, 3)]};
      const bool fresh = GROUPED && S == 0;
      acc = mma(ao, bo, fresh ? zero16 : acc);
      accx = mma(__builtin_bit_cast(h8_t, cx), bo, fresh ? zero16 : accx);
      fetch_x(tag, ks, b + NB);                // the register is free: refill it for the block NB ahead
    };
    kstep(Buf<0>{}); kstep(Buf<1>{}); kstep(Buf<2>{}); kstep(Buf<3>{});
    kstep(Buf<4>{}); kstep(Buf<5>{}); kstep(Buf<6>{}); kstep(Buf<7>{});
    if (GROUPED) {
      scale_in(gi);
      if (++gpos == a.bpg) { gpos = 0; ++gi; }
    }
    fetch_codes(tag, b + NB);
    ++b;
  };
  while (b + NB <= wb1) {
    step(Buf<0>{});
    step(Buf<1>{});
    if constexpr (NB == 3) step(Buf<2>{});
  }
  if (b < wb1) step(Buf<0>{});
  if constexpr (NB == 3) {
    if (b < wb1) step(Buf<1>{});
  }
  if (!GROUPED) scale_in(0);

  // ---- (5) weak columns -----------------------------------------------------------------
  if (weak_here) {
    const u32x4 z4 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < WK; ++i) {
      const int s = wslot + wstride * i;
      if (s < ksteps) {                        // same for the whole wave
        const bool uv = 2 * s + kg < kunits;
        h8_t bo;
#pragma unroll
        for (int e = 0; e < 8; ++e) bo[e] = (uv && ((wok[i] >> e) & 1u)) ? wg[i][e] : (_Float16)0;
        tot = mma(__builtin_bit_cast(h8_t, uv ? wa[i] : z4), bo, tot);
      }
    }
    for (int s = wslot + wstride * WK; s < ksteps; s += wstride) {    // many weak columns: no longer ahead
      const int u = 2 * s + kg;
      const bool uv = u < kunits;
      const int uc = uv ? u : 0;
      const u32x4 av = a.weak_w[(size_t)(rt * 32 + n) * kunits + uc];
      h8_t bo;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int j = a.weak_idx[8 * uc + e];
        const _Float16 v = xrow[(u32)j < (u32)a.d_in ? j : 0];
        bo[e] = (uv && (u32)j < (u32)a.d_in) ? v : (_Float16)0;
      }
      tot = mma(__builtin_bit_cast(h8_t, uv ? av : z4), bo, tot);
    }
  }

  // ---- (6) the four waves' results, added in a fixed order ----------------------------
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(w * 16 + r) * 64 + lane] = tot[r];
  __syncthreads();
  for (int e = tid; e < a.ntok * 32; e += 256) {
    const int nn = e >> 5, row = e & 31;
    const int r = 4 * (row >> 3) + (row & 3), ln = nn + 32 * ((row >> 2) & 1);
    const float v = ((red[(0 * 16 + r) * 64 + ln] + red[(1 * 16 + r) * 64 + ln]) + red[(2 * 16 + r) * 64 + ln]) +
                    red[(3 * 16 + r) * 64 + ln];
    const int grow = rt * 32 + row;
    if (a.split == 1) {
      if (grow < a.d_out) a.y[(size_t)nn * a.d_out + grow] = (_Float16)v;
    } else {
      a.part[(size_t)(sp * 32 + nn) * a.d_out_pad + grow] = v;
    }
  }
}

// Adds the results of the column ranges of every row (fixed order) and rounds to fp16.
__global__ __launch_bounds__(256) void owq_tile_small_sum(const float *part, _Float16 *y, int split, int ntok, int d_out,
                                                          int d_out_pad) {
  const int row = blockIdx.x * 256 + threadIdx.x, nn = blockIdx.y;
  if (row >= d_out || nn >= ntok) return;
  float v = 0.f;
  for (int s = 0; s < split; ++s) v += part[(size_t)(s * 32 + nn) * d_out_pad + row];
  y[(size_t)nn * d_out + row] = (_Float16)v;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
typedef void (*small_fn)(const SmallArgs);

static small_fn pick_small(int bits, bool grouped) {
  if (bits == 3) return grouped ? owq_tile_small<3, true> : owq_tile_small<3, false>;
  return grouped ? owq_tile_small<4, true> : owq_tile_small<4, false>;
}

static int real_blocks(const owq_layer_info_t &g) { return (g.d_in + kBlockCols - 1) / kBlockCols; }

// LDS bytes of the small-batch kernel with `split` column ranges per row tile; 0 = that split
// does not fit the kernel's staging (groups or blocks per workgroup) or the room for partial sums.
static int32_t small_lds_bytes(const owq_layer_info_t &g, int32_t split) {
  const int nblk = real_blocks(g);
  if (split < 1 || split > nblk) return 0;
  const int bpg = g.group_size ? g.group_size / kBlockCols : nblk;
  int ng_max = 1, nbw_max = 1;
  for (int sp = 0; sp < split; ++sp) {
    const int b0 = (int)((int64_t)nblk * sp / split), b1 = (int)((int64_t)nblk * (sp + 1) / split);
    const int ng = g.n_groups > 1 ? (b1 - 1) / bpg - b0 / bpg + 1 : 1;
    if (ng > ng_max) ng_max = ng;
    if (b1 - b0 > nbw_max) nbw_max = b1 - b0;
  }
  if (ng_max > kSmallSzUnits * 256 / 8 || nbw_max > 256) return 0;
  if (split > 1) {
    const TileScratch ts = tile_scratch(g);
    if ((uint64_t)split * 32 * g.d_out_pad * 4 > ts.total - ts.off_slots) return 0;
  }
  return (kSmallRedUnits + ng_max * 16 + nbw_max) * 16;
}

// Column ranges per row tile when the caller does not say: as few as fill the chip's 512
// places for workgroups of four waves, weighing a workgroup's fixed cost (its first loads,
// the set-up, the last sums) and the second launch against the blocks each wave streams.
static int32_t small_default_split(const owq_layer_info_t &g) {
  const int nblk = real_blocks(g);
  double best = 0.0;
  int32_t pick = 0;
  for (int32_t s = 1; s <= 16 && s <= nblk; ++s) {
    if (small_lds_bytes(g, s) == 0 || small_lds_bytes(g, s) > 65536) continue;
    const double wgs = (double)g.n_rt * s;
    const double rounds = wgs <= 512.0 ? 1.0 : wgs / 512.0;
    const double per_wave = (double)((nblk + s - 1) / s + kSmallWaves - 1) / kSmallWaves;
    const double cost = rounds * (per_wave + 6.0) + (s > 1 ? 6.0 : 0.0);
    if (pick == 0 || cost < best) { best = cost; pick = s; }
  }
  return pick;
}

bool tile_small_split_ok(const owq_layer_info_t &g, int32_t split) {
  const int32_t lds = small_lds_bytes(g, split);
  return lds > 0 && lds <= 65536;
}

// One pass of up to 32 tokens.  split = 0: the default.  Returns a hipError_t as int, or -1 when
// this layer (or this call's x) does not fit the kernel and the caller has to take the
// three-launch path.
int launch_tile_small(const owq_layer_info_t &g, void *blob, int32_t split, const void *x, void *y, int32_t ntok,
                      void *stream) {
  if (ntok < 1 || ntok > 32) return -1;
  if ((reinterpret_cast<uintptr_t>(x) & 15) != 0 || g.d_in % kBlockCols != 0) return -1;   // whole blocks, aligned rows
  if (split == 0) split = small_default_split(g);
  if (split < 1 || !tile_small_split_ok(g, split)) return -1;
  const TileScratch ts = tile_scratch(g);
  uint8_t *base = static_cast<uint8_t *>(blob);
  SmallArgs a;
  a.codes = reinterpret_cast<const u32x4 *>(base + g.off_codes);
  a.sz = reinterpret_cast<const u32 *>(base + g.off_sz);
  a.wmask = base + g.off_wmask;
  a.weak_idx = reinterpret_cast<const int *>(base + g.off_weak_idx);
  a.weak_w = reinterpret_cast<const u32x4 *>(base + g.off_weak_w);
  a.x = static_cast<const _Float16 *>(x);
  a.y = static_cast<_Float16 *>(y);
  a.part = reinterpret_cast<float *>(base + g.off_scratch + ts.off_slots);
  a.d_in = g.d_in; a.d_out = g.d_out; a.d_out_pad = g.d_out_pad; a.ntok = ntok; a.nbp = g.nbp;
  a.nblk = real_blocks(g);
  a.bpg = g.group_size ? g.group_size / kBlockCols : a.nblk;
  a.kp = g.kp; a.split = split;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(pick_small(g.bits, g.n_groups > 1), dim3((unsigned)(g.n_rt * split), 1, 1), dim3(256, 1, 1),
                     (size_t)small_lds_bytes(g, split), st, a);
  if (split > 1)
    hipLaunchKernelGGL(owq_tile_small_sum, dim3((unsigned)((g.d_out + 255) / 256), (unsigned)ntok, 1), dim3(256, 1, 1), 0, st,
                       a.part, a.y, split, ntok, g.d_out, g.d_out_pad);
  return (int)hipGetLastError();
}

}  // namespace owq
