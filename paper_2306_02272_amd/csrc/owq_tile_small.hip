// Tile layout, 32 tokens or fewer: the whole layer in one launch on the matrix cores of
// gfx950 (two when the columns of a row tile are split over several workgroups).
//
// Same result as the other kernels (paper: storage paragraph of "Outlier-Aware Weight
// Quantization", section "Acceleration on Real Device"):
//     y[n,i] = sum_{j not weak} s_ig (q_ij - z_ig) x[n,j]  +  sum_t Ww_it x[n, idx_t]
//
// With few tokens the layer is bound by its weight stream and by latency, so the only thing
// in flight in the main loop is that stream.  A workgroup of four waves owns RT row tiles of
// 32 rows (RT = 1, 2 or 4) and a range of blocks of 128 columns, cut into 4 / RT slices: wave
// = (row tile, slice).  At the start the workgroup copies the activations of its range into
// LDS, in the order the matrix instruction reads them, gathers the activations at the weak
// indices, and stages the scales of its rows and the weak masks of its blocks.
// Then every wave streams its codes, several blocks ahead: a pair of codes is masked out of a
// dword and OR-ed into the mantissas of 2^(10-o), giving the A operand 2^(10-o)+q exactly;
// the B operand comes from LDS.  While staging, the workgroup also sums, per token and block,
// X = sum x and C = sum c x (c = the constant 2^(10-o) of every column).  A ninth matrix
// instruction per block, in bf16 (whose range is that of fp32), subtracts C + z X from the
// accumulators: its A operand holds -1 and -z of the row (z in two exact bf16 pieces), its B
// operand C and X of the token (three exact bf16 pieces each).  What is left per block is
// tot += s acc, one operation per element, and it runs while the matrix cores work on the next
// block, into the other accumulator.  The product of the fp16 weak columns with the gathered
// activations is a few more k-steps into tot.
// The waves of a row tile add their results through LDS in a fixed order; with more than one
// column range per row tile the sums go to memory and a second small kernel adds them, again
// in a fixed order.  No atomics.
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
  float *part;                 // split > 1: [split][ntok][d_out_pad]
  int d_in, d_out, d_out_pad, n_rt, ntok, nbp, kp, split;
  int blk_base, blk_rem;       // blocks per column range: range sp has blk_base + (sp < blk_rem) of them
  int lg_bpg;                  // blocks per group of scales: 1 << lg_bpg (one scale per row: 30, a single group)
  int lg_tok;                  // tokens are padded to 1 << lg_tok in LDS
  int lg_rt;                   // row tiles per workgroup: 1 << lg_rt
};

template <int J> struct Buf {};   // tag: register buffer J of the blocks in flight, or k-step J
template <int J> __device__ std::integral_constant<int, J> buf_index(Buf<J>);

constexpr int kSmallWaves = 4;
constexpr int kSmallSzUnits = 2;      // 16-byte units of scales a thread stages: groups x row tiles <= 64
constexpr int kSmallXUnits = 12;      // 16-byte units of activations a thread stages: blocks x padded tokens <= 192
constexpr int kSmallRedUnits = 1024;  // LDS units of the waves' results: [4][16][64] floats
constexpr int kSmallGather = 8;       // gathered activations a thread fetches at once: 2048 (weak column, token) pairs
constexpr int kSmallLdsMax = 80 * 1024;   // two workgroups per compute unit

// grid (column ranges, groups of row tiles).  Layers with one scale per row run as one group of
// scales that spans all blocks.
template <int BITS>
__global__ __launch_bounds__(256, 2) void owq_tile_small(const SmallArgs a) {
  constexpr int CH = BITS == 3 ? 3 : 4;
  // Code buffers per wave: one block in flight behind the one in use.  More were slower, step by step
  // (6 buffers: 15.1 / 20.1 us per call on the LLaMA-13B-like layers at 4 / 16 tokens, 4: 14.1 / 19.1,
  // 2: 13.5 / 18.5): with eight waves on a compute unit the loads of deeper pipelines wait for request
  // slots, and the set-up's loads wait behind them.
  constexpr int NB = 2;
  constexpr int WK = 2;                   // k-steps of weak columns whose weights a wave fetches ahead of its blocks
  extern __shared__ u32x4 lds[];

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, kg = lane >> 5;
  const int RT = 1 << a.lg_rt, KS = kSmallWaves >> a.lg_rt;
  const int rtl = w & (RT - 1), ks = w >> a.lg_rt;
  const int sp = blockIdx.x, rg = blockIdx.y;
  const int b0 = sp * a.blk_base + (sp < a.blk_rem ? sp : a.blk_rem);
  const int nbw = a.blk_base + (sp < a.blk_rem ? 1 : 0);       // >= 1: split <= number of blocks
  const int b1 = b0 + nbw;
  const int wb0 = b0 + ((nbw * ks) >> (2 - a.lg_rt)), wb1 = b0 + ((nbw * (ks + 1)) >> (2 - a.lg_rt));
  const bool rt_ok = rg * RT + rtl < a.n_rt;                    // the last group of row tiles may be short
  const int rt = rt_ok ? rg * RT + rtl : a.n_rt - 1;

  // ---- (1) the first blocks of codes, then the loads of the set-up ------------------------
  // Past the wave's range the code loads still go out (to a block that exists) and are dropped: the
  // number of loads in flight is the same on every path and the waits can be exact.
  u32x4 cA[NB];
  u32x4 cB[NB];      // 4-bit: second chunk; 3-bit: .xy = the block's half of the middle chunk
  const char *cbase = reinterpret_cast<const char *>(a.codes);
  const u32 coff = ((u32)(rt * a.nbp) * (CH * 64) + (u32)lane) * 16u;      // byte offsets: the blob is below 4 GiB
  auto fetch_codes = [&](auto tag, int b) __attribute__((always_inline)) {
    constexpr int J = decltype(buf_index(tag))::value;
    const int bc = b < wb1 ? b : b0;
    const int bp = bc >> 1, h = bc & 1;
    const u32 t = coff + (u32)bp * (CH * 64 * 16);
    cA[J] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(cbase + (t + (u32)(2 * h * 1024))));
    if (BITS == 4) {
      cB[J] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(cbase + (t + (u32)((2 * h + 1) * 1024))));
    } else {
      const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(cbase + (t + (u32)(1024 + 8 * h))));
      cB[J].x = v.x; cB[J].y = v.y;
    }
  };
  fetch_codes(Buf<0>{}, wb0);
  if constexpr (NB > 2) fetch_codes(Buf<1 % NB>{}, wb0 + 1);
  if constexpr (NB > 3) fetch_codes(Buf<2 % NB>{}, wb0 + 2);
  if constexpr (NB > 4) fetch_codes(Buf<3 % NB>{}, wb0 + 3);
  if constexpr (NB > 5) fetch_codes(Buf<4 % NB>{}, wb0 + 4);
  __builtin_amdgcn_sched_barrier(0);         // the weight stream goes out first

  const int g_lo = b0 >> a.lg_bpg;
  const int ng = ((b1 - 1) >> a.lg_bpg) - g_lo + 1;
  const int np = 1 << a.lg_tok, nm = n & (np - 1);
  const int kunits = a.kp >> 3, ksteps = (kunits + 1) >> 1;
  // LDS map, in 16-byte units.  The waves' results reuse the room of the activations at the end.
  const int nr = nbw * 16;                                      // octets of the workgroup's range
  const int pitch = nr | 1;                                     // odd: the tokens of a k-step fall into different banks
  const int npairs = nbw << a.lg_tok;                           // (block, token) pairs
  u32x4 *xs = lds;                                              // [np tokens][pitch]: 8 activations per unit
  float *red = reinterpret_cast<float *>(lds);                  // [4 waves][16][64]
  f2_t *szl = reinterpret_cast<f2_t *>(lds + (np * pitch > kSmallRedUnits ? np * pitch : kSmallRedUnits));   // [groups][row tiles]: 32 scales, 32 zero points
  u32x4 *xw = reinterpret_cast<u32x4 *>(szl) + ng * RT * 16;    // [kunits][np tokens] 8 gathered activations
  unsigned short *xw_h = reinterpret_cast<unsigned short *>(xw);
  u32x4 *bs = xw + kunits * np;                                 // [blocks][np tokens][2]: B operand of the block's ninth instruction

  // Which of the staging loads go out depends on sizes only, the same for the whole workgroup.
  // Gathers: element e = tid + 256 i is token e & (np - 1) and weak column e >> lg_tok.
  const int tok = tid & (np - 1), r0 = tid >> a.lg_tok, rstep = 256 >> a.lg_tok;
  const bool tok_ok = tok < a.ntok;
  const u32 tok_off = (u32)(tok_ok ? tok : 0) * (u32)a.d_in;
  int gj[kSmallGather];
#pragma unroll
  for (int i = 0; i < kSmallGather; ++i) {
    const int t = r0 + i * rstep;
    gj[i] = -1;
    if (i * rstep < a.kp) gj[i] = a.weak_idx[(u32)(t < a.kp ? t : 0)];
  }
  u32x4 szv[kSmallSzUnits];
#pragma unroll
  for (int j = 0; j < kSmallSzUnits; ++j) {
    const int i = tid + 256 * j, ic = i < ng * RT * 8 ? i : 0;
    const int gq = (ic >> 3) >> a.lg_rt, rq = (ic >> 3) & (RT - 1);
    int rtq = rg * RT + rq;
    if (rtq > a.n_rt - 1) rtq = a.n_rt - 1;
    szv[j] = *reinterpret_cast<const u32x4 *>(a.sz + (u32)((g_lo + gq) * a.d_out_pad + rtq * 32 + (ic & 7) * 4));
  }
  // Activations: 16 lanes take the 16 octets of a (block, token) pair; pair p = (tid >> 4) + 16 j is token
  // p & (np - 1) of block p >> lg_tok.
  const int o16 = tid & 15, pg = tid >> 4;
  u32x4 xv[kSmallXUnits];
  u32 xm[kSmallXUnits];         // the octet's byte of the weak mask
#pragma unroll
  for (int j = 0; j < kSmallXUnits; ++j) {
    const int pr = pg + 16 * j, prc = pr < npairs ? pr : 0;
    const int tk = prc & (np - 1), bl = prc >> a.lg_tok;
    if (16 * j < npairs) {
      xv[j] = *reinterpret_cast<const u32x4 *>(a.x + ((u32)(tk < a.ntok ? tk : 0) * (u32)a.d_in + (u32)((b0 + bl) * 128 + o16 * 8)));
      xm[j] = a.wmask[(u32)((b0 + bl) * 16 + o16)];
    }
  }
  // weak columns: the k-steps are dealt out to the waves of the row tile in all its workgroups;
  // the weights of a wave's first WK k-steps ride ahead of its blocks
  const int wslot = sp * KS + ks, wstride = a.split * KS;
  u32x4 wa[WK];
#pragma unroll
  for (int i = 0; i < WK; ++i) {
    const int u = 2 * (wslot + wstride * i) + kg;
    wa[i] = a.weak_w[(u32)((rt * 32 + n) * kunits + (u < kunits ? u : 0))];
  }
  __builtin_amdgcn_sched_barrier(0);         // all of these are in flight before anything waits

  // ---- (2) the gathers go out once their indices are there; scales and activations into LDS ---
  // The gathered values stay in registers until the wave's blocks are done: nothing waits for them.
  u32 gv[kSmallGather];     // one fp16 each, kept apart: packing them here would wait for the loads
  u32 gok = 0u;
  const unsigned short *xbits = reinterpret_cast<const unsigned short *>(a.x);
#pragma unroll
  for (int i = 0; i < kSmallGather; ++i) {
    const int t = r0 + i * rstep;
    const bool ok = t < a.kp && tok_ok && (u32)gj[i] < (u32)a.d_in;
    gv[i] = xbits[ok ? tok_off + (u32)gj[i] : 0u];     // always issued: a load under a branch would be waited for there
    gok |= ok ? (1u << i) : 0u;
  }
#pragma unroll
  for (int j = 0; j < kSmallSzUnits; ++j) {
    const int i = tid + 256 * j;
    if (i < ng * RT * 8) {
      const u32 d[4] = {szv[j].x, szv[j].y, szv[j].z, szv[j].w};
      // unit i = rows 4 (i & 7) .. + 3 of (group, row tile) i >> 3: 32 scales, then 32 zero points
      float *dst = reinterpret_cast<float *>(szl) + (i >> 3) * 64 + (i & 7) * 4;
      *reinterpret_cast<f4_t *>(dst) = (f4_t){half_lo(d[0]), half_lo(d[1]), half_lo(d[2]), half_lo(d[3])};
      *reinterpret_cast<f4_t *>(dst + 32) = (f4_t){half_hi(d[0]), half_hi(d[1]), half_hi(d[2]), half_hi(d[3])};
    }
  }
  {
    // constants 2^(10-o) of the pairs of this lane's octet: its k-step is o16 >> 1, whose place in the quad of 32 codes decides
    float c0 = 0.f, c1 = 0.f, c2 = 0.f, c3 = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (((o16 >> 1) & 3) == q) {
        c0 = (float)(1 << (10 - pair_offset(BITS, q, 0))); c1 = (float)(1 << (10 - pair_offset(BITS, q, 1)));
        c2 = (float)(1 << (10 - pair_offset(BITS, q, 2))); c3 = (float)(1 << (10 - pair_offset(BITS, q, 3)));
      }
#pragma unroll
    for (int j = 0; j < kSmallXUnits; ++j) {
      const int pr = pg + 16 * j;
      if (16 * j < npairs) {                   // same for the whole workgroup
        const int prc = pr < npairs ? pr : 0;
        const int tk = prc & (np - 1), bl = prc >> a.lg_tok;
        u32x4 v = tk < a.ntok ? xv[j] : (u32x4){0u, 0u, 0u, 0u};
        // weak columns contribute nothing to the dense term
        const u32 m = xm[j];
        if (m != 0u) {
          if (m & 0x01u) v.x &= 0xffff0000u;
          if (m & 0x02u) v.x &= 0x0000ffffu;
          if (m & 0x04u) v.y &= 0xffff0000u;
          if (m & 0x08u) v.y &= 0x0000ffffu;
          if (m & 0x10u) v.z &= 0xffff0000u;
          if (m & 0x20u) v.z &= 0x0000ffffu;
          if (m & 0x40u) v.w &= 0xffff0000u;
          if (m & 0x80u) v.w &= 0x0000ffffu;
        }
        if (pr < npairs) xs[tk * pitch + bl * 16 + o16] = v;
        // sum x and sum c*x over the block: the 16 octets sit in 16 neighbouring lanes
        const float p0 = dot2(v.x, kOnes, 0.f), p1 = dot2(v.y, kOnes, 0.f), p2 = dot2(v.z, kOnes, 0.f), p3 = dot2(v.w, kOnes, 0.f);
        const float sx = row16_sum((p0 + p1) + (p2 + p3));
        const float sb = row16_sum(__builtin_fmaf(p3, c3, __builtin_fmaf(p2, c2, __builtin_fmaf(p1, c1, p0 * c0))));
        if (o16 == 0 && pr < npairs) {
          // C = sb and X = sx in three bf16 pieces each (the top 16 bits of what is left: exact)
          const u32 ch = __builtin_bit_cast(u32, sb) & 0xffff0000u;
          const float cr = sb - __builtin_bit_cast(float, ch);
          const u32 cm = __builtin_bit_cast(u32, cr) & 0xffff0000u;
          const u32 cl = __builtin_bit_cast(u32, cr - __builtin_bit_cast(float, cm)) & 0xffff0000u;
          const u32 xh = __builtin_bit_cast(u32, sx) & 0xffff0000u;
          const float xr = sx - __builtin_bit_cast(float, xh);
          const u32 xmid = __builtin_bit_cast(u32, xr) & 0xffff0000u;
          const u32 xl = __builtin_bit_cast(u32, xr - __builtin_bit_cast(float, xmid)) & 0xffff0000u;
          // k = 0..7: C_h C_m C_l X_h X_m X_l X_h X_m; k = 8: X_l
          bs[2 * prc] = (u32x4){(ch >> 16) | cm, (cl >> 16) | xh, (xmid >> 16) | xl, (xh >> 16) | xmid};
          bs[2 * prc + 1] = (u32x4){xl >> 16, 0u, 0u, 0u};
        }
      }
      __builtin_amdgcn_sched_barrier(0);     // one unit at a time: interleaving them costs registers, not time
    }
  }
  __syncthreads();

  // ---- (3) the wave's blocks ------------------------------------------------------------
  Magic M;
  M.init();
  f16_t acc0, acc1, tot;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; tot[r] = 0.f; }
  const f16_t zero16 = tot;
  int b = wb0;
  const int bpg_mask = (1 << a.lg_bpg) - 1;
  int gi = (wb0 >> a.lg_bpg) - g_lo, gpos = wb0 & bpg_mask;
  int gi_prev = 0;

  // tot += s * acc with the staged scales of group g
  auto scale_in = [&](const f16_t &acc, int g) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f4_t sc = *reinterpret_cast<const f4_t *>(reinterpret_cast<const float *>(szl) + (g * RT + rtl) * 64 + 8 * q + 4 * kg);
#pragma unroll
      for (int e = 0; e < 4; ++e) tot[4 * q + e] = __builtin_fmaf(sc[e], acc[4 * q + e], tot[4 * q + e]);
    }
  };

  // One block out of code buffer J: eight k-steps of codes, then the ninth instruction that
  // takes sum c*x + z * sum x away.  The products go to the accumulator of the block's parity;
  // the scaling of the previous block (the other accumulator) runs after the first k-steps have
  // been issued, while the matrix cores work.
  auto step = [&](auto tag) __attribute__((always_inline)) {
    constexpr int J = decltype(buf_index(tag))::value;
    // refill the buffer of the previous step (its registers are dead; the one in use is still
    // being read) for the block NB - 1 ahead
    fetch_codes(Buf<(J + NB - 1) % NB>{}, b + NB - 1);
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
    const u32x4 *xb = xs + nm * pitch + (b - b0) * 16 + kg;
    f16_t &acc = (J & 1) ? acc1 : acc0;
    auto kstep = [&](auto ks_tag) __attribute__((always_inline)) {
      constexpr int S = decltype(buf_index(ks_tag))::value;
      const h8_t bo = __builtin_bit_cast(h8_t, xb[2 * S]);
      const h8_t ao = a_operand<BITS, S>(wd, M);
      acc = mma(ao, bo, S == 0 ? zero16 : acc);
    };
    kstep(Buf<0>{}); kstep(Buf<1>{});
    if (b > wb0) {
      if (J & 1) scale_in(acc0, gi_prev); else scale_in(acc1, gi_prev);
    }
    kstep(Buf<2>{}); kstep(Buf<3>{});
    kstep(Buf<4>{}); kstep(Buf<5>{}); kstep(Buf<6>{}); kstep(Buf<7>{});
    {
      // ninth instruction: A = (-1 -1 -1 -zh -zh -zh -zl -zl | -zl 0 ...) of this lane's row, zh + zl = z exactly
      const float z = reinterpret_cast<const float *>(szl)[(gi * RT + rtl) * 64 + 32 + n];
      const u32 zh = __builtin_bit_cast(u32, z) & 0xffff0000u;
      const u32 zl = __builtin_bit_cast(u32, z - __builtin_bit_cast(float, zh)) & 0xffff0000u;
      const u32 nzh = zh ^ 0x80000000u, nzl = zl ^ 0x80000000u;
      const u32 m1 = 0xbf80u;                  // bf16 -1
      u32x4 ae;
      if (kg == 0) ae = (u32x4){m1 | (m1 << 16), m1 | nzh, (nzh >> 16) | nzh, (nzl >> 16) | nzl};
      else ae = (u32x4){nzl >> 16, 0u, 0u, 0u};
      const u32x4 be = bs[2 * (((b - b0) << a.lg_tok) + nm) + kg];
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8_t, ae), __builtin_bit_cast(bf8_t, be), acc, 0, 0, 0);
    }
    gi_prev = gi;
    if (++gpos > bpg_mask) { gpos = 0; ++gi; }
    ++b;
    __builtin_amdgcn_sched_barrier(0);         // blocks are scheduled one by one: mixing them costs registers
  };
#pragma unroll 1
  while (b + NB <= wb1) {
    step(Buf<0>{});
    step(Buf<1>{});
    if constexpr (NB > 2) step(Buf<2 % NB>{});
    if constexpr (NB > 3) step(Buf<3 % NB>{});
    if constexpr (NB > 4) step(Buf<4 % NB>{});
    if constexpr (NB > 5) step(Buf<5 % NB>{});
  }
  if (b < wb1) step(Buf<0>{});
  if constexpr (NB > 2) { if (b < wb1) step(Buf<1 % NB>{}); }
  if constexpr (NB > 3) { if (b < wb1) step(Buf<2 % NB>{}); }
  if constexpr (NB > 4) { if (b < wb1) step(Buf<3 % NB>{}); }
  if constexpr (NB > 5) { if (b < wb1) step(Buf<4 % NB>{}); }
  if (b > wb0) {                               // the last block's scaling
    if ((b - 1 - wb0) & 1) scale_in(acc1, gi_prev); else scale_in(acc0, gi_prev);
  }

  // ---- (4) weak columns -----------------------------------------------------------------
  // element (weak column t, token) -> unit t >> 3 of the token, half t & 7
#pragma unroll
  for (int i = 0; i < kSmallGather; ++i) {
    const int t = r0 + i * rstep;
    if (t < a.kp) xw_h[(((t >> 3) << a.lg_tok) + tok) * 8 + (t & 7)] = ((gok >> i) & 1u) ? (unsigned short)gv[i] : (unsigned short)0;
  }
  for (int tb = kSmallGather * rstep; tb < a.kp; tb += kSmallGather * rstep) {     // many weak columns: further rounds
    int j2[kSmallGather];
#pragma unroll
    for (int i = 0; i < kSmallGather; ++i) {
      const int t = tb + r0 + i * rstep;
      j2[i] = a.weak_idx[(u32)(t < a.kp ? t : 0)];
    }
    u32 v2[kSmallGather];
#pragma unroll
    for (int i = 0; i < kSmallGather; ++i) {
      const int t = tb + r0 + i * rstep;
      const bool ok = t < a.kp && tok_ok && (u32)j2[i] < (u32)a.d_in;
      v2[i] = xbits[ok ? tok_off + (u32)j2[i] : 0u];
      j2[i] = ok ? 1 : 0;
    }
#pragma unroll
    for (int i = 0; i < kSmallGather; ++i) {
      const int t = tb + r0 + i * rstep;
      if (t < a.kp) xw_h[(((t >> 3) << a.lg_tok) + tok) * 8 + (t & 7)] = j2[i] ? (unsigned short)v2[i] : (unsigned short)0;
    }
  }
  __syncthreads();        // every wave is past its blocks: the room of the activations is free for the results
  if (kunits > 0) {
    const u32x4 z4 = {0u, 0u, 0u, 0u};
    const u32x4 *xwl = xw + nm;
#pragma unroll
    for (int i = 0; i < WK; ++i) {
      const int s = wslot + wstride * i;
      if (s < ksteps) {                        // same for the whole wave
        const int u = 2 * s + kg;
        const bool uv = u < kunits;
        const u32x4 bv = xwl[(uv ? u : 0) << a.lg_tok];
        tot = mma(__builtin_bit_cast(h8_t, uv ? wa[i] : z4), __builtin_bit_cast(h8_t, uv ? bv : z4), tot);
      }
    }
    for (int s = wslot + wstride * WK; s < ksteps; s += wstride) {    // many weak columns: no longer ahead
      const int u = 2 * s + kg;
      const bool uv = u < kunits;
      const u32x4 av = a.weak_w[(u32)((rt * 32 + n) * kunits + (uv ? u : 0))];
      const u32x4 bv = xwl[(uv ? u : 0) << a.lg_tok];
      tot = mma(__builtin_bit_cast(h8_t, uv ? av : z4), __builtin_bit_cast(h8_t, uv ? bv : z4), tot);
    }
  }

  // ---- (5) the results of the waves of a row tile, added in a fixed order ----------------
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(w * 16 + r) * 64 + lane] = tot[r];
  __syncthreads();
  for (int e = tid; e < (a.ntok << (5 + a.lg_rt)); e += 256) {
    const int row = e & 31, rq = (e >> 5) & (RT - 1), nn = e >> (5 + a.lg_rt);
    const int r = 4 * (row >> 3) + (row & 3), ln = nn + 32 * ((row >> 2) & 1);
    float v = 0.f;
    for (int q = 0; q < KS; ++q) v += red[(((q << a.lg_rt) + rq) * 16 + r) * 64 + ln];
    const int grow = (rg * RT + rq) * 32 + row;
    if (a.split == 1) {
      if (grow < a.d_out) a.y[(size_t)nn * a.d_out + grow] = (_Float16)v;
    } else if (grow < a.d_out_pad) {
      a.part[(size_t)(sp * a.ntok + nn) * a.d_out_pad + grow] = v;
    }
  }
}

// Adds the results of the column ranges of every row (fixed order) and rounds to fp16.
__global__ __launch_bounds__(256) void owq_tile_small_sum(const float *part, _Float16 *y, int split, int ntok, int d_out,
                                                          int d_out_pad) {
  const int row = blockIdx.x * 256 + threadIdx.x, nn = blockIdx.y;
  if (row >= d_out || nn >= ntok) return;
  float v = 0.f;
  const float *p0 = part + (size_t)nn * d_out_pad + row;
  const size_t pitch = (size_t)ntok * d_out_pad;
  for (int s0 = 0; s0 < split; s0 += 16) {        // sixteen loads in flight; the additions keep their order
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) p[i] = p0[(size_t)(s0 + i < split ? s0 + i : s0) * pitch];
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (s0 + i < split) v += p[i];
  }
  y[(size_t)nn * d_out + row] = (_Float16)v;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
typedef void (*small_fn)(const SmallArgs);

static small_fn pick_small(int bits) { return bits == 3 ? owq_tile_small<3> : owq_tile_small<4>; }

static int real_blocks(const owq_layer_info_t &g) { return (g.d_in + kBlockCols - 1) / kBlockCols; }

static int log2_ceil(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

// log2 of the blocks per group of scales (one scale per row: 30, a single group); -1 = not a power of two
static int log2_bpg(const owq_layer_info_t &g) {
  if (g.n_groups <= 1) return 30;
  const int bpg = g.group_size / kBlockCols;
  const int l = log2_ceil(bpg);
  return (1 << l) == bpg ? l : -1;
}

// LDS bytes of the kernel for `split` column ranges per row tile, 1 << lg_rt row tiles per
// workgroup and tokens padded to 1 << lg_tok; 0 = does not fit the kernel's staging (units per
// thread), the LDS of two workgroups per compute unit or the room for partial sums.
static int32_t small_lds_bytes(const owq_layer_info_t &g, int32_t split, int lg_rt, int lg_tok, uint64_t part_bytes) {
  const int nblk = real_blocks(g), lb = log2_bpg(g);
  if (split < 1 || split > nblk || lb < 0) return 0;
  const int rt = 1 << lg_rt, np = 1 << lg_tok;
  const int base = nblk / split, rem = nblk % split;
  int ng_max = 1;
  for (int sp = 0; sp < split; ++sp) {
    const int b0 = sp * base + (sp < rem ? sp : rem), b1 = b0 + base + (sp < rem ? 1 : 0);
    const int ng = ((b1 - 1) >> lb) - (b0 >> lb) + 1;
    if (ng > ng_max) ng_max = ng;
  }
  const int nbw_max = base + (rem > 0 ? 1 : 0);
  if (ng_max * rt * 8 > kSmallSzUnits * 256 || nbw_max * np > kSmallXUnits * 16) return 0;
  if (split > 1 && (uint64_t)split * 32 * g.d_out_pad * 4 > part_bytes) return 0;
  const int xunits = np * ((nbw_max * 16) | 1);
  // activations (or the waves' results), scales, gathered activations, sums per block and token
  const int64_t units = (int64_t)(xunits > kSmallRedUnits ? xunits : kSmallRedUnits) + ng_max * rt * 16 + (int64_t)(g.kp / 8) * np +
                        2 * nbw_max * np;
  if (units * 16 > kSmallLdsMax) return 0;
  return (int32_t)(units * 16);
}

// Work split when the caller does not say: a rough model of the launch in microseconds (a
// workgroup's fixed cost, the blocks each wave streams, the traffic of activations and of
// partial sums, the second launch), minimised over the row tiles per workgroup and the ranges.
static double small_default_shape(const owq_layer_info_t &g, int ntok, int32_t want_split, int want_lg_rt, uint64_t part_bytes,
                                  int32_t *split, int *lg_rt) {
  const int nblk = real_blocks(g), lg_tok = log2_ceil(ntok);
  double best = 0.0;
  *split = 0;
  *lg_rt = 0;
  for (int l = 2; l >= 0; --l) {
    if (want_lg_rt >= 0 && l != want_lg_rt) continue;
    const int rt = 1 << l, ks = kSmallWaves >> l;
    const int n_rg = (g.n_rt + rt - 1) / rt;
    for (int32_t s = 1; s <= 64 && s <= nblk; ++s) {
      if (want_split > 0 && s != want_split) continue;
      if (small_lds_bytes(g, s, l, lg_tok, part_bytes) == 0) continue;
      const int64_t wgs = (int64_t)n_rg * s;
      const double rounds = (double)((wgs + 511) / 512);      // 512 places: a few workgroups more cost a whole round
      const int nbw = (nblk + s - 1) / s;
      const double per_wave = (double)((nbw + ks - 1) / ks);
      const double part_mb = s > 1 ? 2.0 * s * ntok * g.d_out * 4.0 / 1e6 : 0.0;
      // fitted to measurements of 5120x5120, 5120x13824 and 13824x5120 layers at 2 to 16 tokens
      const double cost = rounds * (3.0 + 0.55 * per_wave + 0.02 * nbw * (1 << lg_tok)) + part_mb / 3.0 + (s > 1 ? 2.5 : 0.0);
      if (*split == 0 || cost < best) { best = cost; *split = s; *lg_rt = l; }
    }
  }
  return best;
}

// owq_set_launch: is this split possible at all (one token, any number of row tiles per workgroup)?
bool tile_small_split_ok(const owq_layer_info_t &g, int32_t split) {
  const TileScratch ts = tile_scratch(g);
  for (int l = 0; l <= 2; ++l)
    if (small_lds_bytes(g, split, l, 0, ts.total - ts.off_slots) > 0) return true;
  return false;
}

int prepare_tile_small_kernels() {
  for (int bits = 3; bits <= 4; ++bits) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_small(bits)),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kSmallLdsMax);
    if (e != hipSuccess) return (int)e;
  }
  return (int)hipSuccess;
}

// Passes of more tokens than this take the three-launch path unless the caller sets a shape:
// there the activations of a workgroup's range no longer fit LDS without many column ranges.
constexpr int kSmallAutoTokens = 16;

// One pass of up to 32 tokens.  shape = S + 100 c: S column ranges per row tile (0 = the
// library's choice), c = 0: the library chooses the row tiles per workgroup, c = 1, 2, 3: 1, 2
// or 4 of them.  Returns a hipError_t as int, -1 when this layer or the alignment of x does not
// fit the kernel and the caller has to take the three-launch path, -2 when the caller asked
// for a shape that does not fit this number of tokens.
int launch_tile_small(const owq_layer_info_t &g, void *blob, void *part, uint64_t part_bytes, int32_t shape, const void *x,
                      void *y, int32_t ntok, void *stream) {
  if (ntok < 1 || ntok > 32 || shape < 0 || (shape == 0 && ntok > kSmallAutoTokens)) return -1;
  if ((reinterpret_cast<uintptr_t>(x) & 15) != 0 || g.d_in % kBlockCols != 0) return -1;   // whole blocks, aligned rows
  if (log2_bpg(g) < 0) return -1;                                                            // groups of 2^n blocks
  int32_t split = 0;
  int lg_rt = 0;
  const double cost = small_default_shape(g, ntok, shape % 100, shape / 100 - 1, part_bytes, &split, &lg_rt);
  if (split < 1) return shape > 0 ? -2 : -1;
  if (shape == 0) {
    // Large layers stream so many blocks per wave that the three launches do as well or better: their
    // time is about 15 us + 1 us per 4.2 MB of codes at these batch sizes (measured on 13 to 127 MB layers).
    const double code_mb = (double)g.n_rt * g.nbp * 64 * g.chunks * 16 / 1e6;
    if (cost * 1.15 >= 15.0 + code_mb / 4.2) return -1;
  }
  const int lg_tok = log2_ceil(ntok);
  uint8_t *base = static_cast<uint8_t *>(blob);
  SmallArgs a;
  a.codes = reinterpret_cast<const u32x4 *>(base + g.off_codes);
  a.sz = reinterpret_cast<const u32 *>(base + g.off_sz);
  a.wmask = base + g.off_wmask;
  a.weak_idx = reinterpret_cast<const int *>(base + g.off_weak_idx);
  a.weak_w = reinterpret_cast<const u32x4 *>(base + g.off_weak_w);
  a.x = static_cast<const _Float16 *>(x);
  a.y = static_cast<_Float16 *>(y);
  a.part = static_cast<float *>(part);
  a.d_in = g.d_in; a.d_out = g.d_out; a.d_out_pad = g.d_out_pad; a.n_rt = g.n_rt; a.ntok = ntok; a.nbp = g.nbp;
  const int nblk = real_blocks(g);
  a.blk_base = nblk / split; a.blk_rem = nblk % split;
  a.lg_bpg = log2_bpg(g);
  a.kp = g.kp; a.split = split; a.lg_tok = lg_tok; a.lg_rt = lg_rt;
  const int n_rg = (g.n_rt + (1 << lg_rt) - 1) >> lg_rt;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(pick_small(g.bits), dim3((unsigned)split, (unsigned)n_rg, 1), dim3(256, 1, 1),
                     (size_t)small_lds_bytes(g, split, lg_rt, lg_tok, part_bytes), st, a);
  if (split > 1)
    hipLaunchKernelGGL(owq_tile_small_sum, dim3((unsigned)((g.d_out + 255) / 256), (unsigned)ntok, 1), dim3(256, 1, 1), 0, st,
                       a.part, a.y, split, ntok, g.d_out, g.d_out_pad);
  return (int)hipGetLastError();
}

}  // namespace owq
