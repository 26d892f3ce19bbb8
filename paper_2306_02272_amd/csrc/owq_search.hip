// Quantization configuration search (paper, section "Quantization Configuration Search") for
// gfx950: for every (output row, group of input columns) a two-dimensional grid of narrowed
// ranges is tried and the step size and zero point with the least rounding error are kept.
//
// The work is plain fp32 arithmetic, five vector instructions per weight and grid point, so the
// kernel is laid out for the vector units, not for memory: one wave owns one (row, group), every
// lane owns up to four grid points (its step size, zero point and running error stay in
// registers), and the weights of the group are moved through LDS once (converted to fp32, the
// weak columns dropped) and then read back four at a time at one address for the whole wave,
// which LDS serves as a broadcast.  No reduction across lanes happens until the grid points of
// a group are ranked at its end.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>

#include "owq.h"

namespace owq {
namespace {

typedef unsigned int u32;
typedef float f4v __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;            // waves per workgroup, each with its own LDS area
constexpr int kChunk = 1024;         // columns moved through LDS at a time
constexpr int kMaskBytesMax = 47 * 1024;   // LDS left for the weak-column bit mask of a row: 64 KiB less the kernel's static 16.1 KiB

struct SearchArgs {
  const _Float16 *w;
  const int *weak_idx;
  uint16_t *scale, *zero;
  uint8_t *codes;
  float *err;
  int *choice;
  int d_in, g, n_groups, k, n_lo, n_hi, units, units_per_wave;
  float qmax, shrink;
};

struct Cand {
  float s, inv, a, b;                // step size, its reciprocal, -z, qmax - z
};

// op over the 64 lanes of the wave, every lane gets the result: four steps inside the rows of
// 16 lanes on the data-parallel path, then the four row results through scalar registers
template <class T, class F>
__device__ __forceinline__ T wave_all(T v, F op) {
  auto dpp = [](T x, auto ctrl) __attribute__((always_inline)) {
    return __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, false));
  };
  v = op(v, dpp(v, std::integral_constant<int, 0xB1>{}));    // lanes ^ 1
  v = op(v, dpp(v, std::integral_constant<int, 0x4E>{}));    // lanes ^ 2
  v = op(v, dpp(v, std::integral_constant<int, 0x141>{}));   // mirror in 8
  v = op(v, dpp(v, std::integral_constant<int, 0x140>{}));   // mirror in 16
  const int i = __builtin_bit_cast(int, v);
  const T r0 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(i, 0)), r1 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(i, 16));
  const T r2 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(i, 32)), r3 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(i, 48));
  return op(op(r0, r1), op(r2, r3));
}

// Step size, reciprocal and zero point of the grid point that cuts the fractions fa and fb of
// the range from its ends.  Every operation is a single binary32 operation in the order the
// interface states; nothing may be fused here.
__device__ __forceinline__ Cand candidate(float lo, float hi, float fa, float fb, float qmax) {
#pragma clang fp contract(off)
  const float r = hi - lo;
  const float pa = fa * r, pb = fb * r;
  const float lo_i = lo + pa, hi_j = hi - pb;
  const float width = hi_j - lo_i;
  float s32 = width / qmax;
  s32 = s32 > 0x1p-14f ? s32 : 0x1p-14f;
  const float s = (float)(_Float16)s32;
  const float inv = 1.0f / s;
  const float zl = -lo_i * inv;
  float z = __builtin_rintf(zl);
  z = z < -2048.f ? -2048.f : (z > 2048.f ? 2048.f : z);
  Cand c;
  c.s = s;
  c.inv = inv;
  c.a = 0.f - z;                     // 0 - z: no negative zero
  c.b = qmax - z;
  return c;
}

// fraction of the range that grid point i of n cuts: binary32 of (shrink * i) / (n - 1) in binary64
__device__ __forceinline__ float cut_fraction(float shrink, int i, int n) {
  if (n == 1) return 0.f;
  return (float)((double)shrink * (double)i / (double)(n - 1));
}

__device__ __forceinline__ void wave_lds_fence() {
  // LDS serves one wave's instructions in order; this keeps the compiler from moving them
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ bool is_weak(const u32 *mask, int col) {
  return ((mask[col >> 5] >> (col & 31)) & 1u) != 0u;
}

// Moves the non-weak weights of columns [col0, col0 + n) of a row into `list` as fp32, in
// order, and returns how many there are.  n <= kChunk.
__device__ __forceinline__ int stage(const _Float16 *wrow, int col0, int n, float *list, const u32 *mask, int lane) {
  int cnt = 0;
  for (int t = 0; t < n; t += 64) {
    const int c = t + lane;
    const bool valid = c < n;
    const float v = valid ? (float)wrow[col0 + c] : 0.f;
    const bool keep = valid && !is_weak(mask, col0 + c);
    const unsigned long long m = __ballot(keep);
    const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
    if (keep) list[pos] = v;
    cnt += __builtin_popcountll(m);
  }
  wave_lds_fence();
  return cnt;
}

template <int CPL>
__device__ __forceinline__ void accumulate(const Cand (&cd)[CPL], float (&e)[CPL], float w) {
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const float t = w * cd[c].inv;
    const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(t), cd[c].a, cd[c].b);   // q - z
    const float d = __builtin_fmaf(-cd[c].s, q, w);
    e[c] = __builtin_fmaf(d, d, e[c]);
  }
}

// What the search of one (row, group) yields.
struct Best {
  float s, inv, z, e;
  int id;
};

// The grid points of this lane for the range [lo, hi], errors cleared.
template <int CPL>
__device__ __forceinline__ void make_cands(float lo, float hi, const float (&fa)[CPL], const float (&fb)[CPL],
                                           float qmax, Cand (&cd)[CPL], float (&e)[CPL]) {
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    cd[c] = candidate(lo, hi, fa[c], fb[c], qmax);
    e[c] = 0.f;
  }
}

// Adds the errors of list[0 .. cnt) to every grid point of this lane.
template <int CPL>
__device__ __forceinline__ void accumulate_list(const float *list, int cnt, const Cand (&cd)[CPL], float (&e)[CPL]) {
  const f4v *l4 = reinterpret_cast<const f4v *>(list);
  int i = 0;
  f4v nxt = l4[0];                                 // one address for the wave: a broadcast
  for (; i + 4 <= cnt; i += 4) {
    const f4v v = nxt;
    nxt = l4[(i >> 2) + 1];                        // one step ahead (the list has four spare entries)
    accumulate<CPL>(cd, e, v[0]);
    accumulate<CPL>(cd, e, v[1]);
    accumulate<CPL>(cd, e, v[2]);
    accumulate<CPL>(cd, e, v[3]);
  }
  for (; i < cnt; ++i) accumulate<CPL>(cd, e, list[i]);
}

// Ranks this lane's grid points, then the wave's; equal errors go to the lower index.  The
// winner's step size and zero point are read from the lane that holds them.
template <int CPL>
__device__ __forceinline__ Best pick(const Cand (&cd)[CPL], const float (&e)[CPL], int ncand, int lane) {
  float eb = INFINITY;
  int ib = 0x7fffffff;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int id = lane + 64 * c;
    if (id < ncand && (e[c] < eb || (e[c] == eb && id < ib))) {
      eb = e[c];
      ib = id;
    }
  }
  const float e_min = wave_all(eb, [](float x, float y) { return x < y ? x : y; });
  ib = wave_all(eb == e_min ? ib : 0x7fffffff, [](int x, int y) { return x < y ? x : y; });
  ib = __builtin_amdgcn_readfirstlane(ib);
  const int slot = ib >> 6, src = ib & 63;
  auto from_lane = [&](float v) __attribute__((always_inline)) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src));
  };
  Best b;
  b.s = from_lane(cd[0].s);
  b.inv = from_lane(cd[0].inv);
  float neg_z = from_lane(cd[0].a);
#pragma unroll
  for (int c = 1; c < CPL; ++c) {                  // slot is the same for the whole wave
    const float s = from_lane(cd[c].s), inv = from_lane(cd[c].inv), na = from_lane(cd[c].a);
    b.s = slot == c ? s : b.s;
    b.inv = slot == c ? inv : b.inv;
    neg_z = slot == c ? na : neg_z;
  }
  b.z = 0.f - neg_z;
  b.e = e_min;
  b.id = ib;
  return b;
}

// Widens a zero-width range to reach 0; true if there is nothing to search.
__device__ __forceinline__ bool degenerate(float &lo, float &hi, int kept) {
  if (kept == 0) return true;
  if (hi == lo) {
    lo = lo < 0.f ? lo : 0.f;
    hi = hi > 0.f ? hi : 0.f;
    return hi == lo;
  }
  return false;
}

__device__ __forceinline__ void store_choice(const SearchArgs &a, int row, int gi, const Best &b, int lane) {
  if (lane == 0) {
    const size_t o = (size_t)row * a.n_groups + gi;
    a.scale[o] = __builtin_bit_cast(uint16_t, (_Float16)b.s);
    a.zero[o] = __builtin_bit_cast(uint16_t, (_Float16)b.z);
    if (a.err != nullptr) a.err[o] = b.e;
    if (a.choice != nullptr) a.choice[o] = b.id;
  }
}

__device__ __forceinline__ uint8_t code_of(float v, const Best &b, float qmax) {
  const float za = 0.f - b.z, zb = qmax - b.z;
  return (uint8_t)(int)(__builtin_amdgcn_fmed3f(__builtin_rintf(v * b.inv), za, zb) - za);
}

// NT > 0: groups of at most 64 NT columns.  A lane keeps its NT weights of the group in
// registers (they serve the range, the list in LDS and the codes), and the weights of the
// wave's next group are fetched while the current one is searched.
// NT = 0: longer groups, moved through LDS kChunk columns at a time, three passes over the row
// (range, errors, codes).
template <int CPL, int NT>
__global__ __launch_bounds__(kWaves * 64) void owq_search_kernel(const SearchArgs a) {
  __shared__ __attribute__((aligned(16))) float lists[kWaves][kChunk + 4];   // + 4: read one step ahead
  extern __shared__ u32 mask[];                    // bit c = column c is weak; (d_in + 31) / 32 words
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float *list = lists[wv];
  // every thread of the workgroup passes these two barriers before anything may leave
  for (int i = threadIdx.x; i < (a.d_in + 31) >> 5; i += kWaves * 64) mask[i] = 0u;
  __syncthreads();
  for (int p = threadIdx.x; p < a.k; p += kWaves * 64) {
    const u32 c = (u32)a.weak_idx[p];
    if (c < (u32)a.d_in) atomicOr(&mask[c >> 5], 1u << (c & 31));
  }
  __syncthreads();
  const int ncand = a.n_lo * a.n_hi;
  // the cut fractions of this lane's grid points do not depend on the group
  float fa[CPL], fb[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int id = lane + 64 * c;
    const int i = id / a.n_hi, j = id - i * a.n_hi;
    fa[c] = cut_fraction(a.shrink, i < a.n_lo ? i : 0, a.n_lo);
    fb[c] = cut_fraction(a.shrink, j, a.n_hi);
  }
  const int u0 = (blockIdx.x * kWaves + wv) * a.units_per_wave;
  const int n_units = a.units - u0 < a.units_per_wave ? a.units - u0 : a.units_per_wave;   // same for the wave
  if (n_units <= 0) return;
  int row = u0 / a.n_groups, gi = u0 - row * a.n_groups;
  const Best none = {1.f, 1.f, 0.f, 0.f, 0};

  if constexpr (NT > 0) {
    // columns past the end of a short last group are fetched from its last column and dropped
    auto fetch = [&](_Float16 (&dst)[NT], int r, int g) __attribute__((always_inline)) {
      const int c0 = g * a.g;
      const int last = (a.d_in - c0 < a.g ? a.d_in - c0 : a.g) - 1;
      const _Float16 *src = a.w + (size_t)r * a.d_in + c0;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int c = t * 64 + lane;
        dst[t] = src[c < last ? c : last];
      }
    };
    _Float16 cur[NT], nxt[NT];
    fetch(cur, row, gi);
    for (int uu = 0; uu < n_units; ++uu) {
      const int c0 = gi * a.g;
      const int len = a.d_in - c0 < a.g ? a.d_in - c0 : a.g;
      int nrow = row, ngi = gi + 1;
      if (ngi == a.n_groups) {
        ngi = 0;
        ++nrow;
      }
      if (uu + 1 < n_units) fetch(nxt, nrow, ngi);
      // range and list straight from the registers
      float lo = INFINITY, hi = -INFINITY;
      int cnt = 0;
      u32 weak_bits = 0u;                          // bit t: slot t of this lane is no weight of the search
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int c = t * 64 + lane;
        const bool keep = c < len && !is_weak(mask, c0 + (c < len ? c : 0));
        const float v = (float)cur[t];
        const unsigned long long m = __ballot(keep);
        const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
        if (keep) {
          list[pos] = v;
          lo = v < lo ? v : lo;
          hi = v > hi ? v : hi;
        } else {
          weak_bits |= 1u << t;
        }
        cnt += __builtin_popcountll(m);
      }
      wave_lds_fence();
      lo = wave_all(lo, [](float x, float y) { return x < y ? x : y; });
      hi = wave_all(hi, [](float x, float y) { return x > y ? x : y; });
      const bool nothing = degenerate(lo, hi, cnt);
      Best best = none;
      if (!nothing) {
        Cand cd[CPL];
        float e[CPL];
        make_cands<CPL>(lo, hi, fa, fb, a.qmax, cd, e);
        accumulate_list<CPL>(list, cnt, cd, e);
        best = pick<CPL>(cd, e, ncand, lane);
      }
      wave_lds_fence();                            // the list is rewritten for the next group
      store_choice(a, row, gi, best, lane);
      uint8_t *crow = a.codes + (size_t)row * a.d_in + c0;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int c = t * 64 + lane;
        const uint8_t q = (nothing || ((weak_bits >> t) & 1u)) ? (uint8_t)0 : code_of((float)cur[t], best, a.qmax);
        if (c < len) crow[c] = q;
      }
#pragma unroll
      for (int t = 0; t < NT; ++t) cur[t] = nxt[t];
      row = nrow;
      gi = ngi;
    }
  } else {
    for (int uu = 0; uu < n_units; ++uu) {
      const int c0 = gi * a.g;
      const int len = a.d_in - c0 < a.g ? a.d_in - c0 : a.g;
      const _Float16 *wrow = a.w + (size_t)row * a.d_in;
      // least and greatest non-weak weight
      float lo = INFINITY, hi = -INFINITY;
      int kept = 0;
      for (int o = 0; o < len; o += kChunk) {
        const int cnt = stage(wrow, c0 + o, len - o < kChunk ? len - o : kChunk, list, mask, lane);
        kept += cnt;
        for (int e = lane; e < cnt; e += 64) {
          const float v = list[e];
          lo = v < lo ? v : lo;
          hi = v > hi ? v : hi;
        }
        wave_lds_fence();
      }
      lo = wave_all(lo, [](float x, float y) { return x < y ? x : y; });
      hi = wave_all(hi, [](float x, float y) { return x > y ? x : y; });
      const bool nothing = degenerate(lo, hi, kept);
      Best best = none;
      if (!nothing) {
        Cand cd[CPL];
        float e[CPL];
        make_cands<CPL>(lo, hi, fa, fb, a.qmax, cd, e);
        for (int o = 0; o < len; o += kChunk) {
          const int cnt = stage(wrow, c0 + o, len - o < kChunk ? len - o : kChunk, list, mask, lane);
          accumulate_list<CPL>(list, cnt, cd, e);
          wave_lds_fence();                        // the list is rewritten by the next pass
        }
        best = pick<CPL>(cd, e, ncand, lane);
      }
      store_choice(a, row, gi, best, lane);
      // the codes of the group under the chosen step size and zero point; 0 at weak columns
      uint8_t *crow = a.codes + (size_t)row * a.d_in;
      for (int c = c0 + lane; c < c0 + len; c += 64)
        crow[c] = (nothing || is_weak(mask, c)) ? (uint8_t)0 : code_of((float)wrow[c], best, a.qmax);
      if (++gi == a.n_groups) {
        gi = 0;
        ++row;
      }
    }
  }
}

typedef void (*search_fn)(const SearchArgs);
template <int CPL>
search_fn pick_nt(int g) {
  if (g <= 128) return owq_search_kernel<CPL, 2>;
  if (g <= 256) return owq_search_kernel<CPL, 4>;
  if (g <= 512) return owq_search_kernel<CPL, 8>;
  if (g <= kChunk) return owq_search_kernel<CPL, 16>;
  return owq_search_kernel<CPL, 0>;
}

}  // namespace
}  // namespace owq

extern "C" owq_status_t owq_search_config(const owq_search_desc_t *d, const uint16_t *w, const int32_t *weak_idx,
                                          uint16_t *scale, uint16_t *zero, uint8_t *codes, float *err,
                                          int32_t *choice, void *stream) {
  using namespace owq;
  if (!d || !w || !scale || !zero || !codes) return OWQ_ERR_NULL;
  if (d->d_out < 1 || d->d_in < 1) return OWQ_ERR_SHAPE;
  if (d->bits != 3 && d->bits != 4) return OWQ_ERR_BITS;
  if (d->group_size < 0 || d->group_size % 128 != 0) return OWQ_ERR_GROUP;
  if (d->k < 0 || d->k > d->d_in) return OWQ_ERR_INDEX;
  if (d->k > 0 && !weak_idx) return OWQ_ERR_NULL;
  if (d->n_lo < 1 || d->n_lo > 16 || d->n_hi < 1 || d->n_hi > 16) return OWQ_ERR_SHAPE;
  if (!(d->shrink >= 0.f && d->shrink < 0.5f)) return OWQ_ERR_SHAPE;
  const int g = d->group_size == 0 || d->group_size > d->d_in ? d->d_in : d->group_size;
  const long long n_groups = (d->d_in + (long long)g - 1) / g;
  const long long units = n_groups * d->d_out;
  if (units > 0x7fffffffLL) return OWQ_ERR_SHAPE;
  const size_t mask_bytes = (size_t)((d->d_in + 31) / 32) * 4;
  if (mask_bytes > (size_t)kMaskBytesMax) return OWQ_ERR_UNSUPPORTED;
  SearchArgs a;
  a.w = reinterpret_cast<const _Float16 *>(w);
  a.weak_idx = weak_idx;
  a.scale = scale;
  a.zero = zero;
  a.codes = codes;
  a.err = err;
  a.choice = choice;
  a.d_in = d->d_in;
  a.g = g;
  a.n_groups = (int)n_groups;
  a.k = d->k;
  a.n_lo = d->n_lo;
  a.n_hi = d->n_hi;
  a.units = (int)units;
  // several groups per wave once there are enough waves to fill the chip many times over: the
  // per-lane grid set-up is then paid once per wave
  long long upw = units / 32768;
  a.units_per_wave = (int)(upw < 1 ? 1 : (upw > 16 ? 16 : upw));
  a.qmax = (float)((1 << d->bits) - 1);
  a.shrink = d->shrink;
  const long long waves = (units + a.units_per_wave - 1) / a.units_per_wave;
  const dim3 grid((unsigned)((waves + kWaves - 1) / kWaves)), block(kWaves * 64);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int ncand = d->n_lo * d->n_hi;
  const search_fn fn = ncand <= 64 ? pick_nt<1>(g) : ncand <= 128 ? pick_nt<2>(g) : ncand <= 192 ? pick_nt<3>(g) : pick_nt<4>(g);
  hipLaunchKernelGGL(fn, grid, block, mask_bytes, st, a);
  return hipGetLastError() == hipSuccess ? OWQ_OK : OWQ_ERR_HIP;
}
