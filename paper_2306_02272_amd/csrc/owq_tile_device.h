// Device-side pieces shared by the kernels of the tile layout: operand types of the
// 32x32x16 fp16 matrix instruction, the place of every pair of codes inside its 16-bit
// window, and the A operand made straight from a lane's dwords of codes.
#pragma once
#include <hip/hip_runtime.h>

#include "owq_device.h"

namespace owq {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf8_t __attribute__((ext_vector_type(8)));
typedef float f16_t __attribute__((ext_vector_type(16)));
typedef float f4_t __attribute__((ext_vector_type(4)));
typedef float f2_t __attribute__((ext_vector_type(2)));

constexpr int kUnitsPerTile = 2048;   // 16-byte units of one staged activation tile (256 columns x 64 tokens)

// Bit offset o of pair i (columns 2i, 2i+1) of octet t of a block inside its 16-bit window;
// the pair is OR-ed into 2^(10-o).  3-bit: the octet's place in its quad of 32 codes decides.
__device__ __forceinline__ constexpr int pair_offset(int bits, int t, int i) {
  constexpr int off3[4][4] = {{0, 3, 6, 1}, {4, 7, 2, 5}, {0, 3, 6, 1}, {4, 7, 4, 7}};
  constexpr int off4[4] = {0, 4, 2, 6};
  return bits == 3 ? off3[t & 3][i] : off4[i];
}

// A operand of k-step S (16 columns) from the lane's dwords: four packed pairs 2^(10-o)+q.
template <int BITS, int S>
__device__ __forceinline__ h8_t a_operand(const u32 *wd, const Magic &M) {
  u32 r0, r1, r2, r3;
  if (BITS == 3) {
    constexpr int u = S >> 2, o = S & 3;
    const u32 d0 = wd[3 * u], d1 = wd[3 * u + 1], d2 = wd[3 * u + 2];
    if (o == 0) {
      const u32 w1 = __builtin_amdgcn_perm(d1, d0, 0x06030401u);
      r0 = andor(d0, field(3, 0), M.m[0]); r1 = andor(d0, field(3, 3), M.m[3]);
      r2 = andor(d0, field(3, 6), M.m[6]); r3 = andor(w1, field(3, 1), M.m[1]);
    } else if (o == 1) {
      const u32 w1 = __builtin_amdgcn_perm(d1, d0, 0x06030401u);
      r0 = andor(w1, field(3, 4), M.m[4]); r1 = andor(w1, field(3, 7), M.m[7]);
      r2 = andor(d1, field(3, 2), M.m[2]); r3 = andor(d1, field(3, 5), M.m[5]);
    } else if (o == 2) {
      const u32 w3 = __builtin_amdgcn_perm(d2, d1, 0x06030401u);
      r0 = andor(w3, field(3, 0), M.m[0]); r1 = andor(w3, field(3, 3), M.m[3]);
      r2 = andor(w3, field(3, 6), M.m[6]); r3 = andor(d2, field(3, 1), M.m[1]);
    } else {
      const u32 w5 = d2 >> 6;
      r0 = andor(d2, field(3, 4), M.m[4]); r1 = andor(d2, field(3, 7), M.m[7]);
      r2 = andor(w5, field(3, 4), M.m[4]); r3 = andor(w5, field(3, 7), M.m[7]);
    }
  } else {
    const u32 d = wd[S], w = d >> 6;
    r0 = andor(d, field(4, 0), M.m[0]); r1 = andor(d, field(4, 4), M.m[4]);
    r2 = andor(w, field(4, 2), M.m[2]); r3 = andor(w, field(4, 6), M.m[6]);
  }
  const u32x4 v = {r0, r1, r2, r3};
  return __builtin_bit_cast(h8_t, v);
}

__device__ __forceinline__ f16_t mma(h8_t a, h8_t b, f16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

}  // namespace owq
