// Device-side helpers shared by the GEMV and the tile kernels: vector types, the packed
// dot product, and the mask-and-OR unpack of pairs of codes into fp16 mantissas.
#pragma once
#include <hip/hip_runtime.h>

namespace owq {

typedef unsigned int u32;
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));   // native vector: 16-byte loads

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

__device__ __forceinline__ float half_lo(u32 w) {
  return (float)__builtin_bit_cast(h2_t, w)[0];
}
__device__ __forceinline__ float half_hi(u32 w) {
  return (float)__builtin_bit_cast(h2_t, w)[1];
}

// Sum over the 16 lanes of a row of the wave (every lane gets the total), in a fixed order.
__device__ __forceinline__ float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, false));   // lanes ^1
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, false));   // lanes ^2
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, false));  // mirror in 8
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xf, 0xf, false));  // mirror in 16
  return v;
}

// Sum over CW = 16, 32 or 64 consecutive lanes (a tile row of CW blocks), in a fixed order.  The
// total is valid in the last 16 lanes of each group of CW lanes.
template <int CW>
__device__ __forceinline__ float tile_row_sum(float v) {
  v = row16_sum(v);
  if (CW >= 32)   // lane 15 of rows 0 and 2 of the wave added to rows 1 and 3
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xa, 0xf, false));
  if (CW >= 64)   // lane 31 added to rows 2 and 3
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xc, 0xf, false));
  return v;
}

}  // namespace owq
