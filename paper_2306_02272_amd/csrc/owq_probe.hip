// Measurement aids for the benchmark: the time of a pure 128-bit read of the same bytes a layer
// kernel streams, and of a launch that does nothing, on the same stream and in the same launch
// mode as the layer kernels (the context lines beside the layer's own figures).
#include <hip/hip_runtime.h>

#include "owq_device.h"
#include "owq_internal.h"
#include "owq_tile_device.h"

namespace owq {

__device__ u32 g_probe_sink;

// Workgroup b reads 16-byte units [b * per, (b + 1) * per) of p, UNROLL loads of a lane in
// flight; reads past the slab's end re-read its last unit.  With out != nullptr the workgroup
// then writes its share (oper units) of out16 16-byte units: a layer call also ends on a store.
template <int UNROLL>
__global__ __launch_bounds__(256) void owq_read_kernel(const u32x4 *p, u32 n16, u32 per, u32x4 *out, u32 out16, u32 oper) {
  const u32 lo = blockIdx.x * per;
  const u32 hi = min(n16, lo + per);
  if (lo >= hi) return;
  u32 acc = 0;
  for (u32 i = lo + threadIdx.x; i < hi; i += 256 * UNROLL) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const u32 j = i + (u32)u * 256u;
      v[u] = __builtin_nontemporal_load(p + (j < hi ? j : hi - 1));
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  // keeps the loads alive; the stored value is never read
  if (acc == 0x9e3779b9u && per == 0xffffffffu) g_probe_sink = acc;
  if (out != nullptr) {
    const u32 o0 = blockIdx.x * oper, o1 = min(out16, o0 + oper);
    for (u32 i = o0 + threadIdx.x; i < o1; i += 256) out[i] = (u32x4){acc, acc, acc, acc};
  }
}

// The five fp32 instructions the configuration search spends per weight and grid point (multiply,
// round to nearest, clamp, and two fused multiply-adds), on registers only: four grid points per
// lane, eight weights per trip, nothing read or written but one word at the end.  What the
// vector units can issue of exactly this mix.
__global__ __launch_bounds__(256) void owq_alu_kernel(float *out, int trips, float seed) {
  const float lane = (float)(threadIdx.x & 63);
  float inv[4], ns[4], lo[4], hi[4], err[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    inv[c] = 3.f + 0.01f * lane + (float)c;
    ns[c] = -1.f / inv[c];
    lo[c] = -(float)c;
    hi[c] = 7.f - (float)c;
    err[c] = 0.f;
  }
  float w[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) w[j] = seed * (float)(j + 1) + 0.001f * lane;
  for (int t = 0; t < trips; ++t) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(w[j] * inv[c]), lo[c], hi[c]);
        const float d = __builtin_fmaf(q, ns[c], w[j]);
        err[c] = __builtin_fmaf(d, d, err[c]);
      }
    }
    // keeps the trips apart for the compiler without adding an instruction per weight
    asm volatile("" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7]));
  }
  const float e = (err[0] + err[1]) + (err[2] + err[3]);
  if (e == -1.f) out[0] = e;          // never true (a sum of squares); keeps the loop alive
}

// The matrix instruction of the batched path on registers only: 16 of them per trip into four
// independent accumulator tiles (what one k-step of owq_tile_mma issues for its 64 rows x 64
// tokens, four times), two workgroups of four waves per compute unit as there.  What the matrix
// cores deliver of this instruction at the clock the chip holds under it.
__global__ __launch_bounds__(256, 2) void owq_mfma_kernel(float *out, int trips, float seed) {
  const float lane = (float)(threadIdx.x & 63);
  h8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (_Float16)(seed * (1.f + 0.01f * lane + 0.1f * (float)i));
    b[i] = (_Float16)(seed * (2.f - 0.01f * lane));
  }
  f16_t acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int t = 0; t < trips; ++t) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = mma(a, b, acc[i]);
    asm volatile("" : "+v"(a), "+v"(b));   // keeps the trips apart for the compiler
  }
  float e = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) e += acc[i][r];
  if (e == -1.f) out[0] = e;            // never true (sums of positive products); keeps the loop alive
}

__global__ void owq_empty_kernel(int never) {
  if (never == 0x7fffffff) g_probe_sink = 1;
}

// One launch reading `bytes` (a multiple of 16) from dev once with `workgroups` workgroups.
int launch_read(const void *dev, size_t bytes, int32_t workgroups, void *out, size_t out_bytes, void *stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return (int)hipSuccess;
  if (n16 > 0xffffffffull || workgroups < 1) return (int)hipErrorInvalidValue;
  // slabs of whole 4 KiB pieces (one 16-byte load of every lane of a workgroup)
  const u32 per = (u32)(((n16 + workgroups - 1) / workgroups + 255) / 256 * 256);
  const u32 grid = (u32)((n16 + per - 1) / per);
  const u32 out16 = out ? (u32)(out_bytes / 16) : 0u;
  hipLaunchKernelGGL(owq_read_kernel<8>, dim3(grid, 1, 1), dim3(256, 1, 1), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4 *>(dev), (u32)n16, per, static_cast<u32x4 *>(out), out16, (out16 + grid - 1) / grid);
  return (int)hipGetLastError();
}

// workgroups x 256 threads x trips x 32 (weight, grid point) pairs x 5 instructions
int launch_alu(void *dev_word, int32_t workgroups, int32_t trips, void *stream) {
  hipLaunchKernelGGL(owq_alu_kernel, dim3((unsigned)workgroups, 1, 1), dim3(256, 1, 1), 0, static_cast<hipStream_t>(stream),
                     static_cast<float *>(dev_word), trips, 0.37f);
  return (int)hipGetLastError();
}

// workgroups x 4 waves x trips x 16 matrix instructions of 2 * 32 * 32 * 16 flops
int launch_mfma(void *dev_word, int32_t workgroups, int32_t trips, void *stream) {
  hipLaunchKernelGGL(owq_mfma_kernel, dim3((unsigned)workgroups, 1, 1), dim3(256, 1, 1), 0, static_cast<hipStream_t>(stream),
                     static_cast<float *>(dev_word), trips, 0.01f);
  return (int)hipGetLastError();
}

int launch_empty(void *stream) {
  hipLaunchKernelGGL(owq_empty_kernel, dim3(256, 1, 1), dim3(256, 1, 1), 0, static_cast<hipStream_t>(stream), 0);
  return (int)hipGetLastError();
}

}  // namespace owq
