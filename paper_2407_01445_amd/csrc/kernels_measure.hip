// Measurement kernels (not on the step's path): what the matrix cores of this part deliver when nothing else is in
// the way, in the launch shape of the strip kernel.  fastclip_measure_mfma_ceiling runs it and reports the rate, so
// that the MFMA kernels can be priced against a measured ceiling next to the published one.
#include "mfma_common.hpp"

namespace fc {

// 8 waves per workgroup, two per SIMD, each with the strip kernel's 2 x 4 accumulator blocks (128 accumulator
// registers) and register operands that never change: `iters` rounds of 8 independent MFMAs 32x32x16 bf16, no memory
// traffic, no LDS, no barrier.  Operands are pseudo-random bf16 values of magnitude below 1 (the clock under load
// depends on the operand bits: all-zero operands run faster).  out[wave] = {shader cycles, 100 MHz ticks} of the wave's
// loop; the accumulators are written out only if a value is NaN, which cannot happen, to keep them alive.
__global__ void __launch_bounds__(512, 2) k_mfma_ceiling(int iters, uint64_t* __restrict__ out, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16x8 a[2], b[4];
  uint32_t h = (uint32_t)(blockIdx.x * 512 + threadIdx.x) * 2654435761u + 12345u;
  auto next = [&]() {
    h = h * 1664525u + 1013904223u;
    // sign and 7 mantissa bits random, exponent 2^-1 .. 2^-4
    const uint32_t bits = ((h >> 16) & 0x807fu) | ((uint32_t)(123 + ((h >> 9) & 3)) << 7);
    return __builtin_bit_cast(__bf16, (uint16_t)bits);
  };
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) a[i][e] = next();
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) b[i][e] = next();
  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  __syncthreads();
  const uint64_t c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  const uint64_t c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  if (s != s) sink[threadIdx.x] = s;
  if (lane == 0) {
    out[((size_t)blockIdx.x * 8 + wave) * 2 + 0] = c1 - c0;
    out[((size_t)blockIdx.x * 8 + wave) * 2 + 1] = w1 - w0;
  }
}

// What the memory system delivers for the access pattern of the state phase on 32-byte records with nothing else in
// the way: n distinct random records of `stride` floats each, the two 16-byte halves of a record read, changed by one
// multiply-add and written back by two neighbouring lanes.  No sums, no outputs, no transcendental arithmetic.
__global__ void __launch_bounds__(256) k_record_rmw(const int64_t* __restrict__ idx, int64_t n, float* __restrict__ rec,
                                                    int64_t stride) {
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < 2 * n; t += (int64_t)gridDim.x * 256) {
    float4* p = (float4*)(rec + idx[t >> 1] * stride + 4 * (t & 1));
    float4 w = *p;
    w.x = fmaf(0.5f, w.x, 0.25f); w.y = fmaf(0.5f, w.y, 0.25f); w.z = fmaf(0.5f, w.z, 0.25f); w.w = fmaf(0.5f, w.w, 0.25f);
    *p = w;
  }
}

void launch_record_rmw(const int64_t* idx, int64_t n, float* rec, int64_t stride, hipStream_t s) {
  const int64_t blocks = (2 * n + 255) / 256;
  hipLaunchKernelGGL(k_record_rmw, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, s, idx, n, rec, stride);
}

void launch_mfma_ceiling(int workgroups, int iters, uint64_t* out, float* sink, hipStream_t s) {
  hipLaunchKernelGGL(k_mfma_ceiling, dim3((unsigned)workgroups), dim3(512), 0, s, iters, out, sink);
}

}  // namespace fc
