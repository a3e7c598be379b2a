// Measurement aids: what the chip sustains on the two resources the operators are priced
// against, measured with the library's own means so that a benchmark can state fractions of a
// measured peak next to fractions of the data-sheet one.  No part of the operators of Sec. VI.
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

// Dense MFMA rate: every wavefront issues `iters` rounds of eight independent 32x32x16 bf16
// MFMAs on registers (no memory traffic); 2 * 32*32*16 FLOP each.  Four wavefronts per SIMD.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x % kWave;
  // operand bits are irrelevant for the rate; small finite values keep the sums finite
  const uint32_t w = 0x3C003C00u + (uint32_t)lane;
  const uint4 a = make_uint4(w, w, w, w), b = make_uint4(w ^ 0x80008000u, w, w ^ 0x80008000u, w);
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = mfma32<kBf16>(a, b, acc[i]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop; never true in practice
}

// Stream copy, 16 bytes per lane and access, grid-stride: dst[i] = src[i] over n 16-byte units.
__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  // four loads in flight per lane before the first store
  for (; i + 3 * stride < n; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n; i += stride) dst[i] = src[i];
}

constexpr int kProbeWgs = kCUs * 4;   // 4 workgroups of 4 wavefronts per CU: 4 wavefronts per SIMD

hipError_t launch_probe_mfma(int iters, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeWgs), dim3(256), 0, st, iters, sink);
  return hipGetLastError();
}
// FLOP one launch of the MFMA probe performs
double probe_mfma_flops(int iters) {
  return (double)kProbeWgs * 4 * (double)iters * 8 * 2.0 * 32 * 32 * 16;
}
hipError_t launch_probe_copy(const void* src, void* dst, long long units16, hipStream_t st) {
  hipLaunchKernelGGL(probe_copy_kernel, dim3(kCUs * 8), dim3(256), 0, st, (const uint4*)src,
                     (uint4*)dst, units16);
  return hipGetLastError();
}

}  // namespace lx
