// Inference side of the MLP predictor (Sec. V-A) for gfx950: block scores on the MFMA, threshold
// and reduction over a group of tokens fused into the epilogue.  Templates over the 16-bit
// element type like the FFN kernels, whose transfer ring they share.
#include "ffn_ring.h"

namespace lx {

// MLP predictor (Sec. V-A): scores S = X Wa for one 64-token tile and NB groups of 64 neuron
// blocks (rows of Wa_t [nblk, K]), thresholded and OR-reduced over the tokens of a group of
// tiles_per_group tiles: mask[i / tiles_per_group][n] = 1 if any token t of tile i has
// S[t][n] > thr.  The mask has been zeroed before; workgroups only ever store ones, so the
// stores of the tiles of a group to the same byte need no ordering.  Same DMA ring as the sdd
// kernel with 64 + 64*NB rows per stage; the 4*NB accumulator tiles (32 blocks x 32 tokens)
// are dealt to the eight wavefronts (two each for NB = 4, else one; NB = 1 leaves four
// wavefronts with the transfers only).  NB is chosen by the host so that the grid fills the
// chip when nblk is small.
template <int DT, int NB>
__global__ __launch_bounds__(kThreads) void predict_bf16(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wa_t, int tiles, int K, int nblk,
    int tiles_per_group, float thr, uint8_t* __restrict__ mask) {
  constexpr int kSE = (kRowsB + 64 * NB) * kBK;   // stage elements
  constexpr int kNIss = 1 + NB;                   // DMA instructions per wave and stage
  constexpr int kTPW = NB == 4 ? 2 : 1;           // accumulator tiles per wavefront
  // few workgroups, each with little arithmetic per byte: what bounds the small variants is the
  // number of bytes in flight, so their rings take most of the LDS
  constexpr int kNSt = NB == 1 ? 8 : NB == 2 ? 6 : kSddStages;
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kNSt * kSE];
  // Workgroup w runs on XCD w % 8: the workgroups of one token tile (one per chunk of NB groups
  // of rows of Wa_t) are given the same XCD, so the tile's tokens reach one L2 only.
  const int nchunk = nblk / (64 * NB), slot = blockIdx.x / 8;
  const int i = (slot / nchunk) * 8 + blockIdx.x % 8;   // token tile
  const int c0 = (slot % nchunk) * NB;                  // first group of 64 rows of Wa_t
  if (i >= tiles) return;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const uint16_t* src[kNIss];
#pragma unroll
  for (int u = 0; u < kNIss; ++u) {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u == 0)
      src[u] = X + ((long long)i * 64 + row) * K + seg * 8;
    else
      src[u] = Wa_t + ((long long)c0 * 64 + row - kRowsB) * K + seg * 8;
  }
  // tile idx of the workgroup: 32 rows of Wa_t (idx / 2) x 32 tokens (idx % 2)
  const int idx0 = wave * kTPW;
  const bool on = idx0 < 4 * NB;
  const int rgrp = idx0 / 2, r = lane % 32, h2 = lane / 32;
  f32x16 acc[kTPW];
#pragma unroll
  for (int t = 0; t < kTPW; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  run_ring_of<kNSt, kNIss, kSE>(
      K / kBK, src, NoAlt(),
      [](int s, long long& ob, long long& oa) {
        ob = oa = (long long)s * kBK;
        return false;
      },
      ring,
      [&](const uint16_t* stage) {
        if (!on) return;
        uint4 a[4], b[4][kTPW];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int seg = 2 * kk + h2, ra = kRowsB + 32 * rgrp + r;
          a[kk] = *reinterpret_cast<const uint4*>(stage + ra * kBK + ((seg ^ swz(ra)) << 3));
#pragma unroll
          for (int t = 0; t < kTPW; ++t) {
            const int rb = 32 * ((idx0 + t) % 2) + r;
            b[kk][t] = *reinterpret_cast<const uint4*>(stage + rb * kBK + ((seg ^ swz(rb)) << 3));
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int t = 0; t < kTPW; ++t) acc[t] = mfma32<DT>(a[kk], b[kk][t], acc[t]);
      });
  if (!on) return;
  uint8_t* out = mask + (long long)(i / tiles_per_group) * nblk + c0 * 64 + 32 * rgrp;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    // register v of a lane: block 8*(v/4) + 4*(lane/32) + v%4 of the 32, token lane%32
    bool mine = acc[0][v] > thr;
    if (kTPW == 2) mine = mine || acc[kTPW - 1][v] > thr;
    const unsigned long long hit = __ballot(mine);
    const int n = 8 * (v / 4) + v % 4;
    if (lane == 0 && (uint32_t)hit != 0u) out[n] = 1;
    if (lane == 32 && (hit >> 32) != 0ull) out[n + 4] = 1;
  }
}

// Finer variant for so few neuron blocks that even one group of 64 rows of Wa_t per workgroup
// leaves CUs idle: a workgroup takes 32 rows of Wa_t, and a step covers two 64-wide chunks of K
// (64 + 64 token-rows and 32 + 32 rows of Wa_t per stage: three DMA instructions per wave).  The
// 2 x 8 products of a step (token half x k16 slice) are dealt to the eight wavefronts, which sum
// over disjoint parts of K; the four partial sums of a token half are added in a fixed order
// through LDS before the threshold.  Requires K % 128 == 0.
template <int DT>
__global__ __launch_bounds__(kThreads) void predict_half_bf16(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wa_t, int tiles, int K, int nblk,
    int tiles_per_group, float thr, uint8_t* __restrict__ mask) {
  constexpr int kSE = 192 * kBK, kNIss = 3, kNSt = 6;
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kNSt * kSE];
  const int nchunk = nblk / 32, slot = blockIdx.x / 8;
  const int i = (slot / nchunk) * 8 + blockIdx.x % 8;   // token tile; its workgroups share an XCD
  const int r0 = (slot % nchunk) * 32;                  // first row of Wa_t
  if (i >= tiles) return;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const uint16_t* src[kNIss];
#pragma unroll
  for (int u = 0; u < kNIss; ++u) {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;   // stage row 0 .. 191
    const int seg = (lane % 8) ^ swz(row);
    if (u < 2) {
      src[u] = X + ((long long)i * 64 + row - 64 * u) * K + 64 * u + seg * 8;
    } else {
      const int wr = row - 128;                              // 0 .. 63: chunk wr / 32, row wr % 32
      src[u] = Wa_t + ((long long)r0 + wr % 32) * K + 64 * (wr / 32) + seg * 8;
    }
  }
  const int ti = wave % 2, chunk = (wave / 2) % 2, kh = wave / 4;
  const int r = lane % 32, h2 = lane / 32;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  run_ring_of<kNSt, kNIss, kSE>(
      K / (2 * kBK), src, NoAlt(),
      [](int s, long long& ob, long long& oa) {
        ob = oa = (long long)s * (2 * kBK);
        return false;
      },
      ring,
      [&](const uint16_t* stage) {
        uint4 a[2], b[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int seg = 2 * (2 * kh + e) + h2;
          const int ra = 128 + 32 * chunk + r, rb = 64 * chunk + 32 * ti + r;
          a[e] = *reinterpret_cast<const uint4*>(stage + ra * kBK + ((seg ^ swz(ra)) << 3));
          b[e] = *reinterpret_cast<const uint4*>(stage + rb * kBK + ((seg ^ swz(rb)) << 3));
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) acc = mfma32<DT>(a[e], b[e], acc);
      });
  // partial sums of wavefronts 2 .. 7 -> LDS; wavefronts 0, 1 add those of their token half
  float* red = reinterpret_cast<float*>(ring);
  lds_barrier();
  if (wave >= 2) {
#pragma unroll
    for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * kWave + lane] = acc[v];
  }
  lds_barrier();
  if (wave >= 2) return;
#pragma unroll
  for (int p = 1; p < 4; ++p)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += red[((wave + 2 * p) * 16 + v) * kWave + lane];
  uint8_t* out = mask + (long long)(i / tiles_per_group) * nblk + r0;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    // register v of a lane: row 8*(v/4) + 4*(lane/32) + v%4 of the 32, token 32*ti + lane%32
    const unsigned long long hit = __ballot(acc[v] > thr);
    const int n = 8 * (v / 4) + v % 4;
    if (lane == 0 && (uint32_t)hit != 0u) out[n] = 1;
    if (lane == 32 && (hit >> 32) != 0ull) out[n + 4] = 1;
  }
}

__global__ void zero_bytes_kernel(uint8_t* __restrict__ p, int n) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) p[idx] = 0;
}

// mask: [T/64/tiles_per_group][nblk] bytes
template <int DT>
static hipError_t launch_predict_bf16_t(int T, int d, int nblk, int tiles_per_group, const uint16_t* X,
                               const uint16_t* Wa_t, float thr, uint8_t* mask, hipStream_t st) {
  const int Tt = T / 64, total = Tt / tiles_per_group * nblk, ng = nblk / 64;
  hipLaunchKernelGGL(zero_bytes_kernel, dim3((total + 255) / 256), dim3(256), 0, st, mask, total);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the widest workgroup (least re-reading of X) that still gives every CU a workgroup
  ProfScope ps(kKPredict, st);
  const int T8 = (Tt + 7) / 8 * 8;   // grid: 8 XCDs x chunks x ceil(Tt / 8) tiles
  if (ng % 4 == 0 && (long long)ng / 4 * Tt >= kCUs)
    hipLaunchKernelGGL((predict_bf16<DT, 4>), dim3(ng / 4 * T8), dim3(kThreads), 0, st, X, Wa_t, Tt, d,
                       nblk, tiles_per_group, thr, mask);
  else if (ng % 2 == 0 && (long long)ng / 2 * Tt >= kCUs)
    hipLaunchKernelGGL((predict_bf16<DT, 2>), dim3(ng / 2 * T8), dim3(kThreads), 0, st, X, Wa_t, Tt, d,
                       nblk, tiles_per_group, thr, mask);
  else if ((long long)ng * Tt < kCUs && d % 128 == 0)
    hipLaunchKernelGGL(predict_half_bf16<DT>, dim3(2 * ng * T8), dim3(kThreads), 0, st, X, Wa_t, Tt, d,
                       nblk, tiles_per_group, thr, mask);
  else
    hipLaunchKernelGGL((predict_bf16<DT, 1>), dim3(ng * T8), dim3(kThreads), 0, st, X, Wa_t, Tt, d, nblk,
                       tiles_per_group, thr, mask);
  return hipGetLastError();
}

hipError_t launch_predict_bf16(int dt, int T, int d, int nblk, int tiles_per_group, const uint16_t* X,
                               const uint16_t* Wa_t, float thr, uint8_t* mask, hipStream_t st) {
  return LX_BY_DT(launch_predict_bf16_t, T, d, nblk, tiles_per_group, X, Wa_t, thr, mask, st);
}

}  // namespace lx
