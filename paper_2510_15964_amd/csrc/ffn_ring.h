// The global -> LDS transfer ring shared by the 16-bit FFN, predictor and LoRA kernels (gfx950).
//
// Data movement: global memory -> LDS directly (global_load_lds, 16 bytes per lane, no registers
// in between), a ring of stages; the loads of the next K-steps are in flight while the MFMAs of
// the current one run.  LDS rows are 128 bytes (one 64-element K-chunk of one row), unpadded (a
// DMA instruction writes 1 KiB = 8 rows contiguously); the 16-byte slots of a row are
// XOR-swizzled with the row index so that the MFMA operand reads of 16 consecutive rows hit
// distinct banks.
#pragma once
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kFW = 8;             // wavefronts per workgroup
constexpr int kNI = 8 / kFW;       // 32-row groups of the 256 weight rows per wavefront
constexpr int kThreads = kFW * kWave;
constexpr int kBK = 64;            // K-chunk per step: 64 bf16 = 128 bytes per row
constexpr int kRowsB = 64;         // shared operand (token rows)
constexpr int kRowsA = 256;        // per-wave operand (4 x 64 weight rows)
constexpr int kStageRows = kRowsA + kRowsB;
constexpr int kStageElems = kStageRows * kBK;                 // 20480 elements = 40 KiB
constexpr int kIssues = kStageRows / 8 / (kThreads / kWave);  // DMA instructions per wave per stage
// Ring depths.  Measured on the 11 %-dense FFN of the benchmark: a fourth stage (all 160 KiB of
// LDS) does not help the sdd kernels, and the dsd kernel is faster with two resident
// workgroups of two stages each than with one workgroup of three or four.
constexpr int kSddStages = 3, kDsdStages = 2;

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// One stage = NISS DMA instructions per wave (kIssues for the 64 + 256 rows of the FFN kernels).
// Instruction u of wave w fills stage rows 8g .. 8g+7 with g = w + kFW*u (g < 8: the 64 shared
// rows, then the weight blocks); lane l brings the 16-byte slot l%8 of row 8g + l/8.  src[u]
// already points at this lane's (row, swizzled segment); offB / offA are the element offsets of
// the current K-step for the shared rows (the first NSH instructions of a wave) and the weight
// rows.
// With `alt` (wave-uniform) the source of instruction u is alt_ptr(u) instead: a step whose
// operands live in other buffers with another row stride (the LoRA branch).  alt_ptr is
// evaluated only then, so such a step costs no registers in the steady state.
template <int NISS, int NSH, class AltPtr>
__device__ __forceinline__ void issue_stage(uint16_t* stage, const uint16_t* const (&src)[NISS],
                                            AltPtr alt_ptr, bool alt, long long offB,
                                            long long offA) {
  const uint32_t base = lds_addr(stage) + (threadIdx.x / kWave) * 1024;
  if (alt) {
#pragma unroll
    for (int u = 0; u < NISS; ++u) dma16(alt_ptr(u), base + u * (kFW * 1024));
  } else {
#pragma unroll
    for (int u = 0; u < NISS; ++u)
      dma16(src[u] + (u < NSH ? offB : offA), base + u * (kFW * 1024));
  }
}
struct NoAlt {
  __device__ __forceinline__ const uint16_t* operator()(int) const { return nullptr; }
};

// One 64-deep K-step from LDS: wave w multiplies its 32*kNI weight rows (row groups kNI*w ..)
// with the 64 shared rows.  acc[ni][ti]: rows = weight rows 32*(kNI*w + ni).., columns = shared
// rows 32ti..
template <int DT>
__device__ __forceinline__ void mma_step(const uint16_t* stage, int wave, f32x16 (&acc)[kNI][2]) {
  const int lane = threadIdx.x % kWave;
  const int r = lane % 32, h2 = lane / 32;
  // all operand reads of the step are issued first, so that their LDS latency overlaps the
  // MFMAs instead of being paid once per k16 slice
  uint4 a[4][kNI], b[4][2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int seg = 2 * kk + h2;
#pragma unroll
    for (int ni = 0; ni < kNI; ++ni) {
      const int ra = kRowsB + 32 * (kNI * wave + ni) + r;
      a[kk][ni] = *reinterpret_cast<const uint4*>(stage + ra * kBK + ((seg ^ swz(ra)) << 3));
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int rb = 32 * h + r;
      b[kk][h] = *reinterpret_cast<const uint4*>(stage + rb * kBK + ((seg ^ swz(rb)) << 3));
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // keep the reads above: the scheduler would sink them
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
#pragma unroll
    for (int ni = 0; ni < kNI; ++ni)
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) acc[ni][ti] = mfma32<DT>(a[kk][ni], b[kk][ti], acc[ni][ti]);
}

// The same for a stage of 64*TT shared rows (TT = 2 or 4 token tiles) + 256 weight rows and a
// wave tile of 64 weight rows (group rg of four) x 32*TT shared rows (half th of them): half
// (TT = 2) or three eighths (TT = 4) of the LDS bytes per product of the 32 x 64 tile above.
// acc[ni][ti]: weight rows 64*rg + 32*ni.., shared rows 32*TT*th + 32*ti..
template <int TT>
struct MultiStage {
  static constexpr int kShared = kRowsB * TT;
  static constexpr int kElems = (kShared + kRowsA) * kBK;   // 48 / 64 KiB
  static constexpr int kIss = (kShared + kRowsA) / 8 / kFW; // DMA instructions per wave and stage
  static constexpr int kStages = TT == 2 ? 3 : 2;           // what fits 160 KiB of LDS
};
template <int DT, int TT>
__device__ __forceinline__ void mma_step64(const uint16_t* stage, int rg, int th,
                                           f32x16 (&acc)[2][TT]) {
  const int lane = threadIdx.x % kWave;
  const int r = lane % 32, h2 = lane / 32;
  // operands of two k16 slices at a time: 8 + 4*TT registers of reads in flight
#pragma unroll
  for (int k2 = 0; k2 < 2; ++k2) {
    uint4 a[2][2], b[2][TT];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int seg = 2 * (2 * k2 + e) + h2;
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int ra = MultiStage<TT>::kShared + 64 * rg + 32 * ni + r;
        a[e][ni] = *reinterpret_cast<const uint4*>(stage + ra * kBK + ((seg ^ swz(ra)) << 3));
      }
#pragma unroll
      for (int ti = 0; ti < TT; ++ti) {
        const int rb = 32 * TT * th + 32 * ti + r;
        b[e][ti] = *reinterpret_cast<const uint4*>(stage + rb * kBK + ((seg ^ swz(rb)) << 3));
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // keep the reads above: the scheduler would sink them
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mfma32<DT>(a[e][ni], b[e][ti], acc[ni][ti]);
  }
}

// Pipeline over nsteps K-steps through a ring of NST stages: while step s is multiplied, the
// DMA of steps s+1 .. s+NST-1 is in flight (what bounds these kernels is how many bytes a CU
// keeps in flight towards memory, so the ring is as deep as LDS allows).  offs(s, offB, offA)
// yields the element offsets of step s.  A wave first waits until its own DMA of step s has
// landed (its loads retire in order, so the loads of the younger steps may stay outstanding),
// the barrier then guarantees that the whole stage is there and that nobody still reads the
// stage about to be refilled.
// Wait until at most NISS * y DMA instructions are outstanding, for a run-time y <= M (the last
// steps of a ring, when fewer stages than its depth are in flight).
template <int NISS, int M>
__device__ __forceinline__ void wait_tail(int y) {
  if constexpr (M <= 0) {
    wait_vmcnt<0>();
  } else {
    if (y == M)
      wait_vmcnt<NISS * M>();
    else
      wait_tail<NISS, M - 1>(y);
  }
}

// step(stage pointer) is the multiplication of one landed stage; a stage holds SE elements.
// offs(s, offB, offA) yields the element offsets of step s and returns whether the step takes
// its operands from alt_ptr(u).
template <int NST, int NISS, int SE, int NSH = 1, class AltPtr, class Offs, class Step>
__device__ __forceinline__ void run_ring_of(int nsteps, const uint16_t* const (&src)[NISS],
                                            AltPtr alt_ptr, Offs offs, uint16_t* ring, Step step) {
  static_assert(NST >= 2 && NISS * (NST - 2) < 64, "ring depth");
  long long ob, oa;
  auto issue = [&](int s, int stage) {
    const bool alt = offs(s, ob, oa);
    issue_stage<NISS, NSH>(ring + stage * SE, src, alt_ptr, alt, ob, oa);
  };
#pragma unroll
  for (int p = 0; p < NST - 1; ++p)
    if (p < nsteps) issue(p, p);
  int stage = 0;
  for (int s = 0; s < nsteps; ++s) {
    const int younger = nsteps - 1 - s;   // steps after s whose DMA has been issued: min(., NST-2)
    if (younger >= NST - 2)
      wait_vmcnt<NISS * (NST - 2)>();
    else
      wait_tail<NISS, NST - 3>(younger);
    lds_barrier();
    if (s + NST - 1 < nsteps) issue(s + NST - 1, stage == 0 ? NST - 1 : stage - 1);
    step(ring + stage * SE);
    stage = stage + 1 == NST ? 0 : stage + 1;
  }
}

template <int DT, int NST, class AltPtr, class Offs>
__device__ __forceinline__ void run_ring(int nsteps, bool wave_on,
                                         const uint16_t* const (&src)[kIssues], AltPtr alt_ptr,
                                         Offs offs, uint16_t* ring, f32x16 (&acc)[kNI][2]) {
  const int wave = threadIdx.x / kWave;
  run_ring_of<NST, kIssues, kStageElems>(nsteps, src, alt_ptr, offs, ring,
                                         [&](const uint16_t* stage) {
                                           if (wave_on) mma_step<DT>(stage, wave, acc);
                                         });
}

// Host side: calls fn<kF16> or fn<kBf16> according to the run-time element type `dt`.
#define LX_BY_DT(fn, ...) (dt == kF16 ? fn<kF16>(__VA_ARGS__) : fn<kBf16>(__VA_ARGS__))

}  // namespace lx
