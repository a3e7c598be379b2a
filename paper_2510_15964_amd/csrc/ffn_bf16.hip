// bf16 sparse FFN kernels for gfx950 (Sec. VI-B: neuron-centric tiled matrix
// products that take the list of active neuron blocks and load / compute only
// those).  fp32 accumulation on the 32x32x16 MFMA for 16-bit operands.  The kernels are
// templates over the element type DT (bfloat16 or IEEE half, same layouts and data movement);
// "bf16" in their names dates from the first of the two.
//
// Both products of a pass are "NT" contractions whose operands are read along
// their contiguous dimension in 128-byte segments (one 64-element bf16 K-chunk
// of one row), which is what the weight layouts of Sec. VI-B are for:
//   sdd  out block (i, j) = A_i [64 x K] . W[j-block rows, :]^T, K = d
//        one workgroup owns up to four consecutive entries of token tile i's
//        list, so the A_i chunk staged in LDS is shared by four neuron blocks;
//        wave w computes block w (64 neurons) for all 64 tokens.
//   dsd  out tile (i, 256 columns) = sum over listed j of Act_ij [64 x 64] .
//        W[rows n0.., j-block columns]^T: the K loop walks the active list, one
//        64-wide K-step per active block; inactive blocks are never touched.
//
// Data movement: global memory -> LDS directly (global_load_lds, 16 bytes per
// lane, no registers in between), three 40 KiB stages; the loads of K-steps s+1
// and s+2 are in flight while the MFMAs of step s run.  The stages are separate
// LDS arrays on purpose: the compiler tracks LDS-DMA writes per array and would
// otherwise wait for the in-flight stage before every LDS read.
// LDS rows are 128 bytes, unpadded (a DMA instruction writes 1 KiB = 8 rows
// contiguously); the 16-byte slots of a row are XOR-swizzled with the row
// index so that the MFMA operand reads of 16 consecutive rows hit distinct
// banks.
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
// the current K-step for the shared rows and the weight rows.
// With `alt` (wave-uniform) the source of instruction u is alt_ptr(u) instead: a step whose
// operands live in other buffers with another row stride (the LoRA branch).  alt_ptr is
// evaluated only then, so such a step costs no registers in the steady state.
template <int NISS, class AltPtr>
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
      dma16(src[u] + (u < 8 / kFW ? offB : offA), base + u * (kFW * 1024));
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
template <int NST, int NISS, int SE, class AltPtr, class Offs, class Step>
__device__ __forceinline__ void run_ring_of(int nsteps, const uint16_t* const (&src)[NISS],
                                            AltPtr alt_ptr, Offs offs, uint16_t* ring, Step step) {
  static_assert(NST >= 2 && NISS * (NST - 2) < 64, "ring depth");
  long long ob, oa;
  auto issue = [&](int s, int stage) {
    const bool alt = offs(s, ob, oa);
    issue_stage<NISS>(ring + stage * SE, src, alt_ptr, alt, ob, oa);
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

// Work items of the sdd kernel are (token tile, group of `per` consecutive list entries),
// numbered in list order; `rows` counts token tiles, and gt consecutive tiles share one row of
// the list (gt = 1: a list row per tile).  The launch grid is the host-known upper bound on their number and
// every wavefront finds its item from row_ptr with 64-wide scans, so the active workgroups are
// the FIRST ones of the grid and spread evenly over shader engines and CUs (a 2-D grid with
// early exits piles them onto a few CUs).  Workgroup w runs on XCD w % 8; it takes item
// of the range (w % 8) * L .. + L - 1 with L = ceil(total / 8), so each XCD owns a contiguous
// range of items, i.e. of token tiles: a tile's activations are fetched into one L2 only, and
// the weight blocks an XCD needs are those of one eighth of the tiles.  Returns false past the
// end.
__device__ __forceinline__ bool find_work(const int* __restrict__ row_ptr, int rows, int gt, int w,
                                          int per, int& row, int& chunk) {
  const int lane = threadIdx.x % kWave;
  int total = 0;
  for (int base = 0; base < rows; base += kWave) {
    const int r = base + lane;
    int c = 0;
    if (r < rows) c = (row_ptr[r / gt + 1] - row_ptr[r / gt] + per - 1) / per;
#pragma unroll
    for (int dlt = 32; dlt > 0; dlt >>= 1) c += __shfl_xor(c, dlt);
    total += c;
  }
  const int L = (total + 7) / 8;
  // Inside an XCD's range consecutive workgroups are an eighth of the range apart, so the
  // workgroups that run at the same time come from different token tiles and, the lists being
  // sorted, from the same region of the neuron axis: the weight blocks that several tiles of
  // the XCD use are then fetched into its L2 once (with all blocks listed: once per eight tiles).
  const int q = (L + 7) / 8, slot = w / 8;
  const int pos = (slot % 8) * q + slot / 8, work = (w % 8) * L + pos;
  if (slot >= 8 * q || pos >= L || work >= total) return false;
  int running = 0;
  for (int base = 0; base < rows; base += kWave) {
    const int r = base + lane;
    int c = 0;
    if (r < rows) c = (row_ptr[r / gt + 1] - row_ptr[r / gt] + per - 1) / per;
    int incl = c;
#pragma unroll
    for (int dlt = 1; dlt < kWave; dlt <<= 1) {
      const int up = __shfl_up(incl, dlt);
      if (lane >= dlt) incl += up;
    }
    const int seg = __shfl(incl, kWave - 1);
    if (work < running + seg) {
      const unsigned long long hit = __ballot(running + incl > work);
      const int first = __ffsll((long long)hit) - 1;
      row = base + first;
      chunk = work - running - __shfl(incl - c, first);
      return true;
    }
    running += seg;
  }
  return false;
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[kNI][2]) {
#pragma unroll
  for (int a = 0; a < kNI; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
}

// MODE 0: out = bf16(max(acc + bias, 0));  MODE 1: out = gate > 0 ? bf16(acc) : 0;
// MODE 2: out = bf16(acc).
// LORA: one more 64-deep step after the K loop with the operands A2 [T,64] (rows of the token
// tile) and W2 [F,64] (rows of the listed blocks): acc += A2_i W2_j^T, the low-rank branch
// z = W x + B (A x) of Sec. II-C with A2 = X A^T computed beforehand and W2 = B, both padded to
// rank 64.
template <int DT, int MODE, bool LORA>
__global__ __launch_bounds__(kThreads) void ffn_sdd_bf16(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
    const uint16_t* __restrict__ bias, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int rows, int gt, int K, int nnz_cap,
    uint16_t* __restrict__ out_act, const uint16_t* __restrict__ gate_act,
    const uint16_t* __restrict__ A2, const uint16_t* __restrict__ W2) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kSddStages * kStageElems];
  int i, chunk;
  if (!find_work(row_ptr, rows, gt, blockIdx.x, 4, i, chunk)) return;
  const int rs = row_ptr[i / gt], n_i = row_ptr[i / gt + 1] - rs;
  const int first = chunk * 4;
  const int p0 = rs + first;
  if (p0 >= nnz_cap) return;       // entries beyond the capacity of the list buffers are ignored
  const int nb = min(min(4, n_i - first), nnz_cap - p0);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;

  // per-instruction source pointers of this lane (K offset added per step)
  const uint16_t* src[kIssues];
#pragma unroll
  for (int u = 0; u < kIssues; ++u) {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < 8 / kFW) {
      src[u] = A + ((long long)i * 64 + row) * K + seg * 8;
    } else {
      const int blk = g / 8 - 1, r = row - kRowsB - 64 * blk;
      // blocks past the end of the list are filled from the first block (never used)
      const int j = col_idx[p0 + (blk < nb ? blk : 0)];
      src[u] = W + ((long long)j * 64 + r) * K + seg * 8;
    }
  }
  // the same for the low-rank step (rows of 64 elements), computed when that step is issued
  auto src2 = [&](int u) -> const uint16_t* {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < 8 / kFW) return A2 + ((long long)i * 64 + row) * 64 + seg * 8;
    const int blk = g / 8 - 1, r = row - kRowsB - 64 * blk;
    const int j = col_idx[p0 + (blk < nb ? blk : 0)];
    return W2 + ((long long)j * 64 + r) * 64 + seg * 8;
  };
  f32x16 acc[kNI][2];
  zero_acc(acc);
  const int blk_w = kNI * wave / 2;          // list entry (of the four) this wave works on
  const int ksteps = K / kBK;
  run_ring<DT, kSddStages>(ksteps + (LORA ? 1 : 0), blk_w < nb, src, src2,
                       [=](int s, long long& ob, long long& oa) {
                         const bool alt = LORA && s == ksteps;
                         ob = oa = alt ? 0 : (long long)s * kBK;
                         return alt;
                       },
                       ring, acc);
  if (blk_w >= nb) return;

  const int j = col_idx[p0 + blk_w];
  // compact activation block of (tile i, list entry): the entries of a list row are stored as
  // [entry][tile within the row's group of gt tiles]
  const long long p = (long long)rs * gt + (long long)(first + blk_w) * gt + i % gt;
  const int tl = lane % 32, nq = (lane / 32) * 4;
#pragma unroll
  for (int ni = 0; ni < kNI; ++ni) {
    const int nh = (kNI * wave + ni) % 2;    // which 32 neurons of the block
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int t = 32 * ti + tl, n = 32 * nh + 8 * g + nq;
        const long long o = p * 4096 + t * 64 + n;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[ni][ti][4 * g + e];
        if (MODE == 2) {
        } else if (MODE == 0) {
          if (bias) {
            const uint2 bb = *reinterpret_cast<const uint2*>(bias + j * 64 + n);
            v[0] += to_f32<DT>(bb.x & 0xFFFFu); v[1] += to_f32<DT>(bb.x >> 16);
            v[2] += to_f32<DT>(bb.y & 0xFFFFu); v[3] += to_f32<DT>(bb.y >> 16);
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
        } else {
          const uint2 gg = *reinterpret_cast<const uint2*>(gate_act + o);
          if (!(to_f32<DT>(gg.x & 0xFFFFu) > 0.f)) v[0] = 0.f;
          if (!(to_f32<DT>(gg.x >> 16) > 0.f)) v[1] = 0.f;
          if (!(to_f32<DT>(gg.y & 0xFFFFu) > 0.f)) v[2] = 0.f;
          if (!(to_f32<DT>(gg.y >> 16) > 0.f)) v[3] = 0.f;
        }
        uint2 ov;
        ov.x = pack2<DT>(v[0], v[1]);
        ov.y = pack2<DT>(v[2], v[3]);
        *reinterpret_cast<uint2*>(out_act + o) = ov;
      }
  }
}

// Which token tile the workgroups of grid row `slot` work on.  A workgroup of the dsd kernel
// lasts as long as its tile's list is long, and a launch of few tiles lasts as long as its
// slowest CU.  Up to kBalTiles tiles are therefore ranked by list length (ties by index; every
// workgroup computes the same ranking, so the assignment is a permutation): grid rows are
// dispatched in order, so the longest lists start first; and when the whole launch is resident
// at once, two workgroups per CU, rows s and s + Tt/2, which the round robin of the dispatcher
// places on the same CU, get ranks s and Tt - 1 - s, a long list next to a short one.
constexpr int kBalTiles = 128;
__device__ __forceinline__ int balanced_tile(const int* __restrict__ row_ptr, int Tt, int gt,
                                             int nnz_cap, int slot, bool resident, int* lens) {
  if (Tt > kBalTiles || Tt < 3) return slot;
  const int tid = threadIdx.x;
  if (tid < Tt) lens[tid] = min(row_ptr[tid / gt + 1], nnz_cap) - row_ptr[tid / gt];
  __syncthreads();
  const int half = (Tt + 1) / 2;
  const int want = resident && slot >= half ? Tt - 1 - (slot - half) : slot;
  if (tid < Tt) {
    const int n = lens[tid];
    int rank = 0;
    for (int u = 0; u < Tt; ++u) {
      const int m = lens[u];
      rank += (m > n || (m == n && u < tid)) ? 1 : 0;
    }
    if (rank == want) lens[kBalTiles] = tid;
  }
  __syncthreads();
  const int tile = __builtin_amdgcn_readfirstlane(lens[kBalTiles]);
  __syncthreads();   // lens is memory the caller reuses
  return tile;
}

// out[i-tile rows, n0 .. n0+255] = sum_s act[p_s] [64 x 64] . W[n0.., j_s*64 ..]^T (+ bias)
// LORA: one more step with the operands act2 [T,64] (the token tile's 64 x 64 block) and
// W2 [ncols_out, 64]: out += act2_i W2[n0..]^T, the low-rank part (dZ B) A of the input gradient.
template <int DT, bool LORA>
__global__ __launch_bounds__(kThreads) void ffn_dsd_bf16(
    const uint16_t* __restrict__ act, const uint16_t* __restrict__ W, long long ldw,
    const uint16_t* __restrict__ bias, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int gt, int ncols_out, int nnz_cap,
    uint16_t* __restrict__ out, const uint16_t* __restrict__ act2,
    const uint16_t* __restrict__ W2) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kDsdStages * kStageElems];
  const int i = balanced_tile(row_ptr, gridDim.y, gt, nnz_cap, blockIdx.y,
                              gridDim.x * gridDim.y <= 2 * kCUs, reinterpret_cast<int*>(ring));
  const int n0 = blockIdx.x * kRowsA;
  const int rs = row_ptr[i / gt];
  const int n_i = min(row_ptr[i / gt + 1], nnz_cap) - rs;   // <= 0: nothing within the capacity
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const bool wave_on = n0 + 32 * kNI * wave < ncols_out;

  const uint16_t* src[kIssues];
#pragma unroll
  for (int u = 0; u < kIssues; ++u) {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < 8 / kFW) {
      src[u] = act + row * 64 + seg * 8;          // inside a compact 64x64 activation block
    } else {
      const int n = min(n0 + row - kRowsB, ncols_out - 1);   // rows past the edge: re-read the last
      src[u] = W + (long long)n * ldw + seg * 8;
    }
  }
  auto src2 = [&](int u) -> const uint16_t* {     // the low-rank step, computed when it is issued
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < 8 / kFW) return act2 + ((long long)i * 64 + row) * 64 + seg * 8;
    const int n = min(n0 + row - kRowsB, ncols_out - 1);
    return W2 + (long long)n * 64 + seg * 8;
  };
  f32x16 acc[kNI][2];
  zero_acc(acc);
  const int lsteps = n_i > 0 ? n_i : 0;
  run_ring<DT, kDsdStages>(lsteps + (LORA ? 1 : 0), wave_on, src, src2,
               [&](int s, long long& ob, long long& oa) {
                 const bool alt = LORA && s == lsteps;
                 ob = alt ? 0 : ((long long)(rs + s) * gt + i % gt) * 4096;
                 oa = alt ? 0 : (long long)col_idx[rs + s] * 64;
                 return alt;
               },
                       ring, acc);
  if (!wave_on) return;

  const int tl = lane % 32, nq = (lane / 32) * 4;
#pragma unroll
  for (int ni = 0; ni < kNI; ++ni) {
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int t = i * 64 + 32 * ti + tl;
        const int n = n0 + 32 * (kNI * wave + ni) + 8 * g + nq;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[ni][ti][4 * g + e];
        if (bias) {
          const uint2 bb = *reinterpret_cast<const uint2*>(bias + n);
          v[0] += to_f32<DT>(bb.x & 0xFFFFu); v[1] += to_f32<DT>(bb.x >> 16);
          v[2] += to_f32<DT>(bb.y & 0xFFFFu); v[3] += to_f32<DT>(bb.y >> 16);
        }
        uint2 ov;
        ov.x = pack2<DT>(v[0], v[1]);
        ov.y = pack2<DT>(v[2], v[3]);
        *reinterpret_cast<uint2*>(out + (long long)t * ncols_out + n) = ov;
      }
  }
}

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

// pass 0 (forward):  A = X,  W1 = W_up [F,d],     W2 = W_down [d,F], act_out = H_act, out = Y
// pass 1 (backward): A = dY, W1 = W_down_t [F,d], W2 = W_up_t [d,F], act_out = dZ_act,
//                    act_gate = H_act, out = dX
static dim3 sdd_grid(int Tt, int gt, int nnz_cap) {
  // items <= nnz_cap / 4 + Tt; per XCD L = ceil(items / 8) of them in 8 * ceil(L / 8) slots
  const long long items = ((long long)nnz_cap * gt + 3) / 4 + Tt;
  const int Lub = (int)((items + 7) / 8);
  return dim3(8 * 8 * ((Lub + 7) / 8));
}

template <int DT>
static hipError_t launch_ffn_bf16_t(int pass, int Tt, int gt, int Fb, int d, int F, const uint16_t* A,
                           const uint16_t* W1, const uint16_t* b1, const uint16_t* W2,
                           const uint16_t* b2, const int* row_ptr, const int* col_idx, int nnz_cap,
                           uint16_t* act_out, const uint16_t* act_gate, uint16_t* out,
                           hipStream_t st) {
  (void)Fb;
  if (((long long)nnz_cap * gt + 3) / 4 + Tt > (1ll << 30)) return hipErrorInvalidValue;
  const dim3 g1 = sdd_grid(Tt, gt, nnz_cap);
  const uint16_t* none = nullptr;
  {
    ProfScope ps(pass == 0 ? kKFfnUp : kKFfnDh, st);
    if (pass == 0)
      hipLaunchKernelGGL((ffn_sdd_bf16<DT, 0, false>), g1, dim3(kThreads), 0, st, A, W1, b1, row_ptr,
                         col_idx, Tt, gt, d, nnz_cap, act_out, none, none, none);
    else
      hipLaunchKernelGGL((ffn_sdd_bf16<DT, 1, false>), g1, dim3(kThreads), 0, st, A, W1, none, row_ptr,
                         col_idx, Tt, gt, d, nnz_cap, act_out, act_gate, none, none);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfScope ps(pass == 0 ? kKFfnDown : kKFfnDx, st);
  hipLaunchKernelGGL((ffn_dsd_bf16<DT, false>), dim3((d + kRowsA - 1) / kRowsA, Tt), dim3(kThreads), 0, st,
                     (const uint16_t*)act_out, W2, (long long)F, b2, row_ptr, col_idx, gt, d, nnz_cap,
                     out, none, none);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// LoRA branch on the up-projection (Sec. II-C: z = W x + B A x; Sec. II-D: its gradients).
// A_pad [64, d] and B_pad [F, 64] hold A [r, d] and B [F, r] zero-padded to rank 64.
// ---------------------------------------------------------------------------

// The small products of the branch work on pairs of [64 x 64] bf16 tiles: a stage of the ring
// holds tile P in rows 0..63 and tile Q in rows 64..127 (16 KiB, two DMA instructions per wave:
// rows 8*wave + lane/8 of each).  Four stages = 64 KiB: two workgroups per CU.
constexpr int kPairElems = 128 * kBK;
constexpr int kPairStages = 4;

// Byte offset of element (row, col) inside a staged [64 x 64] tile.
__device__ __forceinline__ uint32_t tile64_off(int row, int col) {
  return (uint32_t)(row * 128 + (((col >> 3) ^ swz(row)) << 4) + (col & 7) * 2);
}

// This lane's source pointers of the two instructions: P and Q point at the first element of the
// tiles of step 0, ldp / ldq are their row strides in elements.
__device__ __forceinline__ void pair_src(const uint16_t* P, long long ldp, const uint16_t* Q,
                                         long long ldq, const uint16_t* (&src)[2]) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int row = 8 * wave + lane / 8, seg = (lane % 8) ^ swz(row);
  src[0] = P + row * ldp + seg * 8;
  src[1] = Q + row * ldq + seg * 8;
}

// The eight wavefronts of such a product: wavefront w owns the 32 x 32 quadrant (w % 2, (w / 2) % 2)
// of the 64 x 64 result and half w / 4 of the contraction index.  fold_khalves adds the second
// halves to the first ones through 16 KiB of LDS, in a fixed order; it returns true in the
// wavefronts 0 .. 3, which then hold the sums.
__device__ __forceinline__ bool fold_khalves(float* area, f32x16& acc) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  lds_barrier();   // nobody reads the ring any more
  if (wave >= 4) {
#pragma unroll
    for (int v = 0; v < 16; ++v) area[((wave - 4) * 16 + v) * kWave + lane] = acc[v];
  }
  lds_barrier();
  if (wave >= 4) return false;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] += area[(wave * 16 + v) * kWave + lane];
  return true;
}

// U = X A_pad^T (Sec. II-C: the inner factor A x of the branch) for token tile blockIdx.x over
// the range of K-steps of blockIdx.y.  gridDim.y == 1: U [T,64] is stored as bf16; otherwise
// fp32 partial sums part[y][T][64], which lora_u_reduce_kernel adds.
template <int DT>
__global__ __launch_bounds__(kThreads) void lora_u_kernel(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ A_pad, int K,
    uint16_t* __restrict__ U, float* __restrict__ part, long long part_stride) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kPairStages * kPairElems];
  const int i = blockIdx.x, ksteps = K / kBK;
  const int per = (ksteps + gridDim.y - 1) / gridDim.y;
  const int s_lo = blockIdx.y * per, s_hi = min(ksteps, s_lo + per);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int th = wave % 2, qh = (wave / 2) % 2, kh = wave / 4;
  const int r = lane % 32, h2 = lane / 32;
  const uint16_t* src[2];
  pair_src(X + (long long)i * 64 * K, K, A_pad, K, src);
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  run_ring_of<kPairStages, 2, kPairElems>(
      s_hi - s_lo, src, NoAlt(),
      [=](int s, long long& ob, long long& oa) {
        ob = oa = (long long)(s_lo + s) * kBK;
        return false;
      },
      ring,
      [&](const uint16_t* stage) {
        uint4 a[2], b[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int seg = 2 * (2 * kh + e) + h2;
          const int ra = 64 + 32 * qh + r, rb = 32 * th + r;
          a[e] = *reinterpret_cast<const uint4*>(stage + ra * kBK + ((seg ^ swz(ra)) << 3));
          b[e] = *reinterpret_cast<const uint4*>(stage + rb * kBK + ((seg ^ swz(rb)) << 3));
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) acc = mfma32<DT>(a[e], b[e], acc);
      });
  if (!fold_khalves(reinterpret_cast<float*>(ring), acc)) return;
  // register v: rank index 32*qh + 8*(v/4) + 4*h2 + v%4, token 32*th + lane%32
  const long long o = ((long long)i * 64 + 32 * th + r) * 64 + 32 * qh + 4 * h2;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    if (gridDim.y == 1) {
      uint2 ov;
      ov.x = pack2<DT>(acc[4 * g], acc[4 * g + 1]);
      ov.y = pack2<DT>(acc[4 * g + 2], acc[4 * g + 3]);
      *reinterpret_cast<uint2*>(U + o + 8 * g) = ov;
    } else {
      const float4 ov = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
      *reinterpret_cast<float4*>(part + blockIdx.y * part_stride + o + 8 * g) = ov;
    }
  }
}
// U = bf16(sum of the parts, in order); n4 = number of groups of four elements
template <int DT>
__global__ void lora_u_reduce_kernel(const float* __restrict__ part, int parts, long long n4,
                                     uint16_t* __restrict__ U) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n4) return;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = 0; p < parts; ++p) {
    const float4 v = *reinterpret_cast<const float4*>(part + ((long long)p * n4 + idx) * 4);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  uint2 ov;
  ov.x = pack2<DT>(s.x, s.y);
  ov.y = pack2<DT>(s.z, s.w);
  *reinterpret_cast<uint2*>(U + idx * 4) = ov;
}

// forward: U = X A_pad^T [T,64];  H_act = ReLU(X W_up^T + U B_pad^T) on the listed blocks;
// Y = H W_down^T.  u_part: lora_u_split(Tt, d) * T * 64 floats of scratch (unused for a split of 1).
template <int DT>
static hipError_t launch_ffn_lora_fwd_bf16_t(int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* W_up, const uint16_t* A_pad,
                                    const uint16_t* B_pad, const uint16_t* W_down,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* U, uint16_t* H_act, uint16_t* Y, float* u_part,
                                    hipStream_t st) {
  if (((long long)nnz_cap * gt + 3) / 4 + Tt > (1ll << 30)) return hipErrorInvalidValue;
  const uint16_t* none = nullptr;
  {
    ProfScope ps(kKLora, st);
    const int split = lora_u_split(Tt, d);
    const long long n = (long long)Tt * 4096;
    hipLaunchKernelGGL(lora_u_kernel<DT>, dim3(Tt, split), dim3(kThreads), 0, st, X, A_pad, d, U, u_part,
                       n);
    if (split > 1)
      hipLaunchKernelGGL(lora_u_reduce_kernel<DT>, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st,
                         (const float*)u_part, split, n / 4, U);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKFfnUp, st);
    hipLaunchKernelGGL((ffn_sdd_bf16<DT, 0, true>), sdd_grid(Tt, gt, nnz_cap), dim3(kThreads), 0, st, X,
                       W_up, none, row_ptr, col_idx, Tt, gt, d, nnz_cap, H_act, none,
                       (const uint16_t*)U, B_pad);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfScope ps(kKFfnDown, st);
  hipLaunchKernelGGL((ffn_dsd_bf16<DT, false>), dim3((d + kRowsA - 1) / kRowsA, Tt), dim3(kThreads), 0, st,
                     (const uint16_t*)H_act, W_down, (long long)F, none, row_ptr, col_idx, gt, d,
                     nnz_cap, Y, none, none);
  return hipGetLastError();
}

// Per-lane LDS offsets of the operands of a product out[a][b] = sum_t P[t][a] Q[t][b] whose
// contraction index is the ROW of both staged tiles: both are read with the transposing read.
// For the 16-row slice i of this wavefront's half of t, a lane gets rows
// {4*h2 .. +3} and {8 + 4*h2 .. +3} of the slice (h2 = lane / 32) of column lane % 32 of its
// quadrant, for P and Q alike, so the two operands of the MFMA agree on the order of t.
struct TnLane {
  uint32_t p[2][2], q[2][2];   // [slice][rows +0 / +8]
  __device__ __forceinline__ void init(int ah, int bh, int kh) {
    const int lane = threadIdx.x % kWave, h2 = lane / 32, j = lane % 16;
    const int col = 16 * ((lane / 16) % 2) + 4 * (j % 4);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int row = 32 * kh + 16 * i + 8 * e + 4 * h2 + j / 4;
        p[i][e] = tile64_off(row, 32 * ah + col);
        q[i][e] = 64 * 128 + tile64_off(row, 32 * bh + col);
      }
  }
};
template <int DT>
__device__ __forceinline__ void tn_step(uint32_t stage, const TnLane& lo, f32x16& acc) {
  uint4 a[2], b[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const uint2 al = lds_read8_tr(stage + lo.p[i][0]), ah = lds_read8_tr(stage + lo.p[i][1]);
    const uint2 bl = lds_read8_tr(stage + lo.q[i][0]), bh = lds_read8_tr(stage + lo.q[i][1]);
    a[i] = make_uint4(al.x, al.y, ah.x, ah.y);
    b[i] = make_uint4(bl.x, bl.y, bh.x, bh.y);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) acc = mfma32<DT>(a[i], b[i], acc);
}

// Gradients of the two LoRA matrices (Sec. II-D), fp32, as sums of 64 x 64 products
// out[a][b] = sum over steps of sum_t P[t][a] Q[t][b] on the MFMA:
// MODE 0, dB = dZ^T U over the listed blocks: blockIdx.x = neuron block j; the steps are the
//   token tiles i of the range of blockIdx.y whose list row holds j (found by bisection of the
//   sorted row, one tile per thread, and kept in list order): P = dZ_ij, Q = U_i;
//   out = rows 64j .. of dB [F,64].
// MODE 1, dA = G^T X: blockIdx.x = 64-column chunk c of X; the steps are all tiles of the range:
//   P = G_i, Q = X_i[:, 64c ..]; out = columns 64c .. of dA [64,d].
// The sums over the gridDim.y tile ranges go to part[y] (part_stride elements apart; with one
// range, part is the result itself) and are added by lora_grad_reduce_kernel.
template <int DT, int MODE>
__global__ __launch_bounds__(kThreads) void lora_tn_kernel(
    const uint16_t* __restrict__ P, const uint16_t* __restrict__ Q, long long ldq,
    const int* __restrict__ row_ptr, const int* __restrict__ col_idx, int Tt, int gt, int nnz_cap,
    float* __restrict__ part, long long part_stride, int ld_out) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kPairStages * kPairElems];
  __shared__ long long s_p[MODE == 0 ? kThreads : 1], s_q[MODE == 0 ? kThreads : 1];
  __shared__ int wcount[kFW];
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int per = (Tt + gridDim.y - 1) / gridDim.y;
  const int i_lo = blockIdx.y * per, i_hi = min(Tt, i_lo + per);
  const int ah = wave % 2, bh = (wave / 2) % 2;
  const uint16_t* src[2];
  pair_src(P, 64, Q + (MODE == 1 ? blockIdx.x * 64 : 0), ldq, src);
  TnLane lo;
  lo.init(ah, bh, wave / 4);
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  auto step = [&](const uint16_t* stage) { tn_step<DT>(lds_addr(stage), lo, acc); };
  if (MODE == 1) {
    run_ring_of<kPairStages, 2, kPairElems>(
        i_hi - i_lo, src, NoAlt(),
        [=](int s, long long& ob, long long& oa) {
          ob = (long long)(i_lo + s) * 4096;
          oa = (long long)(i_lo + s) * 64 * ldq;
          return false;
        },
        ring, step);
  } else {
    // one tile per thread: the host splits so that a range holds at most kThreads tiles
    const int j = blockIdx.x, i = i_lo + tid;
    long long blk = -1;   // compact activation block of (tile i, block j)
    if (i < i_hi) {
      const int rs = row_ptr[i / gt];
      int lo_ = 0, hi_ = min(row_ptr[i / gt + 1], nnz_cap) - rs;   // entries beyond the capacity are ignored
      while (lo_ < hi_) {
        const int mid = (lo_ + hi_) / 2, c = col_idx[rs + mid];
        if (c == j) {
          blk = ((long long)rs + mid) * gt + i % gt;
          break;
        }
        if (c < j) lo_ = mid + 1; else hi_ = mid;
      }
    }
    const unsigned long long hit = __ballot(blk >= 0);
    if (lane == 0) wcount[wave] = __popcll(hit);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kFW; ++w) {
      const int c = wcount[w];
      if (w < wave) before += c;
      total += c;
    }
    if (blk >= 0) {
      const int idx = before + __popcll(hit & ((1ull << lane) - 1ull));
      s_p[idx] = blk * 4096;
      s_q[idx] = (long long)i * 64 * ldq;
    }
    __syncthreads();
    run_ring_of<kPairStages, 2, kPairElems>(
        __builtin_amdgcn_readfirstlane(total), src, NoAlt(),
        [&](int s, long long& ob, long long& oa) {
          ob = s_p[s];
          oa = s_q[s];
          return false;
        },
        ring, step);
  }
  if (!fold_khalves(reinterpret_cast<float*>(ring), acc)) return;
  // register v: a = 32*ah + 8*(v/4) + 4*(lane/32) + v%4, b = 32*bh + lane%32
  const long long row0 = MODE == 0 ? (long long)blockIdx.x * 64 : 0;
  const int col0 = MODE == 0 ? 0 : blockIdx.x * 64;
  float* o = part + blockIdx.y * part_stride + (row0 + 32 * ah + 4 * (lane / 32)) * ld_out + col0 +
             32 * bh + lane % 32;
#pragma unroll
  for (int v = 0; v < 16; ++v) o[(long long)(8 * (v / 4) + v % 4) * ld_out] = acc[v];
}
// dB and dA = sums of their parts, in order, four elements per thread; a result with one part
// was written in place and has n4 = 0 here.
__global__ void lora_grad_reduce_kernel(const float* __restrict__ part_b, int parts_b, long long n4_b,
                                        float* __restrict__ dB, const float* __restrict__ part_a,
                                        int parts_a, long long n4_a, float* __restrict__ dA) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const float* part = part_b;
  int parts = parts_b;
  long long n4 = n4_b;
  float* out = dB;
  if (idx >= n4_b) {
    idx -= n4_b;
    part = part_a; parts = parts_a; n4 = n4_a; out = dA;
    if (idx >= n4_a) return;
  }
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = 0; p < parts; ++p) {
    const float4 v = *reinterpret_cast<const float4*>(part + ((long long)p * n4 + idx) * 4);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  *reinterpret_cast<float4*>(out + idx * 4) = s;
}

// 64 x 64 tile transposes of both LoRA matrices in one launch: workgroups 0 .. d/64 - 1 turn
// A_pad [64,d] into A_t [d,64], the others B_pad [F,64] into B_t [64,F].
__global__ __launch_bounds__(256) void lora_transpose_kernel(
    const uint16_t* __restrict__ A_pad, int d, uint16_t* __restrict__ A_t,
    const uint16_t* __restrict__ B_pad, int F, uint16_t* __restrict__ B_t) {
  __shared__ __attribute__((aligned(16))) uint16_t t[64][72];
  const int tid = threadIdx.x;
  const bool is_a = (int)blockIdx.x < d / 64;
  const long long c = is_a ? blockIdx.x : blockIdx.x - d / 64;
  const uint16_t* src = is_a ? A_pad + c * 64 : B_pad + c * 4096;
  const long long lds = is_a ? d : 64;
  uint16_t* dst = is_a ? A_t + c * 4096 : B_t + c * 64;
  const long long ldd = is_a ? 64 : F;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int piece = tid + h * 256, r = piece / 8, c8 = (piece % 8) * 8;
    const uint4 v = *reinterpret_cast<const uint4*>(src + r * lds + c8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      t[c8 + 2 * e][r] = (uint16_t)(w[e] & 0xFFFFu);
      t[c8 + 2 * e + 1][r] = (uint16_t)(w[e] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int piece = tid + h * 256, r = piece / 8, c8 = (piece % 8) * 8;
    *reinterpret_cast<uint4*>(dst + r * ldd + c8) = *reinterpret_cast<const uint4*>(&t[r][c8]);
  }
}

// backward: dZ = (dY W_down) (.) [H > 0] on the listed blocks;  G = dZ B_pad [T,64];
// dX = dZ W_up + G A_pad;  dB = dZ^T U;  dA = G^T X.
// Scratch: B_t [64,F], A_t [d,64], G [T,64], da_part [lora_da_split][64][d] and
// db_part [lora_db_split][F][64] (each unused for a split of 1).
template <int DT>
static hipError_t launch_ffn_lora_bwd_bf16_t(int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* dY, const uint16_t* H_act, const uint16_t* U,
                                    const uint16_t* W_down_t, const uint16_t* W_up_t,
                                    const uint16_t* A_pad, const uint16_t* B_pad,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* dZ, uint16_t* B_t, uint16_t* A_t, uint16_t* G,
                                    float* da_part, float* db_part, uint16_t* dX, float* dA,
                                    float* dB, hipStream_t st) {
  if (((long long)nnz_cap * gt + 3) / 4 + Tt > (1ll << 30)) return hipErrorInvalidValue;
  const uint16_t* none = nullptr;
  {
    ProfScope ps(kKFfnDh, st);
    hipLaunchKernelGGL((ffn_sdd_bf16<DT, 1, false>), sdd_grid(Tt, gt, nnz_cap), dim3(kThreads), 0, st, dY,
                       W_down_t, none, row_ptr, col_idx, Tt, gt, d, nnz_cap, dZ, H_act, none, none);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKLora, st);
    hipLaunchKernelGGL(lora_transpose_kernel, dim3(d / 64 + F / 64), dim3(256), 0, st, A_pad, d, A_t,
                       B_pad, F, B_t);
    hipLaunchKernelGGL((ffn_dsd_bf16<DT, false>), dim3(1, Tt), dim3(kThreads), 0, st, (const uint16_t*)dZ,
                       (const uint16_t*)B_t, (long long)F, none, row_ptr, col_idx, gt, 64, nnz_cap, G,
                       none, none);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKFfnDx, st);
    hipLaunchKernelGGL((ffn_dsd_bf16<DT, true>), dim3((d + kRowsA - 1) / kRowsA, Tt), dim3(kThreads), 0, st,
                       (const uint16_t*)dZ, W_up_t, (long long)F, none, row_ptr, col_idx, gt, d,
                       nnz_cap, dX, (const uint16_t*)G, (const uint16_t*)A_t);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfScope ps(kKLora, st);
  const int sb = lora_db_split(Tt, F), sa = lora_da_split(Tt, d);
  const long long nb = (long long)F * 64, na = (long long)64 * d;
  hipLaunchKernelGGL((lora_tn_kernel<DT, 0>), dim3(F / 64, sb), dim3(kThreads), 0, st, (const uint16_t*)dZ, U,
                     64ll, row_ptr, col_idx, Tt, gt, nnz_cap, sb > 1 ? db_part : dB, nb, 64);
  hipLaunchKernelGGL((lora_tn_kernel<DT, 1>), dim3(d / 64, sa), dim3(kThreads), 0, st, (const uint16_t*)G, X,
                     (long long)d, row_ptr, col_idx, Tt, gt, nnz_cap, sa > 1 ? da_part : dA, na, d);
  const long long n4b = sb > 1 ? nb / 4 : 0, n4a = sa > 1 ? na / 4 : 0;
  if (n4b + n4a > 0)
    hipLaunchKernelGGL(lora_grad_reduce_kernel, dim3((unsigned)((n4b + n4a + 255) / 256)), dim3(256), 0,
                       st, (const float*)db_part, sb, n4b, dB, (const float*)da_part, sa, n4a, dA);
  return hipGetLastError();
}

// Entry points of this file: dt selects the element type (kBf16 or kF16).
#define LX_BY_DT(fn, ...) (dt == kF16 ? fn<kF16>(__VA_ARGS__) : fn<kBf16>(__VA_ARGS__))
hipError_t launch_predict_bf16(int dt, int T, int d, int nblk, int tiles_per_group, const uint16_t* X,
                               const uint16_t* Wa_t, float thr, uint8_t* mask, hipStream_t st) {
  return LX_BY_DT(launch_predict_bf16_t, T, d, nblk, tiles_per_group, X, Wa_t, thr, mask, st);
}
hipError_t launch_ffn_bf16(int dt, int pass, int Tt, int gt, int Fb, int d, int F, const uint16_t* A,
                           const uint16_t* W1, const uint16_t* b1, const uint16_t* W2,
                           const uint16_t* b2, const int* row_ptr, const int* col_idx, int nnz_cap,
                           uint16_t* act_out, const uint16_t* act_gate, uint16_t* out,
                           hipStream_t st) {
  return LX_BY_DT(launch_ffn_bf16_t, pass, Tt, gt, Fb, d, F, A, W1, b1, W2, b2, row_ptr, col_idx,
                  nnz_cap, act_out, act_gate, out, st);
}
hipError_t launch_ffn_lora_fwd_bf16(int dt, int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* W_up, const uint16_t* A_pad,
                                    const uint16_t* B_pad, const uint16_t* W_down,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* U, uint16_t* H_act, uint16_t* Y, float* u_part,
                                    hipStream_t st) {
  return LX_BY_DT(launch_ffn_lora_fwd_bf16_t, Tt, gt, d, F, X, W_up, A_pad, B_pad, W_down, row_ptr,
                  col_idx, nnz_cap, U, H_act, Y, u_part, st);
}
hipError_t launch_ffn_lora_bwd_bf16(int dt, int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* dY, const uint16_t* H_act, const uint16_t* U,
                                    const uint16_t* W_down_t, const uint16_t* W_up_t,
                                    const uint16_t* A_pad, const uint16_t* B_pad,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* dZ, uint16_t* B_t, uint16_t* A_t, uint16_t* G,
                                    float* da_part, float* db_part, uint16_t* dX, float* dA,
                                    float* dB, hipStream_t st) {
  return LX_BY_DT(launch_ffn_lora_bwd_bf16_t, Tt, gt, d, F, X, dY, H_act, U, W_down_t, W_up_t,
                  A_pad, B_pad, row_ptr, col_idx, nnz_cap, dZ, B_t, A_t, G, da_part, db_part, dX,
                  dA, dB, st);
}
#undef LX_BY_DT

}  // namespace lx
