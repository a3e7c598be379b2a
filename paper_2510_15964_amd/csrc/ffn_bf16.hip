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
// Data movement: the transfer ring of ffn_ring.h, three 40 KiB stages in the sdd kernel (the
// loads of K-steps s+1 and s+2 are in flight while the MFMAs of step s run), two in the dsd
// kernel (two resident workgroups per CU).
//
// The LoRA branch on the up-projection (Sec. II-C / II-D) is one more step of either ring; the
// calls that add it are at the end of this file, its small products in lora_bf16.hip.
#include "ffn_ring.h"

namespace lx {

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
                                          int per, int nnz_cap, int& row, int& chunk) {
  const int lane = threadIdx.x % kWave;
  // entries of a list row that lie within the capacity of the list buffers: the items are
  // counted from these, so that their number never exceeds the bound the grid was sized from
  auto row_len = [&](int lr) { return min(row_ptr[lr + 1], nnz_cap) - min(row_ptr[lr], nnz_cap); };
  if (gt >= rows && rows >= 8) {
    // One list row for all token tiles: the items are a regular rows x C grid, and every XCD
    // takes a rectangle of it, rows / xr tiles by C / (8 / xr) groups of entries, that it walks
    // in columns.  The workgroups that run together on an XCD (32 consecutive slots) then share
    // a few activation tiles and a few weight blocks alike, instead of two tiles and sixteen
    // groups of blocks: a third fewer bytes miss its L2.
    const int C = (row_len(0) + per - 1) / per;
    int xr = 8;
    while (xr > 1 && (rows % xr != 0 || C % (8 / xr) != 0 || rows / xr < 4)) xr >>= 1;
    if (C > 0 && rows % xr == 0 && C % (8 / xr) == 0) {
      const int Rr = rows / xr, Cc = C / (8 / xr);
      const int x = w % 8, s = w / 8;
      if (s >= Rr * Cc) return false;
      row = (x % xr) * Rr + s % Rr;
      chunk = (x / xr) * Cc + s / Rr;
      return true;
    }
  }
  int total = 0;
  for (int base = 0; base < rows; base += kWave) {
    const int r = base + lane;
    int c = 0;
    if (r < rows) c = (row_len(r / gt) + per - 1) / per;
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
    if (r < rows) c = (row_len(r / gt) + per - 1) / per;
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
// NST: stages of the transfer ring.  Three stages leave room for one workgroup per CU, two for two:
// the launcher takes two when the items are more than one but at most two per CU, so that all
// of them are resident at once instead of running as a full round and a partly filled one.
template <int DT, int MODE, bool LORA, int NST = kSddStages>
__global__ __launch_bounds__(kThreads, NST == 2 ? 2 : 1) void ffn_sdd_bf16(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
    const uint16_t* __restrict__ bias, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int rows, int gt, int K, int nnz_cap,
    uint16_t* __restrict__ out_act, const uint16_t* __restrict__ gate_act,
    const uint16_t* __restrict__ A2, const uint16_t* __restrict__ W2) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[NST * kStageElems];
  int i, chunk;
  if (!find_work(row_ptr, rows, gt, blockIdx.x, 4, nnz_cap, i, chunk)) return;
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
  run_ring<DT, NST>(ksteps + (LORA ? 1 : 0), blk_w < nb, src, src2,
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
// The launch covers the Tt tiles first .. first + Tt - 1; the result is a tile of that range.
__device__ __forceinline__ int balanced_tile(const int* __restrict__ row_ptr, int first, int Tt,
                                             int gt, int nnz_cap, int slot, bool resident,
                                             int* lens) {
  if (Tt > kBalTiles || Tt < 3) return first + slot;
  const int tid = threadIdx.x;
  if (tid < Tt) {
    const int r = (first + tid) / gt;
    lens[tid] = min(row_ptr[r + 1], nnz_cap) - row_ptr[r];
  }
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
  return first + tile;
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
    const uint16_t* __restrict__ W2, int tile0) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kDsdStages * kStageElems];
  // the launch covers the token tiles tile0 .. tile0 + gridDim.y - 1
  const int i = balanced_tile(row_ptr, tile0, gridDim.y, gt, nnz_cap, blockIdx.y,
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

// ---------------------------------------------------------------------------
// Several token tiles per workgroup.  When TT = 2 or 4 consecutive token tiles share a list row
// (the paper's reduced mask, or a dense layer), they can be multiplied with the same weight
// rows: 64*TT token rows + 256 weight rows per stage (48 KiB in a ring of three, or 64 KiB in a
// ring of two; one workgroup per CU) and a wave tile of 64 x 32*TT, i.e. 0.6 / 0.4 times the
// transferred and a half / three eighths of the LDS-read bytes per product of the kernels above.
// Every output element sees the same products in the same order, so the results are
// bit-identical to the one-tile kernels'.  It pays when the launch still fills the chip with
// a half or a quarter as many workgroups (large or dense layers); the host chooses
// (launch_ffn_bf16).
// ---------------------------------------------------------------------------

// Epilogue of one 64 x 64 token tile of a wave tile: acc[ni][2*tile + ti] -> rows 32*ti + lane%32
// (stride ld elements) and columns 32*ni + 8*g + 4*(lane/32) + e of `out`; bias over the
// columns, gate with the same indexing (both may be null).
template <int DT, int MODE, int TT>
__device__ __forceinline__ void store_tile64(const f32x16 (&acc)[2][TT], int tile,
                                             uint16_t* __restrict__ out, long long ld,
                                             const uint16_t* __restrict__ bias,
                                             const uint16_t* __restrict__ gate) {
  const int lane = threadIdx.x % kWave, tl = lane % 32, nq = (lane / 32) * 4;
#pragma unroll
  for (int ni = 0; ni < 2; ++ni)
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = 32 * ni + 8 * g + nq;
        const long long o = (long long)(32 * ti + tl) * ld + n;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[ni][2 * tile + ti][4 * g + e];
        if (bias) {
          const uint2 bb = *reinterpret_cast<const uint2*>(bias + n);
          v[0] += to_f32<DT>(bb.x & 0xFFFFu); v[1] += to_f32<DT>(bb.x >> 16);
          v[2] += to_f32<DT>(bb.y & 0xFFFFu); v[3] += to_f32<DT>(bb.y >> 16);
        }
        if (MODE == 0) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
        } else if (MODE == 1) {
          const uint2 gg = *reinterpret_cast<const uint2*>(gate + o);
          if (!(to_f32<DT>(gg.x & 0xFFFFu) > 0.f)) v[0] = 0.f;
          if (!(to_f32<DT>(gg.x >> 16) > 0.f)) v[1] = 0.f;
          if (!(to_f32<DT>(gg.y & 0xFFFFu) > 0.f)) v[2] = 0.f;
          if (!(to_f32<DT>(gg.y >> 16) > 0.f)) v[3] = 0.f;
        }
        uint2 ov;
        ov.x = pack2<DT>(v[0], v[1]);
        ov.y = pack2<DT>(v[2], v[3]);
        *reinterpret_cast<uint2*>(out + o) = ov;
      }
}

// sdd for groups of TT token tiles: work item = (TT consecutive tiles of one list row, up to four
// consecutive list entries); wave w multiplies entry w % 4 with half w / 4 of the group's tiles.
// `rows` counts token tiles, gt of which share a list row (both multiples of TT).  MODE / LORA as
// above.
template <int DT, int MODE, bool LORA, int TT>
__global__ __launch_bounds__(kThreads) void ffn_sddn_bf16(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
    const uint16_t* __restrict__ bias, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int rows, int gt, int K, int nnz_cap,
    uint16_t* __restrict__ out_act, const uint16_t* __restrict__ gate_act,
    const uint16_t* __restrict__ A2, const uint16_t* __restrict__ W2) {
  using St = MultiStage<TT>;
  __shared__ __attribute__((aligned(1024))) uint16_t ring[St::kStages * St::kElems];
  int grp, chunk;
  if (!find_work(row_ptr, rows / TT, gt / TT, blockIdx.x, 4, nnz_cap, grp, chunk)) return;
  const int i0 = TT * grp;                       // first tile of the group
  const int rs = row_ptr[i0 / gt], n_i = row_ptr[i0 / gt + 1] - rs;
  const int first = chunk * 4;
  const int p0 = rs + first;
  if (p0 >= nnz_cap) return;       // entries beyond the capacity of the list buffers are ignored
  const int nb = min(min(4, n_i - first), nnz_cap - p0);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;

  const uint16_t* src[St::kIss];
#pragma unroll
  for (int u = 0; u < St::kIss; ++u) {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < TT) {
      src[u] = A + ((long long)i0 * 64 + row) * K + seg * 8;      // 64*TT consecutive token rows
    } else {
      const int blk = (row - St::kShared) / 64, r = (row - St::kShared) % 64;
      // blocks past the end of the list are filled from the first block (never used)
      const int j = col_idx[p0 + (blk < nb ? blk : 0)];
      src[u] = W + ((long long)j * 64 + r) * K + seg * 8;
    }
  }
  auto src2 = [&](int u) -> const uint16_t* {    // the low-rank step, computed when it is issued
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < TT) return A2 + ((long long)i0 * 64 + row) * 64 + seg * 8;
    const int blk = (row - St::kShared) / 64, r = (row - St::kShared) % 64;
    const int j = col_idx[p0 + (blk < nb ? blk : 0)];
    return W2 + ((long long)j * 64 + r) * 64 + seg * 8;
  };
  const int rg = wave % 4, th = wave / 4;        // list entry of the four, half of the group's tiles
  const bool wave_on = rg < nb;
  f32x16 acc[2][TT];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < TT; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;
  const int ksteps = K / kBK;
  run_ring_of<St::kStages, St::kIss, St::kElems, TT>(
      ksteps + (LORA ? 1 : 0), src, src2,
      [=](int s, long long& ob, long long& oa) {
        const bool alt = LORA && s == ksteps;
        ob = oa = alt ? 0 : (long long)s * kBK;
        return alt;
      },
      ring, [&](const uint16_t* stage) {
        if (wave_on) mma_step64<DT, TT>(stage, rg, th, acc);
      });
  if (!wave_on) return;
  const int j = col_idx[p0 + rg];
#pragma unroll
  for (int t = 0; t < TT / 2; ++t) {
    const int i = i0 + (TT / 2) * th + t;
    // compact activation block of (tile i, list entry): [entry][tile within the row's group]
    const long long p = (long long)rs * gt + (long long)(first + rg) * gt + i % gt;
    store_tile64<DT, MODE, TT>(acc, t, out_act + p * 4096, 64,
                               MODE == 0 && bias ? bias + j * 64 : nullptr,
                               MODE == 1 ? gate_act + p * 4096 : nullptr);
  }
}

// dsd for groups of TT token tiles: the workgroup of grid row y works on tiles TT*y .. (one list
// row) and 256 output columns; wave w multiplies columns 64 * (w % 4) .. with half w / 4 of the
// group's tiles.
template <int DT, bool LORA, int TT>
__global__ __launch_bounds__(kThreads) void ffn_dsdn_bf16(
    const uint16_t* __restrict__ act, const uint16_t* __restrict__ W, long long ldw,
    const uint16_t* __restrict__ bias, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int gt, int ncols_out, int nnz_cap,
    uint16_t* __restrict__ out, const uint16_t* __restrict__ act2,
    const uint16_t* __restrict__ W2, int group0, int lin0, int nchunks, int ksplit,
    float* __restrict__ part) {
  using St = MultiStage<TT>;
  __shared__ __attribute__((aligned(1024))) uint16_t ring[St::kStages * St::kElems];
  // ksplit == 0: 2-D grid (column chunk, tile group), the launch covers the tile groups group0 ..
  // group0 + gridDim.y - 1.  ksplit >= 1: 1-D grid over (unit, piece): unit lin0 + blockIdx.x /
  // ksplit of the (tile group, column chunk) pairs numbered chunk-fastest, and piece blockIdx.x %
  // ksplit of the unit's list; with `part` the accumulators go there as they are, fp32, for
  // ffn_dsd_reduce to add the pieces of a unit in order (fills the chip when the units of the last
  // round of workgroups are few).
  int i0, n0, piece = 0;
  if (ksplit == 0) {
    i0 = TT * balanced_tile(row_ptr, group0, gridDim.y, gt / TT, nnz_cap, blockIdx.y, false,
                            reinterpret_cast<int*>(ring));
    n0 = blockIdx.x * kRowsA;
  } else {
    const int lin = lin0 + blockIdx.x / ksplit;
    piece = blockIdx.x % ksplit;
    i0 = TT * (lin / nchunks);
    n0 = (lin % nchunks) * kRowsA;
  }
  const int rs0 = row_ptr[i0 / gt];
  const int n_all = min(row_ptr[i0 / gt + 1], nnz_cap) - rs0;   // <= 0: nothing within the capacity
  // this piece's range of the list (the whole list unless ksplit > 1)
  const int nn = n_all > 0 ? n_all : 0;
  const int s_lo = ksplit > 1 ? (int)((long long)nn * piece / ksplit) : 0;
  const int s_hi = ksplit > 1 ? (int)((long long)nn * (piece + 1) / ksplit) : nn;
  const int rs = rs0 + s_lo;
  const int n_i = s_hi - s_lo;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int rg = wave % 4, th = wave / 4;        // 64 output columns of the 256, half of the tiles
  const bool wave_on = n0 + 64 * rg < ncols_out;

  const uint16_t* src[St::kIss];
#pragma unroll
  for (int u = 0; u < St::kIss; ++u) {
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < TT) {
      src[u] = act + row * 64 + seg * 8;          // the tiles' blocks of an entry are adjacent
    } else {
      const int n = min(n0 + row - St::kShared, ncols_out - 1);   // rows past the edge: re-read the last
      src[u] = W + (long long)n * ldw + seg * 8;
    }
  }
  auto src2 = [&](int u) -> const uint16_t* {     // the low-rank step, computed when it is issued
    const int g = wave + kFW * u, row = 8 * g + lane / 8;
    const int seg = (lane % 8) ^ swz(row);
    if (u < TT) return act2 + ((long long)i0 * 64 + row) * 64 + seg * 8;
    const int n = min(n0 + row - St::kShared, ncols_out - 1);
    return W2 + (long long)n * 64 + seg * 8;
  };
  f32x16 acc[2][TT];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < TT; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;
  const int lsteps = n_i > 0 ? n_i : 0;
  run_ring_of<St::kStages, St::kIss, St::kElems, TT>(
      lsteps + (LORA ? 1 : 0), src, src2,
      [&](int s, long long& ob, long long& oa) {
        const bool alt = LORA && s == lsteps;
        ob = alt ? 0 : ((long long)(rs + s) * gt + i0 % gt) * 4096;
        oa = alt ? 0 : (long long)col_idx[rs + s] * 64;
        return alt;
      },
      ring, [&](const uint16_t* stage) {
        if (wave_on) mma_step64<DT, TT>(stage, rg, th, acc);
      });
  if (!wave_on) return;
  if (part) {   // the piece's partial sums: [wave][accumulator][lane][16 registers] (ffn_dsd_reduce reads them the same way)
    f32x4* dst = reinterpret_cast<f32x4*>(part + ((size_t)blockIdx.x * kFW + wave) * (2 * TT * 16) * kWave) + lane * 4;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < TT; ++y)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v4 = {acc[x][y][4 * q], acc[x][y][4 * q + 1], acc[x][y][4 * q + 2], acc[x][y][4 * q + 3]};
          dst[(x * TT + y) * (kWave * 4) + q] = v4;
        }
    return;
  }
  // ncols_out is a multiple of 64 (the host checks d % 64 == 0): a wave's 64 columns are all inside
  const int n = n0 + 64 * rg;
#pragma unroll
  for (int t = 0; t < TT / 2; ++t)
    store_tile64<DT, 2, TT>(acc, t, out + (long long)(i0 + (TT / 2) * th + t) * 64 * ncols_out + n,
                            ncols_out, bias ? bias + n : nullptr, nullptr);
}

// Adds the ksplit pieces of each unit that ffn_dsdn_bf16 left in `part` (piece 0 first, fixed
// order: reproducible) and writes the unit's tile like the kernel's own epilogue: workgroup
// (b, t) is unit lin0 + b and the t-th token tile of each of the kernel's wavefronts; its threads
// hold the same accumulator elements as in the kernel.
template <int DT, int TT, int T>
__device__ __forceinline__ void dsd_reduce_tile(const float* __restrict__ part, int ksplit, int wave,
                                                int lane, uint16_t* __restrict__ out_tile, long long ld,
                                                const uint16_t* __restrict__ bias) {
  f32x16 acc[2][TT];       // only [.][2T], [.][2T + 1] are used
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < TT; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;
  for (int p = 0; p < ksplit; ++p) {
    const f32x4* src = reinterpret_cast<const f32x4*>(
        part + (((size_t)blockIdx.x * ksplit + p) * kFW + wave) * (2 * TT * 16) * kWave) + lane * 4;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v4 = src[(x * TT + 2 * T + ti) * (kWave * 4) + q];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[x][2 * T + ti][4 * q + e] += v4[e];
        }
  }
  store_tile64<DT, 2, TT>(acc, T, out_tile, ld, bias, nullptr);
}
template <int DT, int TT>
__global__ __launch_bounds__(kThreads) void ffn_dsd_reduce(const float* __restrict__ part, int ksplit,
                                                           int lin0, int nchunks, int ncols_out,
                                                           const uint16_t* __restrict__ bias,
                                                           uint16_t* __restrict__ out) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int rg = wave % 4, th = wave / 4;
  const int lin = lin0 + blockIdx.x, t = blockIdx.y;       // t < TT / 2
  const int i0 = TT * (lin / nchunks), n0 = (lin % nchunks) * kRowsA;
  if (n0 + 64 * rg >= ncols_out) return;
  const int n = n0 + 64 * rg;
  uint16_t* out_tile = out + (long long)(i0 + (TT / 2) * th + t) * 64 * ncols_out + n;
  const uint16_t* b = bias ? bias + n : nullptr;
  if (TT == 4 && t == 1)
    dsd_reduce_tile<DT, TT, TT == 4 ? 1 : 0>(part, ksplit, wave, lane, out_tile, ncols_out, b);
  else
    dsd_reduce_tile<DT, TT, 0>(part, ksplit, wave, lane, out_tile, ncols_out, b);
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

// Token tiles per workgroup: 0 = chosen here; 1, 2 or 4 = asked for by the caller.  One value
// per host thread: a thread that sets the knob changes its own later calls only.
static thread_local int g_ffn_tiles_per_wg = 0;
hipError_t set_ffn_tiles_per_wg(int n) {
  if (n != 0 && n != 1 && n != 2 && n != 4) return hipErrorInvalidValue;
  g_ffn_tiles_per_wg = n;
  return hipSuccess;
}
// Groups of tiles need list rows shared by a multiple of that many tiles; left to itself the
// library takes the largest group that still fills the chip, judged by the capacity of the list
// (the true number of entries is known on the device only: a capacity far above it makes the
// choice too optimistic, and the caller's knob overrides it).
static int tiles_per_wg(int Tt, int gt, int nnz_cap) {
  const int want = g_ffn_tiles_per_wg;
  if (want == 1) return 1;
  for (int tt = 4; tt > 1; tt /= 2) {
    if (gt % tt != 0) continue;
    if (want != 0) {
      if (want >= tt) return tt;
      continue;
    }
    // left to itself: the largest group whose work items (tile groups x groups of four list
    // entries, by the host-known bound on the entries) still give every CU a workgroup
    const long long items = (long long)(gt / tt) * ((nnz_cap + 3) / 4);
    if (Tt / tt >= kCUs || items >= kCUs) return tt;
  }
  return 1;
}

// Floats one piece of a split dsd unit leaves in the partial-sum buffer (TT token tiles).
static size_t dsd_piece_floats(int tt) { return (size_t)kFW * 2 * tt * 16 * kWave; }
// How the multi-tile dsd launch is cut when its (tile group, column chunk) units make whole
// rounds of workgroups plus a small rest: the rest's lists are split into `pieces` pieces each,
// so that the last round fills the chip too, and the pieces are added afterwards.  pieces = 0:
// no split (nothing to gain, one list row only, or the bound on the list is too short to cut).
struct DsdSplit {
  long long full;   // units that run whole
  int rest;         // units whose list is split
  int pieces;
};
static DsdSplit dsd_split(int Tt, int gt, int d, int tt, int nnz_cap) {
  DsdSplit sp = {0, 0, 0};
  const int chunks = (d + kRowsA - 1) / kRowsA;
  const long long units = (long long)chunks * (Tt / tt);
  const long long rest = units % kCUs;
  if (gt != Tt || rest == 0 || rest * 5 >= kCUs * 3) return sp;      // one list row for all tiles only
  const int pieces = (int)(kCUs / rest < 4 ? kCUs / rest : 4);
  if (pieces < 2 || nnz_cap < 16 * pieces) return sp;
  sp.full = units - rest;
  sp.rest = (int)rest;
  sp.pieces = pieces;
  return sp;
}
// Bytes of partial sums the split needs for T tokens and d output columns with one list row of
// at most nnz_cap entries, for the tile count the library would choose (0: no split).
size_t ffn_dsd_split_bytes(int Tt, int d, int nnz_cap) {
  size_t need = 0;
  for (int tt = 4; tt > 1; tt /= 2) {
    if (Tt % tt != 0) continue;
    const DsdSplit sp = dsd_split(Tt, Tt, d, tt, nnz_cap);
    const size_t b = (size_t)sp.rest * sp.pieces * dsd_piece_floats(tt) * sizeof(float);
    need = b > need ? b : need;
  }
  return need;
}

// First product of a pass for groups of TT token tiles.
template <int DT, int TT>
static void launch_sdd_multi(int pass, int Tt, int gt, int d, const uint16_t* A, const uint16_t* W1,
                             const uint16_t* b1, const int* row_ptr, const int* col_idx, int nnz_cap,
                             uint16_t* act_out, const uint16_t* act_gate, hipStream_t st) {
  const uint16_t* none = nullptr;
  const dim3 g1 = sdd_grid(Tt / TT, gt / TT, nnz_cap);
  ProfScope ps(pass == 0 ? kKFfnUp : kKFfnDh, st);
  if (pass == 0)
    hipLaunchKernelGGL((ffn_sddn_bf16<DT, 0, false, TT>), g1, dim3(kThreads), 0, st, A, W1, b1, row_ptr,
                       col_idx, Tt, gt, d, nnz_cap, act_out, none, none, none);
  else
    hipLaunchKernelGGL((ffn_sddn_bf16<DT, 1, false, TT>), g1, dim3(kThreads), 0, st, A, W1, none,
                       row_ptr, col_idx, Tt, gt, d, nnz_cap, act_out, act_gate, none, none);
}
// ... one token tile per workgroup
template <int DT>
static void launch_sdd_one(int pass, int Tt, int gt, int d, const uint16_t* A, const uint16_t* W1,
                           const uint16_t* b1, const int* row_ptr, const int* col_idx, int nnz_cap,
                           uint16_t* act_out, const uint16_t* act_gate, hipStream_t st) {
  const dim3 g1 = sdd_grid(Tt, gt, nnz_cap);
  const uint16_t* none = nullptr;
  // more than one item per CU but at most two: two resident workgroups of two stages each
  // (the item count is known on the device only; a list row of n entries makes ceil(n / 4) items,
  // 3/8 of an item more than n / 4 on average, which is what the estimate adds per tile)
  const long long items_est = ((long long)nnz_cap * gt + 3) / 4 + (3 * (long long)Tt + 7) / 8;
  const bool two_resident = items_est > kCUs && items_est <= 2 * kCUs;
  ProfScope ps(pass == 0 ? kKFfnUp : kKFfnDh, st);
  if (pass == 0 && two_resident)
    hipLaunchKernelGGL((ffn_sdd_bf16<DT, 0, false, 2>), g1, dim3(kThreads), 0, st, A, W1, b1, row_ptr,
                       col_idx, Tt, gt, d, nnz_cap, act_out, none, none, none);
  else if (pass == 0)
    hipLaunchKernelGGL((ffn_sdd_bf16<DT, 0, false>), g1, dim3(kThreads), 0, st, A, W1, b1, row_ptr,
                       col_idx, Tt, gt, d, nnz_cap, act_out, none, none, none);
  else if (two_resident)
    hipLaunchKernelGGL((ffn_sdd_bf16<DT, 1, false, 2>), g1, dim3(kThreads), 0, st, A, W1, none, row_ptr,
                       col_idx, Tt, gt, d, nnz_cap, act_out, act_gate, none, none);
  else
    hipLaunchKernelGGL((ffn_sdd_bf16<DT, 1, false>), g1, dim3(kThreads), 0, st, A, W1, none, row_ptr,
                       col_idx, Tt, gt, d, nnz_cap, act_out, act_gate, none, none);
}

// Second product of a pass for groups of TT token tiles.
template <int DT, int TT>
static void launch_dsd_multi(int pass, int Tt, int gt, int d, int F, const uint16_t* W2, const uint16_t* b2,
                             const int* row_ptr, const int* col_idx, int nnz_cap, const uint16_t* act,
                             uint16_t* out, float* part, size_t part_bytes, hipStream_t st) {
  const uint16_t* none = nullptr;
  ProfScope ps(pass == 0 ? kKFfnDown : kKFfnDx, st);
  // The dsd launch has (column chunks) x (tile groups) workgroups, one per CU, all about equally
  // long.  When they make whole rounds plus a small rest, that rest would keep the launch alive
  // for a full round on a fraction of the chip: the tile groups of whole rounds go to this
  // kernel, the remaining tiles to a kernel with shorter rounds: pairs of tiles when this one
  // takes four, else the one-tile kernel (two workgroups per CU).
  const int chunks = (d + kRowsA - 1) / kRowsA;
  int groups = Tt / TT;
  // With room for partial sums: the units of the whole rounds run as they are, the lists of the
  // rest are cut into pieces that fill the last round, and the pieces are added in order.
  const DsdSplit sp = dsd_split(Tt, gt, d, TT, nnz_cap);
  if (part && sp.pieces > 0 &&
      (size_t)sp.rest * sp.pieces * dsd_piece_floats(TT) * sizeof(float) <= part_bytes) {
    float* nopart = nullptr;
    if (sp.full > 0)
      hipLaunchKernelGGL((ffn_dsdn_bf16<DT, false, TT>), dim3((unsigned)sp.full), dim3(kThreads), 0, st,
                         act, W2, (long long)F, b2, row_ptr, col_idx, gt, d,
                         nnz_cap, out, none, none, 0, 0, chunks, 1, nopart);
    hipLaunchKernelGGL((ffn_dsdn_bf16<DT, false, TT>), dim3(sp.rest * sp.pieces), dim3(kThreads), 0, st,
                       act, W2, (long long)F, b2, row_ptr, col_idx, gt, d,
                       nnz_cap, out, none, none, 0, (int)sp.full, chunks, sp.pieces, part);
    hipLaunchKernelGGL((ffn_dsd_reduce<DT, TT>), dim3(sp.rest, TT / 2), dim3(kThreads), 0, st,
                       (const float*)part, sp.pieces, (int)sp.full, chunks, d, b2, out);
    return;
  }
  float* nopart = nullptr;
  const long long wgs = (long long)chunks * groups, rest = wgs % kCUs;
  if (wgs > kCUs && rest > 0 && rest * 5 < kCUs * 3) groups = (int)((wgs - rest) / chunks);
  if (groups > 0)
    hipLaunchKernelGGL((ffn_dsdn_bf16<DT, false, TT>), dim3(chunks, groups), dim3(kThreads), 0, st,
                       act, W2, (long long)F, b2, row_ptr, col_idx, gt, d,
                       nnz_cap, out, none, none, 0, 0, chunks, 0, nopart);
  const int left = Tt - groups * TT;   // a multiple of TT
  if (left > 0 && TT == 4)
    hipLaunchKernelGGL((ffn_dsdn_bf16<DT, false, 2>), dim3(chunks, left / 2), dim3(kThreads), 0, st,
                       act, W2, (long long)F, b2, row_ptr, col_idx, gt, d,
                       nnz_cap, out, none, none, groups * TT / 2, 0, chunks, 0, nopart);
  else if (left > 0)
    hipLaunchKernelGGL((ffn_dsd_bf16<DT, false>), dim3(chunks, left), dim3(kThreads), 0, st,
                       act, W2, (long long)F, b2, row_ptr, col_idx, gt, d,
                       nnz_cap, out, none, none, groups * TT);
}

template <int DT>
static hipError_t launch_ffn_bf16_t(int pass, int Tt, int gt, int Fb, int d, int F, const uint16_t* A,
                           const uint16_t* W1, const uint16_t* b1, const uint16_t* W2,
                           const uint16_t* b2, const int* row_ptr, const int* col_idx, int nnz_cap,
                           uint16_t* act_out, const uint16_t* act_gate, uint16_t* out,
                           float* part, size_t part_bytes, hipStream_t st) {
  (void)Fb;
  if (((long long)nnz_cap * gt + 3) / 4 + Tt > (1ll << 30)) return hipErrorInvalidValue;
  const int tt = tiles_per_wg(Tt, gt, nnz_cap);
  // The first product may take smaller groups than the second (the activation blocks are laid out
  // the same for every group size): its work items, tile groups x groups of four list entries,
  // run in rounds of one per CU, and a round lasts as long as one item's K-steps, whose time is
  // the step's matrix instructions plus its transfers (512 clocks of the first per token tile,
  // 2 clocks per 128-byte row of the second).  The group size with the cheapest rounds wins: e.g.
  // 89 entries for 64 tiles are 368 items = two rounds of four tiles but 736 = three rounds of
  // two, which cost less; 33 entries are one round of four tiles against two of two.
  int tts = tt;
  long long best = -1;
  for (int t = tt; t >= 1; t /= 2) {
    // (host-known bound: the entries of all list rows in groups of four, a ragged group per further row)
    const long long items = (long long)(gt / t) * ((nnz_cap + 3) / 4 + (Tt / gt - 1));
    const long long rounds = (items + kCUs - 1) / kCUs;
    const long long cost = rounds * (512 * t + 2 * (64 * t + 256));
    if (best < 0 || cost < best) {
      best = cost;
      tts = t;
    }
  }
  if (tts == 4)
    launch_sdd_multi<DT, 4>(pass, Tt, gt, d, A, W1, b1, row_ptr, col_idx, nnz_cap, act_out, act_gate, st);
  else if (tts == 2)
    launch_sdd_multi<DT, 2>(pass, Tt, gt, d, A, W1, b1, row_ptr, col_idx, nnz_cap, act_out, act_gate, st);
  else
    launch_sdd_one<DT>(pass, Tt, gt, d, A, W1, b1, row_ptr, col_idx, nnz_cap, act_out, act_gate, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (tt == 4) {
    launch_dsd_multi<DT, 4>(pass, Tt, gt, d, F, W2, b2, row_ptr, col_idx, nnz_cap, act_out, out, part,
                            part_bytes, st);
  } else if (tt == 2) {
    launch_dsd_multi<DT, 2>(pass, Tt, gt, d, F, W2, b2, row_ptr, col_idx, nnz_cap, act_out, out, part,
                            part_bytes, st);
  } else {
    const uint16_t* none = nullptr;
    ProfScope ps(pass == 0 ? kKFfnDown : kKFfnDx, st);
    hipLaunchKernelGGL((ffn_dsd_bf16<DT, false>), dim3((d + kRowsA - 1) / kRowsA, Tt), dim3(kThreads), 0, st,
                       (const uint16_t*)act_out, W2, (long long)F, b2, row_ptr, col_idx, gt, d, nnz_cap,
                       out, none, none, 0);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// LoRA branch on the up-projection (Sec. II-C: z = W x + B A x; Sec. II-D: its gradients).
// A_pad [64, d] and B_pad [F, 64] hold A [r, d] and B [F, r] zero-padded to rank 64.
// ---------------------------------------------------------------------------

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
    const hipError_t eu = launch_lora_u(DT, Tt, d, X, A_pad, U, u_part, st);
    if (eu != hipSuccess) return eu;
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
                     nnz_cap, Y, none, none, 0);
  return hipGetLastError();
}

// backward: dZ = (dY W_down) (.) [H > 0] on the listed blocks;  G = dZ B_pad [T,64];
// dX = dZ W_up + G A_pad;  dB = dZ^T U;  dA = G^T X.
// Scratch: B_t [64,F], A_t [d,64], G [T,64], g_part [lora_g_split][T][64], da_part [lora_da_split][64][d] and
// db_part [lora_db_split][F][64] (each unused for a split of 1).
template <int DT>
static hipError_t launch_ffn_lora_bwd_bf16_t(int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* dY, const uint16_t* H_act, const uint16_t* U,
                                    const uint16_t* W_down_t, const uint16_t* W_up_t,
                                    const uint16_t* A_pad, const uint16_t* B_pad,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* dZ, uint16_t* B_t, uint16_t* A_t, uint16_t* G,
                                    float* g_part, float* da_part, float* db_part, uint16_t* dX,
                                    float* dA, float* dB, hipStream_t st) {
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
    const hipError_t et = launch_lora_transposes(d, F, A_pad, A_t, B_pad, B_t, st);
    if (et != hipSuccess) return et;
    const hipError_t eg = launch_lora_g(DT, Tt, gt, F, dZ, B_t, row_ptr, col_idx, nnz_cap, G, g_part, st);
    if (eg != hipSuccess) return eg;
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKFfnDx, st);
    hipLaunchKernelGGL((ffn_dsd_bf16<DT, true>), dim3((d + kRowsA - 1) / kRowsA, Tt), dim3(kThreads), 0, st,
                       (const uint16_t*)dZ, W_up_t, (long long)F, none, row_ptr, col_idx, gt, d,
                       nnz_cap, dX, (const uint16_t*)G, (const uint16_t*)A_t, 0);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfScope ps(kKLora, st);
  return launch_lora_grads(DT, Tt, gt, d, F, dZ, U, G, X, row_ptr, col_idx, nnz_cap, da_part, db_part, dA,
                           dB, st);
}

// Entry points of this file: dt selects the element type (kBf16 or kF16).
hipError_t launch_ffn_bf16(int dt, int pass, int Tt, int gt, int Fb, int d, int F, const uint16_t* A,
                           const uint16_t* W1, const uint16_t* b1, const uint16_t* W2,
                           const uint16_t* b2, const int* row_ptr, const int* col_idx, int nnz_cap,
                           uint16_t* act_out, const uint16_t* act_gate, uint16_t* out,
                           float* part, size_t part_bytes, hipStream_t st) {
  return LX_BY_DT(launch_ffn_bf16_t, pass, Tt, gt, Fb, d, F, A, W1, b1, W2, b2, row_ptr, col_idx,
                  nnz_cap, act_out, act_gate, out, part, part_bytes, st);
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
                                    float* g_part, float* da_part, float* db_part, uint16_t* dX,
                                    float* dA, float* dB, hipStream_t st) {
  return LX_BY_DT(launch_ffn_lora_bwd_bf16_t, Tt, gt, d, F, X, dY, H_act, U, W_down_t, W_up_t,
                  A_pad, B_pad, row_ptr, col_idx, nnz_cap, dZ, B_t, A_t, G, g_part, da_part, db_part, dX,
                  dA, dB, st);
}

}  // namespace lx
