// Block-sparse attention for gfx950 (Sec. VI-A).  The two block-sparse products
// of the paper -- SDD (scores on listed blocks) and DSD (probabilities times
// V) -- are fused with the softmax in flash style, so the score blocks live
// only in registers; the unit of work is the listed block, which is what keeps
// heads with different patterns balanced (Sec. VI-A, online combination).
//
// Layout of one workgroup (256 threads = 4 wavefronts): it works on a 64-row
// query block (forward, dQ) or a 64-row key block (dK/dV) at a time -- its OWN
// rows -- and streams the [64 x D] tiles of the blocks listed for that row of
// the mask through LDS.  Wavefront w owns 16 of the own rows and works on ALL
// 64 rows of every streamed tile, on the 16x16x32 MFMA with fp32 accumulators:
// no two wavefronts share own rows, so a row of the mask ends without any
// exchange -- each wavefront normalises and stores its own 16 rows -- and the
// accumulators are small enough (D/4 registers per product) for dK and dV to
// be summed in one pass at both head sizes.
//
// At the block densities of the paper a row of the mask lists only a few
// blocks, so a workgroup that handled one row would spend most of its life in
// the chain of dependent loads that starts it (row pointer -> list -> tiles).
// A workgroup therefore owns up to eight rows of one batch entry and walks
// their lists as ONE sequence of ring entries, written once into an LDS table:
// per row an entry that brings the row's own tiles, then its listed blocks.
// The transfers of the entries ahead -- of the same row or of the next -- are
// in flight while the current one is computed, and nothing in the walk reads
// global memory directly.  The rows of a group of up to four consecutive heads
// are ranked by the length of their lists and dealt to the group's workgroups
// in a snake over the ranks, which evens out the number of blocks per
// workgroup for any mask and between heads with long and short lists (all
// workgroups of a launch are resident at once, so the launch lasts as long as
// its longest workgroup).
//
// Data movement: tiles go from global memory straight into LDS
// (global_load_lds, 16 bytes per lane) through a ring of two or three stages.
// Transfers AND result stores are issued as assembly and waited for by
// counting instructions (vmcnt retires them in order), so that no
// compiler-inserted wait drains the stages in flight.  Tiles are row-major,
// unpadded, with the 16-byte slots of a row XOR-swizzled by the row index
// (bank spreading).
//
// Two tricks keep everything in one LDS layout and out of cross-lane shuffles:
//  * the first product is computed transposed (S^T = K Q^T), so every lane
//    holds scores of ONE query and the accumulator registers are fed straight
//    back as the B operand of the second product; the MFMA's k index may be
//    permuted freely as long as both operands agree;
//  * the operands that are needed k-major (V^T, K^T, Q^T, dO^T) are read from
//    the same row-major tile with the transposing LDS read (ds_read_b64_tr_b16:
//    within 16 lanes, lane j receives column c0+j of the four rows addressed by
//    lanes 0-3, 4-7, 8-11, 12-15).
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kAT = 256;                 // threads per workgroup
constexpr int kAW = kAT / kWave;         // wavefronts per workgroup
// ring stages / resident workgroups per CU (= wavefronts per SIMD) the kernels are compiled
// for, head size 64: forward 2 / 4, dQ 2 / 4 (128 registers, four of them spilled), dK/dV 3 / 3
// (measured against 3 / 3, 3 / 3 and 2 / 3, and 2 / 2 or 4 / 2); head size 128: 2 / 2
// everywhere (a stage is 32 KiB)
constexpr int kFwdNs64 = 2, kFwdOcc64 = 4, kDqNs64 = 2, kDqOcc64 = 4, kDkvNs64 = 3, kDkvOcc64 = 3;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSlack = 8.f;            // log2 units; see the forward kernel

template <int D>
__device__ __forceinline__ int tswz(int row) {
  return D == 64 ? ((row ^ (row >> 3)) & 7) : (row & 15);
}

// Per-lane element offsets (relative to the tile's first row) of the DMA instructions this
// wave issues for one [64 x D] tile.  One instruction moves 1 KiB = 64*16/(2D) rows.
template <int D>
struct TileDma {
  static constexpr int kSlots = D / 8;            // 16-byte slots per row
  static constexpr int kRowsPer = 64 / kSlots;    // rows per DMA instruction
  static constexpr int kPerWave = 64 / kRowsPer / kAW;
  long long off[kPerWave];
  __device__ __forceinline__ void init(long long ld) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int g = wave + kAW * u;
      const int row = kRowsPer * g + lane / kSlots;
      const int slot = (lane % kSlots) ^ tswz<D>(row);
      off[u] = (long long)row * ld + slot * 8;
    }
  }
  // tile_addr: LDS byte address of the destination tile
  __device__ __forceinline__ void issue(uint32_t tile_addr, const uint16_t* g0) const {
    const int wave = threadIdx.x / kWave;
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) dma16(g0 + off[u], tile_addr + (wave + kAW * u) * 1024);
  }
};

// LDS byte offsets inside a [64 x D] tile.  Element (row, col) sits at
// row*2D + (((col/8) ^ tswz(row)) << 4) + (col%8)*2.  tswz is linear over XOR and the row, slot
// and in-slot parts occupy disjoint bits, so the offset of (r0 + dr, c0 + dc) is the offset of
// (r0, c0) XOR a compile-time constant whenever r0/dr and c0/dc have disjoint bits.  The kernels
// keep ONE per-lane offset per access pattern in a register and derive every address of the
// pattern with an XOR by a constant (tile base addresses are multiples of the tile size, so they
// combine with OR): this is what keeps the address arithmetic out of the register budget.
template <int D>
__device__ __forceinline__ constexpr uint32_t tile_off(int row, int col) {
  return (uint32_t)(row * 2 * D + ((((col >> 3) ^ tswz<D>(row)) << 4)) + (col & 7) * 2);
}

// ---------------------------------------------------------------------------
// rows of a workgroup and the walk over their blocks
// ---------------------------------------------------------------------------
constexpr int kRMax = 8;   // rows of the mask per workgroup, at most

// The rows (query blocks, or key blocks for dK/dV) of one (batch, head) that workgroup g of G
// owns (see init for how they are chosen; with more than 64 blocks per head: slot j holds block
// j*G + g for even j and (j+1)*G - 1 - g for odd j, counted from the last block if `mirror`, so
// that with the group index as the slowest grid dimension the longest rows of a causal mask are
// dispatched first).  The row pointers of all slots are fetched once and kept in a small LDS table.
struct RowSet {
  const int* tab;   // LDS: blk[kRMax] (-1 = slot not used), rs[kRMax], n[kRMax], head[kRMax]
  int reg;          // the same table, entry i in lane i of every wavefront (one LDS read for all accessors)
  // The rows are those of `heads` consecutive heads, h0 .. (nb1 blocks each, their list rows one
  // after the other from head_row0), ranked and dealt together: heads whose lists differ in
  // length then share their workgroups instead of each keeping G of its own.
  // tab_lds: 4 * kRMax ints of LDS; contains a barrier: call from uniform control flow
  __device__ __forceinline__ void init(int* tab_lds, const int* __restrict__ row_ptr,
                                       int cap, int head_row0, int nb1, int heads, int h0,
                                       const uint8_t* __restrict__ head_active, int g, int G, int R,
                                       bool mirror) {
    tab = tab_lds;
    const int tid = threadIdx.x;
    const int nblk = nb1 * heads;
    if (nblk <= kWave) {
      // Groups balanced by the actual lengths of the lists: the rows of the head are ranked by
      // length (longest first, ties by index) and dealt to the G workgroups in a snake over the
      // ranks, rank k going to slot k / G of workgroup k % G or G - 1 - k % G.  Every workgroup
      // of the head computes the same ranking, one row per lane of its first wavefront.
      if (tid < kWave) {
        const bool valid = tid < nblk;
        const int hh = valid ? tid / nb1 : 0;       // head of this lane's row, relative to h0
        int rs = 0, n = -1;
        if (valid) {
          const bool head_on = !head_active || head_active[h0 + hh] != 0;
          rs = row_ptr[head_row0 + tid];
          // entries beyond the capacity of the index buffer are ignored
          n = head_on ? max(min(row_ptr[head_row0 + tid + 1], cap) - rs, 0) : 0;
        }
        // rank = rows with a longer list + rows before this one with an equally long list, by a
        // radix walk over the bits of the length with one ballot per bit: `gt` collects the lanes
        // known to be longer, `eq` those equal in the bits seen so far (lanes past the last row
        // carry key 0, below every row's)
        const unsigned key = (unsigned)(n + 1);
        unsigned long long gt = 0, eq = ~0ull;
#pragma unroll
        for (int bit = 6; bit >= 0; --bit) {     // a list has at most 64 entries here
          const unsigned long long set = __ballot((key >> bit) & 1u);
          if ((key >> bit) & 1u) {
            eq &= set;
          } else {
            gt |= eq & set;
            eq &= ~set;
          }
        }
        const int rank = __popcll(gt) + __popcll(eq & ((1ull << tid) - 1ull));
        const int j = rank / G, pos = rank - j * G;
        if (valid && ((j & 1) ? G - 1 - pos : pos) == g) {
          tab_lds[j] = tid - hh * nb1;
          tab_lds[kRMax + j] = rs;
          tab_lds[2 * kRMax + j] = n;
          tab_lds[3 * kRMax + j] = h0 + hh;
        }
      } else if (tid < kWave + kRMax) {
        // slots whose rank does not exist (the head has fewer rows than G * kRMax)
        const int j = tid - kWave;
        const int rank = j * G + ((j & 1) ? G - 1 - g : g);
        if (j >= R || rank >= nblk) {
          tab_lds[j] = -1;
          tab_lds[kRMax + j] = 0;
          tab_lds[2 * kRMax + j] = 0;
          tab_lds[3 * kRMax + j] = h0;
        }
      }
    } else if (tid < kRMax) {
      // more rows than lanes: fixed snake over the block index (balanced under a causal mask)
      const int j = tid;                       // (heads == 1 here: the launcher groups heads only
      int bj = (j & 1) ? (j + 1) * G - 1 - g : j * G + g;   //  when their rows fit one wavefront)
      const bool used = j < R && bj < nblk;
      if (mirror) bj = nblk - 1 - bj;
      const bool head_on = !head_active || head_active[h0] != 0;
      int rs = 0, n = 0;
      if (used) {
        rs = row_ptr[head_row0 + bj];
        n = head_on ? max(min(row_ptr[head_row0 + bj + 1], cap) - rs, 0) : 0;
      }
      tab_lds[j] = used ? bj : -1;
      tab_lds[kRMax + j] = rs;
      tab_lds[2 * kRMax + j] = n;
      tab_lds[3 * kRMax + j] = h0;
    }
    __syncthreads();
    reg = tab_lds[threadIdx.x % (4 * kRMax)];
  }
  // k is wave-uniform; the results are scalars taken from the register copy of the table
  __device__ __forceinline__ int blk(int k) const { return __builtin_amdgcn_readlane(reg, k); }
  __device__ __forceinline__ int rs(int k) const { return __builtin_amdgcn_readlane(reg, kRMax + k); }
  __device__ __forceinline__ int n(int k) const { return __builtin_amdgcn_readlane(reg, 2 * kRMax + k); }
  __device__ __forceinline__ int head(int k) const { return __builtin_amdgcn_readlane(reg, 3 * kRMax + k); }
};

// ---------------------------------------------------------------------------
// products of a wavefront: its 16 own rows against the 64 rows of a streamed tile
// ---------------------------------------------------------------------------
// 16x16x32 MFMA on 16-bit operands.  Operand a: lane l holds row l%16, k = 8*(l/16)..+7; operand
// b: column l%16, same k.  Accumulator register v of lane l is C[4*(l/16) + v][l%16].
template <int DT>
__device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  if constexpr (DT == kF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Per-lane offsets of the two access patterns into a streamed [64 x D] tile.
template <int D>
struct LaneOff16 {
  uint32_t rows;   // element (lane%16, 8*(lane/16)); row tile t, k slice kk: XOR tile_off(16t, 32kk)
  uint32_t tr;     // element (4*(lane/16) + (lane%16)/4, 4*(lane%4)); XOR tile_off(32kk + 16i, 16ct)
  __device__ __forceinline__ void init() {
    const int lane = threadIdx.x % kWave, g = lane / 16, j = lane % 16;
    rows = tile_off<D>(j, 8 * g);
    tr = tile_off<D>(4 * g + j / 4, 4 * (j % 4));
  }
};

// acc[t] = R[rows 16t + lane%16][:] . F^T for the four row tiles t of a row-major tile R in LDS
// (byte address `tile`); F: per-lane fragments of the own rows (column index = lane%16).
// Result register v of acc[t]: element (row 16t + 4*(lane/16) + v, own row lane%16).
template <int D, int DT>
__device__ __forceinline__ void mma_rows16(uint32_t tile, const LaneOff16<D>& lo,
                                           const uint4 (&frag)[D / 32], f32x4 (&acc)[4]) {
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  const uint32_t a0 = tile | lo.rows;
  uint4 a[D / 32][4];
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk)
#pragma unroll
    for (int t = 0; t < 4; ++t) a[kk][t] = lds_read16(a0 ^ tile_off<D>(16 * t, 32 * kk));
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk)
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = mfma16<DT>(a[kk][t], frag[kk], kk == 0 ? zero4 : acc[t]);
}

// Operands of out[ct] += T^T . P over all 64 rows of the row-major tile T (two k slices of 32
// rows), read with the transposing read.  k slot 8*(lane/16) + e of slice kk is row
// 32kk + 4*(lane/16) + e (e < 4) or 32kk + 16 + 4*(lane/16) + e - 4: the order in which the
// accumulator tiles 2kk and 2kk+1 of the first product hold their rows.
template <int D>
struct TrOps16 {
  uint4 a[2][D / 16];
};
template <int D>
__device__ __forceinline__ void load_tr16(uint32_t tile, const LaneOff16<D>& lo, TrOps16<D>& t) {
  const uint32_t a0 = tile | lo.tr;
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int ct = 0; ct < D / 16; ++ct) {
      const uint2 l = lds_read8_tr(a0 ^ tile_off<D>(32 * kk, 16 * ct));
      const uint2 h = lds_read8_tr(a0 ^ tile_off<D>(32 * kk + 16, 16 * ct));
      t.a[kk][ct] = make_uint4(l.x, l.y, h.x, h.y);
    }
}
// p[t][v]: accumulator-layout values of the [64 x 16] factor (rounded to the element type here)
template <int D, int DT>
__device__ __forceinline__ void mma_tr16(const TrOps16<D>& t, const f32x4 (&p)[4], f32x4 (&out)[D / 16]) {
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    uint4 b;
    b.x = pack2<DT>(p[2 * kk][0], p[2 * kk][1]);
    b.y = pack2<DT>(p[2 * kk][2], p[2 * kk][3]);
    b.z = pack2<DT>(p[2 * kk + 1][0], p[2 * kk + 1][1]);
    b.w = pack2<DT>(p[2 * kk + 1][2], p[2 * kk + 1][3]);
#pragma unroll
    for (int ct = 0; ct < D / 16; ++ct) out[ct] = mfma16<DT>(t.a[kk][ct], b, out[ct]);
  }
}

// Scores in the layout of mma_rows16 with the streamed rows (16t + 4*(lane/16) + v) being KEYS
// and the lane (own row `ql` of the block) the QUERY: keys after the query get -inf; `above`: the
// whole block lies on the excluded side of the diagonal.  mask_diag16_t: the roles exchanged
// (streamed rows are queries, the lane's own row is the key).
__device__ __forceinline__ void mask_diag16(f32x4 (&s)[4], int ql, bool above) {
  const int g = (threadIdx.x % kWave) / 16;
  const int x = above ? -1 : ql - 4 * g;     // key 16t + v > x: excluded
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (16 * t + v > x) s[t][v] = -INFINITY;
}
__device__ __forceinline__ void mask_diag16_t(f32x4 (&s)[4], int kl, bool above) {
  const int g = (threadIdx.x % kWave) / 16;
  const int x = above ? 64 : kl - 4 * g;     // query 16t + v < x: excluded
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (16 * t + v < x) s[t][v] = -INFINITY;
}

// accumulator layout [c-tile][v] (c = 16ct + 4*(lane/16) + v, row = lane%16) -> global
template <int D, int DT>
__device__ __forceinline__ void store_acc16(const f32x4 (&acc)[D / 16], float mul,
                                            uint16_t* __restrict__ dst_row) {
  const int g = (threadIdx.x % kWave) / 16;
#pragma unroll
  for (int ct = 0; ct < D / 16; ++ct) {
    uint2 o;
    o.x = pack2<DT>(acc[ct][0] * mul, acc[ct][1] * mul);
    o.y = pack2<DT>(acc[ct][2] * mul, acc[ct][3] * mul);
    *reinterpret_cast<uint2*>(dst_row + 16 * ct + 4 * g) = o;
  }
}
template <int N>
__device__ __forceinline__ void zero4(f32x4 (&a)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) a[i] = f32x4{0.f, 0.f, 0.f, 0.f};
}
// sum / maximum over the four lanes that share lane%16
__device__ __forceinline__ float sum_g(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}
__device__ __forceinline__ float max_g(float x) {
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}

// ---------------------------------------------------------------------------
// The work of a workgroup as ONE sequence of ring entries, built once into an LDS table: for
// every row slot with a non-empty list an OWN entry (the row's own tiles travel through the
// ring like any block, so a row starts without a load of its own), in the dQ kernel an AUX entry
// (a third own tile), then its listed blocks, the last one flagged.  Entry: bits 0..23 block
// index, 24..26 row slot.
// ---------------------------------------------------------------------------
constexpr int kTabCap = 512;                       // entries per fill of the table
constexpr int kEOwn = 1 << 30, kELast = 1 << 29, kEAux = 1 << 28;

__device__ __forceinline__ int entry_blk(int e) { return e & 0xFFFFFF; }
__device__ __forceinline__ int entry_slot(int e) { return (e >> 24) & 7; }

// Entries first .. first+cnt-1 of the sequence -> tab[0 .. cnt).  Uniform control flow; ends
// with a barrier.  offs[i]: first entry of slot i (offs[kRMax] = length of the sequence); pre:
// entries of a row before its first block (1: OWN; 2: OWN, AUX).
__device__ __forceinline__ void fill_table(int* tab, const RowSet& rows, const int* __restrict__ col_idx,
                                           const int (&offs)[kRMax + 1], int first, int cnt, int pre) {
  for (int e = first + (int)threadIdx.x; e < first + cnt; e += kAT) {
    int j = 0, o = 0;
#pragma unroll
    for (int i = 1; i < kRMax; ++i)
      if (e >= offs[i]) {
        j = i;
        o = offs[i];
      }
    const int it = e - o - pre;                    // < 0: the row's OWN (first) or AUX entry
    const int n = rows.tab[2 * kRMax + j];
    const int blk = it < 0 ? rows.tab[j] : col_idx[rows.tab[kRMax + j] + it];
    tab[e - first] = blk | (j << 24) | (it == -pre ? kEOwn : 0) | (it < 0 && it > -pre ? kEAux : 0) |
                     (it == n - 1 ? kELast : 0);
  }
  __syncthreads();
}

// s_waitcnt vmcnt(n') with the largest supported n' <= n (n wave-uniform): waiting for more than
// asked is always safe.
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
  switch (n) {
#define LX_W(N) case N: wait_vmcnt<N>(); break;
    LX_W(0) LX_W(1) LX_W(2) LX_W(3) LX_W(4) LX_W(5) LX_W(6) LX_W(7) LX_W(8) LX_W(9) LX_W(10)
    LX_W(11) LX_W(12) LX_W(13) LX_W(14) LX_W(15) LX_W(16) LX_W(17) LX_W(18) LX_W(19) LX_W(20)
    LX_W(21) LX_W(22) LX_W(23) LX_W(24) LX_W(25) LX_W(26) LX_W(27) LX_W(28) LX_W(29) LX_W(30)
    LX_W(31)
#undef LX_W
    default: wait_vmcnt<32>(); break;
  }
}

// Stores issued as assembly: the walk below counts every vector-memory instruction a wavefront
// issues (vmcnt retires loads and stores in order), so their number must not be the compiler's choice.
__device__ __forceinline__ void store8(uint16_t* p, uint2 v) {
  const unsigned long long d = (unsigned long long)v.x | ((unsigned long long)v.y << 32);
  asm volatile("global_store_dwordx2 %0, %1, off" ::"v"(p), "v"(d) : "memory");
}
__device__ __forceinline__ void store4(float* p, float v) {
  asm volatile("global_store_dword %0, %1, off" ::"v"(p), "v"(v) : "memory");
}
// accumulator layout -> global, D/16 store instructions
template <int D, int DT>
__device__ __forceinline__ void store_acc16_asm(const f32x4 (&acc)[D / 16], float mul,
                                                uint16_t* __restrict__ dst_row) {
  const int g = (threadIdx.x % kWave) / 16;
#pragma unroll
  for (int ct = 0; ct < D / 16; ++ct) {
    uint2 o;
    o.x = pack2<DT>(acc[ct][0] * mul, acc[ct][1] * mul);
    o.y = pack2<DT>(acc[ct][2] * mul, acc[ct][3] * mul);
    store8(dst_row + 16 * ct + 4 * g, o);
  }
}

// Walk over the sequence with a ring of NS stages: the transfers of entry t + NS - 1 are issued
// while entry t is computed.  issue_own / issue_aux / issue_blk(stage, e) start the transfers of an
// entry and issue exactly XOWN / XAUX / XBLK vector-memory instructions per wavefront (XAUX < 0: the
// rows have no AUX entry); row_begin(stage, e) takes the own rows' operands out of the stage of an
// OWN entry; aux(stage, e) consumes an AUX entry and issues exactly YAUX store instructions;
// comp(stage, e) consumes a block; row_end(e) stores the row's results with exactly YST store
// instructions per wavefront.  No other vector-memory instruction may be issued inside the walk: a
// wavefront waits for the transfers of entry t by counting what it has issued since (in order: the
// transfers of the entries after t and the stores issued meanwhile).
struct NoAux {
  __device__ __forceinline__ void operator()(int, int) const {}
};
template <int NS, int XOWN, int XAUX, int XBLK, int YAUX, int YST, class IssueOwn, class IssueAux, class IssueBlk,
          class RowBegin, class Aux, class Comp, class RowEnd>
__device__ __forceinline__ void walk_table(int* tab, const RowSet& rows, const int* __restrict__ col_idx,
                                           IssueOwn issue_own, IssueAux issue_aux, IssueBlk issue_blk,
                                           RowBegin row_begin, Aux aux, Comp comp, RowEnd row_end) {
  static_assert(NS >= 2 && NS <= 4, "ring depth");
  static_assert(YAUX < 256 && YST < 256, "store counts are kept a byte each");
  constexpr int kPre = XAUX >= 0 ? 2 : 1;
  int offs[kRMax + 1];
  offs[0] = 0;
#pragma unroll
  for (int i = 0; i < kRMax; ++i) {
    const int ni = rows.n(i);
    offs[i + 1] = offs[i] + (ni > 0 ? ni + kPre : 0);
  }
  const int total = offs[kRMax];
  auto entry = [&](int i) { return __builtin_amdgcn_readfirstlane(tab[i]); };
  auto issue = [&](int stage, int i) {
    const int e = entry(i);
    if (e & kEOwn)
      issue_own(stage, e);
    else if (XAUX >= 0 && (e & kEAux))
      issue_aux(stage, e);
    else
      issue_blk(stage, e);
  };
  auto issued_by = [&](int e) { return (e & kEOwn) ? XOWN : (XAUX >= 0 && (e & kEAux)) ? XAUX : XBLK; };
  for (int first = 0; first < total; first += kTabCap) {
    const int cnt = min(kTabCap, total - first);
    if (first > 0) lds_barrier();        // the previous table and the stages are no longer read
    fill_table(tab, rows, col_idx, offs, first, cnt, kPre);
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
      if (i < cnt) issue(i, i);
    unsigned hist = 0;                   // byte i: store instructions issued while entry t-1-i was consumed
    int stage = 0, istage = NS - 1;      // stage of entry t, stage entry t + NS - 1 goes to
    for (int t = 0; t < cnt; ++t) {
      const int e = entry(t);
      int n = 0;
#pragma unroll
      for (int u = 0; u < NS - 1; ++u) n += (hist >> (8 * u)) & 0xFF;
#pragma unroll
      for (int u = 1; u <= NS - 2; ++u)
        if (t + u < cnt) n += issued_by(entry(t + u));
      wait_vmcnt_dyn(n);
      lds_barrier();
      if (t + NS - 1 < cnt) issue(istage, t + NS - 1);
      int stores = 0;
      if (e & kEOwn) {
        row_begin(stage, e);
      } else if (XAUX >= 0 && (e & kEAux)) {
        aux(stage, e);
        stores = YAUX;
      } else {
        comp(stage, e);
        if (e & kELast) {
          row_end(e);
          stores = YST;
        }
      }
      hist = (hist << 8) | (unsigned)stores;
      stage = stage + 1 == NS ? 0 : stage + 1;
      istage = istage + 1 == NS ? 0 : istage + 1;
    }
  }
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
template <int D, int DT, int NS, int OCC>
__global__ __launch_bounds__(kAT, OCC) void attn_fwd_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t st[NS][2 * 64 * D];   // stage: K tile, V tile
  __shared__ int rowtab[4 * kRMax];
  __shared__ int btab[kTabCap];
  constexpr uint32_t kStage = 4 * 64 * D, kTile = 2 * 64 * D;   // bytes
  const int nqb = a.S / 64;
  const int b = blockIdx.x, h0 = blockIdx.y * a.vheads;   // batch entry fastest: see the launchers
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int g = lane / 16, ql = 16 * wave + lane % 16;    // this lane's query inside the block
  auto base_of = [&](int hh) { return (long long)b * a.sb + (long long)hh * a.sh; };
  auto stat_of = [&](int hh) { return ((long long)b * a.Hh + hh) * a.S; };
  const uint32_t st_addr = lds_addr(&st[0][0]);
  const uint32_t own_off = tile_off<D>(ql, 8 * g);       // this lane's fragments inside an own tile

  RowSet rows;
  rows.init(rowtab, a.row_ptr, a.nnz_cap, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h0) * nqb, nqb,
            a.vheads, h0, a.head_active, blockIdx.z, gridDim.z, a.rows_per_wg, true);
  // rows without a listed block (or of an inactive head): O = 0, LSE = -inf, nothing to read
  for (int j = 0; j < kRMax; ++j)
    if (rows.blk(j) >= 0 && rows.n(j) == 0) {
      f32x4 z[D / 16];
      zero4(z);
      const int hh = rows.head(j);
      store_acc16<D, DT>(z, 0.f, a.Out + base_of(hh) + (long long)(rows.blk(j) * 64 + ql) * a.ss);
      if (g == 0) a.LSE[stat_of(hh) + rows.blk(j) * 64 + ql] = -INFINITY;
    }

  TileDma<D> dma;
  dma.init(a.ss);
  LaneOff16<D> lo;
  lo.init();
  const float sc = a.scale * kLog2e;
  int qb = 0;
  long long qoff = 0, soff = 0;
  uint4 qf[D / 32];
  f32x4 o_acc[D / 16];
  float m = -INFINITY, lsum = 0.f;   // running maximum of the query; this lane's share of its sum

  auto issue_own = [&](int stage, int e) {
    const long long t0 = base_of(rows.head(entry_slot(e))) + (long long)entry_blk(e) * 64 * a.ss;
    dma.issue(st_addr + stage * kStage, a.Q + t0);
  };
  auto issue_blk = [&](int stage, int e) {
    const long long t0 = base_of(rows.head(entry_slot(e))) + (long long)entry_blk(e) * 64 * a.ss;
    const uint32_t dst = st_addr + stage * kStage;
    dma.issue(dst, a.K + t0);
    dma.issue(dst + kTile, a.V + t0);
  };
  auto row_begin = [&](int stage, int e) {
    qb = entry_blk(e);
    const int hh = rows.head(entry_slot(e));
    qoff = base_of(hh) + (long long)(qb * 64 + ql) * a.ss;
    soff = stat_of(hh) + qb * 64 + ql;
    const uint32_t q0 = (st_addr + stage * kStage) | own_off;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) qf[kk] = lds_read16(q0 ^ tile_off<D>(0, 32 * kk));
    zero4(o_acc);
    m = -INFINITY;
    lsum = 0.f;
  };
  auto comp = [&](int stage, int e) {
    const int col = entry_blk(e);
    const uint32_t stg = st_addr + stage * kStage;
    f32x4 s[4];
    mma_rows16<D, DT>(stg, lo, qf, s);          // S^T[key][q]
    TrOps16<D> vt;                              // independent of the scores: latency hides behind the softmax
    load_tr16<D>(stg + kTile, lo, vt);
    __builtin_amdgcn_sched_barrier(0);
    if (a.causal && col >= qb) mask_diag16(s, ql, col > qb);
    float mloc = fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3]));
#pragma unroll
    for (int t = 1; t < 4; ++t) mloc = fmaxf(mloc, fmaxf(fmaxf(s[t][0], s[t][1]), fmaxf(s[t][2], s[t][3])));
    mloc = max_g(mloc);
    // The reference point m of the running sums only has to bound the scores from above up to a
    // factor that fp32 holds comfortably: it follows the running maximum only when that has moved
    // by more than kSlack (then exp2(score - m) <= 2^kSlack), so most blocks need no rescaling.
    const float cand = mloc * sc;
    const float m_new = cand > m + kSlack ? cand : m;
    // a query none of whose keys so far is allowed keeps m = -inf; subtracting 0 instead keeps
    // the exponentials below at exp2(-inf) = 0 rather than exp2(-inf + inf)
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_use);
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[t][v], sc, -m_use));
        s[t][v] = p;
        psum += p;
      }
    lsum = lsum * alpha + psum;     // the four lanes of a query add their shares at the row's end
    const bool rescale = __any(alpha != 1.f && m != -INFINITY);
    m = m_new;
    if (rescale) {
#pragma unroll
      for (int ct = 0; ct < D / 16; ++ct) o_acc[ct] *= alpha;
    }
    mma_tr16<D, DT>(vt, s, o_acc);              // O^T += V^T P^T
  };
  auto row_end = [&](int) {
    const float l = sum_g(lsum);
    const bool any = l > 0.f;
    const float inv = any ? 1.f / l : 0.f;
    store_acc16_asm<D, DT>(o_acc, inv, a.Out + qoff);
    // (the four lanes of a query store the same value)
    store4(a.LSE + soff, any ? (m + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY);
  };
  walk_table<NS, TileDma<D>::kPerWave, -1, 2 * TileDma<D>::kPerWave, 0, D / 16 + 1>(
      btab, rows, a.col_idx, issue_own, NoAux(), issue_blk, row_begin, NoAux(), comp, row_end);
}

// ---------------------------------------------------------------------------
// backward, query side
// ---------------------------------------------------------------------------
template <int D, int DT, int NS, int OCC>
__global__ __launch_bounds__(kAT, OCC) void attn_bwd_dq_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t st[NS][2 * 64 * D];   // stage: K, V (or Q, dO; or O) tile
  __shared__ __attribute__((aligned(256))) float slse[NS][4][16];   // stage, wavefront: LSE of its 16 own rows
  __shared__ int rowtab[4 * kRMax];
  __shared__ int btab[kTabCap];
  constexpr uint32_t kStage = 4 * 64 * D, kTile = 2 * 64 * D;
  const int nqb = a.S / 64;
  const int b = blockIdx.x, h0 = blockIdx.y * a.vheads;   // batch entry fastest: see the launchers
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int g = lane / 16, ql = 16 * wave + lane % 16;
  auto base_of = [&](int hh) { return (long long)b * a.sb + (long long)hh * a.sh; };
  auto stat_of = [&](int hh) { return ((long long)b * a.Hh + hh) * a.S; };
  const uint32_t st_addr = lds_addr(&st[0][0]), slse_addr = lds_addr(&slse[0][0][0]);
  const uint32_t own_off = tile_off<D>(ql, 8 * g);

  RowSet rows;
  rows.init(rowtab, a.row_ptr, a.nnz_cap, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h0) * nqb, nqb,
            a.vheads, h0, a.head_active, blockIdx.z, gridDim.z, a.rows_per_wg, true);
  // rows without a listed block (or of an inactive head): dQ = 0, Delta = 0, nothing to read
  for (int j = 0; j < kRMax; ++j)
    if (rows.blk(j) >= 0 && rows.n(j) == 0) {
      f32x4 z[D / 16];
      zero4(z);
      const int hh = rows.head(j);
      store_acc16<D, DT>(z, 0.f, a.dQ + base_of(hh) + (long long)(rows.blk(j) * 64 + ql) * a.ss);
      if (g == 0) {
        a.Delta[stat_of(hh) + rows.blk(j) * 64 + ql] = 0.f;
        a.NegLse2[stat_of(hh) + rows.blk(j) * 64 + ql] = INFINITY;
      }
    }

  TileDma<D> dma;
  dma.init(a.ss);
  LaneOff16<D> lo;
  lo.init();
  const float sc = a.scale * kLog2e;
  int qb = 0;
  long long qoff = 0;
  long long soff = 0;
  uint4 qf[D / 32], dof[D / 32];
  float delta = 0.f, lse2 = 0.f;
  f32x4 dq_acc[D / 16];

  auto issue_own = [&](int stage, int e) {
    const long long t0 = base_of(rows.head(entry_slot(e))) + (long long)entry_blk(e) * 64 * a.ss;
    const uint32_t dst = st_addr + stage * kStage;
    dma.issue(dst, a.Q + t0);
    dma.issue(dst + kTile, a.dO + t0);
  };
  // the row's O tile, needed once for Delta = rowsum(dO . O), and the LSE of its 64 queries
  // (lanes 0-15 of wavefront w bring those of its own rows 16w .. 16w+15)
  auto issue_aux = [&](int stage, int e) {
    const int hh = rows.head(entry_slot(e)), blk = entry_blk(e);
    dma.issue(st_addr + stage * kStage, a.O + base_of(hh) + (long long)blk * 64 * a.ss);
    if (lane < 16) dma4(a.LSEin + stat_of(hh) + blk * 64 + ql, slse_addr + stage * 256 + wave * 64);
  };
  auto issue_blk = [&](int stage, int e) {
    const long long t0 = base_of(rows.head(entry_slot(e))) + (long long)entry_blk(e) * 64 * a.ss;
    const uint32_t dst = st_addr + stage * kStage;
    dma.issue(dst, a.K + t0);
    dma.issue(dst + kTile, a.V + t0);
  };
  auto row_begin = [&](int stage, int e) {
    qb = entry_blk(e);
    const int slot = entry_slot(e);
    qoff = base_of(rows.head(slot)) + (long long)(qb * 64 + ql) * a.ss;
    soff = stat_of(rows.head(slot)) + qb * 64 + ql;
    const uint32_t q0 = (st_addr + stage * kStage) | own_off;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      qf[kk] = lds_read16(q0 ^ tile_off<D>(0, 32 * kk));
      dof[kk] = lds_read16((q0 + kTile) ^ tile_off<D>(0, 32 * kk));
    }
    zero4(dq_acc);
  };
  // Delta and -LSE in log2 units of the row, kept for its blocks and written for the key-side kernel
  auto aux = [&](int stage, int) {
    const uint32_t o0 = (st_addr + stage * kStage) | own_off;
    float sum = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      const uint4 of = lds_read16(o0 ^ tile_off<D>(0, 32 * kk));
      const uint32_t x[4] = {dof[kk].x, dof[kk].y, dof[kk].z, dof[kk].w};
      const uint32_t y[4] = {of.x, of.y, of.z, of.w};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        sum += to_f32<DT>(x[q] & 0xFFFFu) * to_f32<DT>(y[q] & 0xFFFFu) + to_f32<DT>(x[q] >> 16) * to_f32<DT>(y[q] >> 16);
    }
    delta = sum_g(sum);
    // a row whose listed blocks hold no allowed key has LSE = -inf: +inf here makes every
    // probability exp2(score - inf) = 0, also for excluded scores (-inf), which -(-inf) would not
    const float lse_in = slse[stage][wave][lane % 16];
    lse2 = lse_in == -INFINITY ? INFINITY : lse_in * kLog2e;
    // (the four lanes of a query store the same values)
    store4(a.Delta + soff, delta);
    store4(a.NegLse2 + soff, -lse2);
  };
  auto comp = [&](int stage, int e) {
    const int col = entry_blk(e);
    const uint32_t stg = st_addr + stage * kStage;
    f32x4 s[4], dp[4];
    mma_rows16<D, DT>(stg, lo, qf, s);                   // S^T[key][q]
    mma_rows16<D, DT>(stg + kTile, lo, dof, dp);         // dP^T[key][q]
    if (a.causal && col >= qb) mask_diag16(s, ql, col > qb);   // excluded keys: P = exp2(-inf) = 0
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[t][v], sc, -lse2));
        s[t][v] = p * (dp[t][v] - delta);       // dS^T
      }
    __builtin_amdgcn_sched_barrier(0);
    TrOps16<D> kt;
    load_tr16<D>(stg, lo, kt);
    mma_tr16<D, DT>(kt, s, dq_acc);             // dQ^T += K^T dS^T
  };
  auto row_end = [&](int) { store_acc16_asm<D, DT>(dq_acc, a.scale, a.dQ + qoff); };
  walk_table<NS, 2 * TileDma<D>::kPerWave, TileDma<D>::kPerWave + 1, 2 * TileDma<D>::kPerWave, 2, D / 16>(
      btab, rows, a.col_idx, issue_own, issue_aux, issue_blk, row_begin, aux, comp, row_end);
}

// ---------------------------------------------------------------------------
// backward, key side: a wavefront owns 16 keys; the streamed tiles are Q and dO of the listed
// query blocks, with the queries' -LSE*log2(e) and Delta beside them
// ---------------------------------------------------------------------------
template <int D, int DT, int NS, int OCC>
__global__ __launch_bounds__(kAT, OCC) void attn_bwd_dkv_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t st[NS][2 * 64 * D];   // stage: Q, dO (or K, V) tile
  __shared__ __attribute__((aligned(512))) float sstat[NS][4][32];   // stage, query tile: -LSE*log2e [16], Delta [16]
  __shared__ int rowtab[4 * kRMax];
  __shared__ int btab[kTabCap];
  constexpr uint32_t kStage = 4 * 64 * D, kTile = 2 * 64 * D;
  const int nkb = a.S / 64;
  const int b = blockIdx.x, h0 = blockIdx.y * a.vheads;   // batch entry fastest: see the launchers
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int g = lane / 16, kl = 16 * wave + lane % 16;    // this lane's key inside the block
  auto base_of = [&](int hh) { return (long long)b * a.sb + (long long)hh * a.sh; };
  auto stat_of = [&](int hh) { return ((long long)b * a.Hh + hh) * a.S; };
  const uint32_t st_addr = lds_addr(&st[0][0]), sstat_addr = lds_addr(&sstat[0][0][0]);
  const uint32_t own_off = tile_off<D>(kl, 8 * g);

  RowSet rows;
  rows.init(rowtab, a.crow_ptr, a.cnnz_cap, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h0) * nkb, nkb,
            a.vheads, h0, a.head_active, blockIdx.z, gridDim.z, a.rows_per_wg, false);
  // key blocks used by no query block: zero gradients, nothing to read
  for (int j = 0; j < kRMax; ++j)
    if (rows.blk(j) >= 0 && rows.n(j) == 0) {
      f32x4 z[D / 16];
      zero4(z);
      const long long koff = base_of(rows.head(j)) + (long long)(rows.blk(j) * 64 + kl) * a.ss;
      store_acc16<D, DT>(z, 0.f, a.dV + koff);
      store_acc16<D, DT>(z, 0.f, a.dK + koff);
    }

  TileDma<D> dma;
  dma.init(a.ss);
  LaneOff16<D> lo;
  lo.init();
  const float sc = a.scale * kLog2e;
  // lanes 0-15 of wave w bring -LSE*log2(e), lanes 16-31 Delta of queries 16w .. 16w+15 of a block
  const float* stat_src = (lane < 16 ? a.NegLse2 : a.Delta) + 16 * wave + lane % 16;
  int kb = 0;
  long long koff = 0;
  uint4 kf[D / 32], vf[D / 32];
  f32x4 dk_acc[D / 16], dv_acc[D / 16];

  auto issue_own = [&](int stage, int e) {
    const long long t0 = base_of(rows.head(entry_slot(e))) + (long long)entry_blk(e) * 64 * a.ss;
    const uint32_t dst = st_addr + stage * kStage;
    dma.issue(dst, a.K + t0);
    dma.issue(dst + kTile, a.V + t0);
  };
  auto issue_blk = [&](int stage, int e) {
    const int hh = rows.head(entry_slot(e)), qbk = entry_blk(e);
    const long long t0 = base_of(hh) + (long long)qbk * 64 * a.ss;
    const uint32_t dst = st_addr + stage * kStage;
    dma.issue(dst, a.Q + t0);
    dma.issue(dst + kTile, a.dO + t0);
    if (lane < 32) dma4(stat_src + stat_of(hh) + qbk * 64, sstat_addr + stage * 512 + wave * 128);
  };
  auto row_begin = [&](int stage, int e) {
    kb = entry_blk(e);
    koff = base_of(rows.head(entry_slot(e))) + (long long)(kb * 64 + kl) * a.ss;
    const uint32_t k0 = (st_addr + stage * kStage) | own_off;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      kf[kk] = lds_read16(k0 ^ tile_off<D>(0, 32 * kk));
      vf[kk] = lds_read16((k0 + kTile) ^ tile_off<D>(0, 32 * kk));
    }
    zero4(dk_acc);
    zero4(dv_acc);
  };
  auto comp = [&](int stage, int e) {
    const int col = entry_blk(e);
    const uint32_t stg = st_addr + stage * kStage;
    f32x4 s[4], dp[4];
    mma_rows16<D, DT>(stg, lo, kf, s);                   // S[q][key]
    mma_rows16<D, DT>(stg + kTile, lo, vf, dp);          // dP[q][key]
    // diagonal block: here the rows of the score tile are queries and the lane is the key
    if (a.causal && col <= kb) mask_diag16_t(s, kl, col < kb);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float4 nl = *reinterpret_cast<const float4*>(&sstat[stage][t][4 * g]);
      const float4 dl = *reinterpret_cast<const float4*>(&sstat[stage][t][16 + 4 * g]);
      const float nls[4] = {nl.x, nl.y, nl.z, nl.w}, dls[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[t][v], sc, nls[v]));
        s[t][v] = p;                                  // P
        dp[t][v] = p * (dp[t][v] - dls[v]);           // dS
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    {
      TrOps16<D> dot;
      load_tr16<D>(stg + kTile, lo, dot);
      mma_tr16<D, DT>(dot, s, dv_acc);                // dV^T += dO^T P
    }
    {
      TrOps16<D> qt;
      load_tr16<D>(stg, lo, qt);
      mma_tr16<D, DT>(qt, dp, dk_acc);                // dK^T += Q^T dS
    }
  };
  auto row_end = [&](int) {
    store_acc16_asm<D, DT>(dv_acc, 1.f, a.dV + koff);
    store_acc16_asm<D, DT>(dk_acc, a.scale, a.dK + koff);
  };
  walk_table<NS, 2 * TileDma<D>::kPerWave, -1, 2 * TileDma<D>::kPerWave + 1, 0, 2 * (D / 16)>(
      btab, rows, a.ccol_idx, issue_own, NoAux(), issue_blk, row_begin, NoAux(), comp, row_end);
}

// Rows per workgroup: the smallest count with which all workgroups of the launch are resident at
// once on the chip's `slots` workgroup slots (a causal mask keeps the groups balanced for every
// count, because slots are filled in pairs k, 2G-1-k), unless the caller fixed the number.
static thread_local int g_rows_per_wg = 0;   // one value per host thread
hipError_t set_attn_rows_per_wg(int r) {
  if (r < 0 || r > kRMax) return hipErrorInvalidValue;
  g_rows_per_wg = r;
  return hipSuccess;
}
// Heads per group of workgroups: as many consecutive heads (4, 2 or 1) as divide the head count
// and whose rows one wavefront can rank (64 lanes).  The rows of the group are dealt to its
// workgroups together, so heads with long and with short lists even each other out.
static int heads_per_group(int nblk, int heads) {
  for (int v = 4; v > 1; v /= 2)
    if (heads % v == 0 && v * nblk <= kWave) return v;
  return 1;
}
static int rows_per_wg(int nblk, int heads, int B, int slots) {
  int r = 1;
  while (r < kRMax && (long long)((nblk + r - 1) / r) * heads * B > slots) ++r;
  if (g_rows_per_wg > 0) r = g_rows_per_wg;
  return r > nblk ? nblk : r;
}

// Grid: (batch entry, head group, workgroup of the group).  Workgroups go to the eight XCDs round
// robin by their linear index, so with the batch entry fastest an XCD gets the same mix of heads
// as every other one (the masks of the batch entries are the same or alike, those of the heads
// are not), and all workgroups of a (batch, head) pair share one L2.
template <int D, int DT>
static hipError_t launch_fwd(AttnArgs a, int B, hipStream_t st) {
  ProfScope ps(kKAttnFwd, st);
  const int nblk = a.S / 64;
  a.vheads = heads_per_group(nblk, a.Hh);
  constexpr int kNs = D == 64 ? kFwdNs64 : 2, kOcc = D == 64 ? kFwdOcc64 : 2;
  a.rows_per_wg = rows_per_wg(nblk, a.Hh, B, kCUs * kOcc);
  const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
  hipLaunchKernelGGL((attn_fwd_bf16<D, DT, kNs, kOcc>), dim3(B, a.Hh / a.vheads, G * a.vheads), dim3(kAT), 0,
                     st, a);
  return hipGetLastError();
}

template <int D, int DT>
static hipError_t launch_bwd(AttnArgs a, int B, hipStream_t st) {
  const int nblk = a.S / 64;
  a.vheads = heads_per_group(nblk, a.Hh);
  {
    ProfScope ps(kKAttnDq, st);
    constexpr int kNs = D == 64 ? kDqNs64 : 2, kOcc = D == 64 ? kDqOcc64 : 2;
    a.rows_per_wg = rows_per_wg(nblk, a.Hh, B, kCUs * kOcc);
    const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
    hipLaunchKernelGGL((attn_bwd_dq_bf16<D, DT, kNs, kOcc>), dim3(B, a.Hh / a.vheads, G * a.vheads),
                       dim3(kAT), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKAttnDkv, st);
    constexpr int kNs = D == 64 ? kDkvNs64 : 2, kOcc = D == 64 ? kDkvOcc64 : 2;
    a.rows_per_wg = rows_per_wg(nblk, a.Hh, B, kCUs * kOcc);
    const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
    hipLaunchKernelGGL((attn_bwd_dkv_bf16<D, DT, kNs, kOcc>), dim3(B, a.Hh / a.vheads, G * a.vheads),
                       dim3(kAT), 0, st, a);
  }
  return hipGetLastError();
}

// dt: element type (kBf16 or kF16)
hipError_t launch_attn_fwd_bf16(int dt, int D, int B, const AttnArgs& a, hipStream_t st) {
  if (dt == kF16) return D == 64 ? launch_fwd<64, kF16>(a, B, st) : launch_fwd<128, kF16>(a, B, st);
  return D == 64 ? launch_fwd<64, kBf16>(a, B, st) : launch_fwd<128, kBf16>(a, B, st);
}
hipError_t launch_attn_bwd_bf16(int dt, int D, int B, const AttnArgs& a, hipStream_t st) {
  if (dt == kF16) return D == 64 ? launch_bwd<64, kF16>(a, B, st) : launch_bwd<128, kF16>(a, B, st);
  return D == 64 ? launch_bwd<64, kBf16>(a, B, st) : launch_bwd<128, kBf16>(a, B, st);
}

}  // namespace lx
