// Block-sparse attention for gfx950 (Sec. VI-A).  The two block-sparse products
// of the paper -- SDD (scores on listed blocks) and DSD (probabilities times
// V) -- are fused with the softmax in flash style, so the score blocks live
// only in registers; the unit of work is the listed block, which is what keeps
// heads with different patterns balanced (Sec. VI-A, online combination).
//
// Layout of one workgroup (256 threads = 4 wavefronts): it works on a 64-row
// query block (forward, dQ) or a 64-row key block (dK/dV) at a time -- its OWN
// rows -- and streams the [64 x D] tiles of the blocks listed for that row of
// the mask through LDS.  Wavefront w owns 32 of the own rows (w % 2) and works
// on 32 of the 64 rows of every streamed tile (w / 2).  The two wavefronts that
// share own rows keep separate partial results (running maximum, sum and
// output in the forward pass; gradient sums in the backward pass) and combine
// them once per row of the mask, through LDS; inside the walk over the blocks
// they never communicate.  Splitting the streamed tile, rather than giving a
// wavefront more own rows, halves the time one block takes on the critical
// path of a row, which is what bounds a kernel whose rows list few blocks.
// All products run on the 32x32x16 bf16 MFMA with fp32 accumulators.
//
// At the block densities of the paper a row of the mask lists only a few
// blocks, so a workgroup that handled one row would spend most of its life in
// the chain of dependent loads that starts it (row pointer -> list -> tiles).
// A workgroup therefore owns up to eight rows of one batch entry and walks
// their lists as ONE stream of blocks: the metadata of all its rows is read up
// front, and the tile transfer of the next block -- of the same row or of the
// next one -- is always in flight while the current block is computed.  The
// rows of a group of up to four consecutive heads are ranked by the length of
// their lists and dealt to the group's workgroups in a snake over the ranks,
// which evens out the number of blocks per workgroup for any mask and between
// heads with long and short lists (all workgroups of a launch are resident at
// once, so the launch lasts as long as its longest workgroup).
//
// Data movement: the [64 x D] tiles of the listed blocks go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane), double buffered.  The
// transfers are issued as assembly and waited for explicitly, so that no
// compiler-inserted wait drains the stage in flight.  Tiles are row-major,
// unpadded, with the 16-byte slots of a row XOR-swizzled by the row index
// (bank spreading).
//
// Two tricks keep everything in one LDS layout and out of cross-lane shuffles:
//  * the first product is computed transposed (S^T = K Q^T), so every lane
//    holds scores of ONE query and the accumulator registers are fed straight
//    back as the B operand of the second product; the MFMA's k index may be
//    permuted freely as long as both operands agree: { 16s+4h..+3, 16s+8+4h..+3 };
//  * the operands that are needed k-major (V^T, K^T, Q^T, dO^T) are read from
//    the same row-major tile with the transposing LDS read (ds_read_b64_tr_b16:
//    within 16 lanes, lane j receives column c0+j of the four rows addressed by
//    lanes 0-3, 4-7, 8-11, 12-15).
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kAT = 256;                 // threads per workgroup
constexpr int kAW = kAT / kWave;         // wavefronts per workgroup
// resident workgroups per CU (= wavefronts per SIMD) the D = 64 kernels are compiled for
constexpr int kFwdOcc64 = 4, kDqOcc64 = 3, kDkvOcc64 = 2;
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

// Per-lane offsets of the two access patterns of a wavefront that works on rows 32*half..+31
// of the streamed tiles.
template <int D>
struct LaneOff {
  uint32_t rows;   // mma_rows: element (32*half + lane%32, 8*(lane/32))
  uint32_t tr;     // load_tr: element (32*half + 4*(lane/32) + (lane%16)/4, 16*((lane/16)%2) + 4*(lane%4))
  __device__ __forceinline__ void init(int half) {
    const int lane = threadIdx.x % kWave, h2 = lane / 32, j = lane % 16;
    rows = tile_off<D>(32 * half + lane % 32, 8 * h2);
    tr = tile_off<D>(32 * half + 4 * h2 + j / 4, 16 * ((lane / 16) % 2) + 4 * (j % 4));
  }
};

// acc = R[rows 32*half + lane%32][:] . F^T   where R is a row-major tile in LDS (byte address
// `tile`) and F the per-lane register fragments (column index = lane%32).  Result register v of
// a lane is element (row 32*half + 8*(v/4) + 4*(lane/32) + v%4, column lane%32).  The operand
// reads are issued ahead of the MFMAs, so their LDS latency is paid once, not once per k16 slice.
template <int D, int DT>
__device__ __forceinline__ void mma_rows(uint32_t tile, const LaneOff<D>& lo,
                                         const uint4 (&frag)[D / 16], f32x16& acc) {
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const uint32_t a0 = tile | lo.rows;
  uint4 a[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) a[s] = lds_read16(a0 ^ tile_off<D>(0, 16 * s));
  __builtin_amdgcn_sched_barrier(0);   // keep the reads above: the scheduler would sink them
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    // the first product starts from a literal zero (no register clearing)
    acc = mfma32<DT>(a[s], frag[s], s == 0 ? zero16 : acc);
}

// Operands of out[ct] += T[rows 32*half ..+31][:]^T . P (two k-slices of 16 rows of T), read from
// the row-major [64 x D] tile T in LDS (byte address `tile`) with the transposing read.
template <int D>
struct TrOps {
  uint4 a[2][D / 32];
};
template <int D>
__device__ __forceinline__ void load_tr(uint32_t tile, const LaneOff<D>& lo, TrOps<D>& t) {
  const uint32_t a0 = tile | lo.tr;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) {
      const uint2 l = lds_read8_tr(a0 ^ tile_off<D>(16 * i, 32 * ct));
      const uint2 h = lds_read8_tr(a0 ^ tile_off<D>(16 * i + 8, 32 * ct));
      t.a[i][ct] = make_uint4(l.x, l.y, h.x, h.y);
    }
}
// p[v]: accumulator-layout values of the [32 x 32] factor P (rounded to bf16 here).
template <int D, int DT>
__device__ __forceinline__ void mma_tr(const TrOps<D>& t, const f32x16& p, f32x16 (&out)[D / 32]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    uint4 b;
    b.x = pack2<DT>(p[8 * i + 0], p[8 * i + 1]);
    b.y = pack2<DT>(p[8 * i + 2], p[8 * i + 3]);
    b.z = pack2<DT>(p[8 * i + 4], p[8 * i + 5]);
    b.w = pack2<DT>(p[8 * i + 6], p[8 * i + 7]);
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) out[ct] = mfma32<DT>(t.a[i][ct], b, out[ct]);
  }
}

// Diagonal block of a causal mask, scores in accumulator layout with the streamed rows (index
// 32*part + 8*(v/4) + 4*(lane/32) + v%4) being KEYS and the lane (32*own + lane%32) the QUERY:
// keys after the query get -inf.  mask_diag_t: the same with the roles exchanged (rows are
// queries, the lane is the key).
// `above`: the block lies wholly on the excluded side of the diagonal (a block the list should not
// hold under a causal mask): every score of it is excluded.
__device__ __forceinline__ void mask_diag(f32x16& s, int own, int part, bool above) {
  const int lane = threadIdx.x % kWave;
  // key 8*(v/4) + v%4 > x: excluded
  const int x = above ? -1 : lane % 32 + 32 * (own - part) - 4 * (lane / 32);
#pragma unroll
  for (int v = 0; v < 16; ++v)
    if (8 * (v / 4) + v % 4 > x) s[v] = -INFINITY;
}
__device__ __forceinline__ void mask_diag_t(f32x16& s, int own, int part, bool above) {
  const int lane = threadIdx.x % kWave;
  // query 8*(v/4) + v%4 < x: excluded
  const int x = above ? 64 : lane % 32 + 32 * (own - part) - 4 * (lane / 32);
#pragma unroll
  for (int v = 0; v < 16; ++v)
    if (8 * (v / 4) + v % 4 < x) s[v] = -INFINITY;
}

template <int N>
__device__ __forceinline__ void zero(f32x16 (&a)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) a[i][v] = 0.f;
}

// accumulator layout [c-tile][v] (c = 32ct + 8(v/4) + 4(lane/32) + v%4, row = lane%32) -> global;
// c-tiles C0 .. C0+N-1 only
template <int D, int DT, int C0 = 0, int N = D / 32>
__device__ __forceinline__ void store_acc(const f32x16 (&acc)[D / 32], float mul,
                                          uint16_t* __restrict__ dst_row) {
  const int h2 = (threadIdx.x % kWave) / 32;
#pragma unroll
  for (int ct = C0; ct < C0 + N; ++ct)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 o;
      o.x = pack2<DT>(acc[ct][4 * g] * mul, acc[ct][4 * g + 1] * mul);
      o.y = pack2<DT>(acc[ct][4 * g + 2] * mul, acc[ct][4 * g + 3] * mul);
      *reinterpret_cast<uint2*>(dst_row + 32 * ct + 8 * g + 4 * h2) = o;
    }
}

// Exchange of accumulators between the two wavefronts that share own rows (parts 0 and 1),
// through an LDS area of 4 * (D/4) * 64 floats (exactly one stage of tiles).  Each of the two
// finishes one half of the c-tiles: part p keeps tiles p*D/64 .. and hands the other half to its
// partner, so both halves of the pair share the combination and the stores.  Layout
// [writer's part][own][register][lane]: a wavefront's 64 lanes write and read consecutive words.
template <int D, int PART>
__device__ __forceinline__ void put_half(float* area, int own, const f32x16 (&acc)[D / 32]) {
  constexpr int kN = D / 64, kC0 = (1 - PART) * kN;   // the partner's tiles
  float* p = area + (PART * 2 + own) * (16 * kN) * 64 + threadIdx.x % kWave;
#pragma unroll
  for (int ct = 0; ct < kN; ++ct)
#pragma unroll
    for (int v = 0; v < 16; ++v) p[(16 * ct + v) * 64] = acc[kC0 + ct][v];
}
// own tiles: acc = acc * mine + partner's * theirs
template <int D, int PART>
__device__ __forceinline__ void merge_half(const float* area, int own, float mine, float theirs,
                                           f32x16 (&acc)[D / 32]) {
  constexpr int kN = D / 64, kC0 = PART * kN;
  const float* p = area + ((1 - PART) * 2 + own) * (16 * kN) * 64 + threadIdx.x % kWave;
#pragma unroll
  for (int ct = 0; ct < kN; ++ct)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      acc[kC0 + ct][v] = acc[kC0 + ct][v] * mine + p[(16 * ct + v) * 64] * theirs;
}

// One-sided variant (the wavefront with part 1 hands over all its tiles, part 0 finishes them),
// area layout [own][register][lane]: used where the symmetric exchange does not fit the
// register budget.
template <int D>
__device__ __forceinline__ void put_all(float* area, int own, const f32x16 (&acc)[D / 32]) {
  float* p = area + own * (D / 2) * 64 + threadIdx.x % kWave;
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
    for (int v = 0; v < 16; ++v) p[(16 * ct + v) * 64] = acc[ct][v];
}
template <int D>
__device__ __forceinline__ void merge_all(const float* area, int own, f32x16 (&acc)[D / 32]) {
  const float* p = area + own * (D / 2) * 64 + threadIdx.x % kWave;
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[ct][v] += p[(16 * ct + v) * 64];
}

// ---------------------------------------------------------------------------
// rows of a workgroup and the walk over their blocks
// ---------------------------------------------------------------------------
constexpr int kRMax = 8;   // rows of the mask per workgroup, at most

typedef const __attribute__((address_space(4))) int* ScalarIntPtr;   // loads become scalar loads

// The rows (query blocks, or key blocks for dK/dV) of one (batch, head) that workgroup g of G
// owns (see init for how they are chosen; with more than 64 blocks per head: slot j holds block
// j*G + g for even j and (j+1)*G - 1 - g for odd j, counted from the last block if `mirror`, so
// that with the group index as the slowest grid dimension the longest rows of a causal mask are
// dispatched first).  The row pointers
// of all slots are fetched once, before the walk, and kept in a small LDS table; the walk reads
// the table and the list entries with LDS reads and scalar loads, which are counted apart from
// the vector-memory counter that the tile transfers are waited on.
struct RowSet {
  ScalarIntPtr col_idx;
  const int* tab;   // LDS: blk[kRMax] (-1 = slot not used), rs[kRMax], n[kRMax], head[kRMax]
  // The rows are those of `heads` consecutive heads, h0 .. (nb1 blocks each, their list rows one
  // after the other from head_row0), ranked and dealt together: heads whose lists differ in
  // length then share their workgroups instead of each keeping G of its own.
  // tab_lds: 4 * kRMax ints of LDS; contains a barrier: call from uniform control flow
  __device__ __forceinline__ void init(int* tab_lds, const int* __restrict__ row_ptr,
                                       const int* __restrict__ col_idx_, int cap, int head_row0,
                                       int nb1, int heads, int h0,
                                       const uint8_t* __restrict__ head_active, int g, int G, int R,
                                       bool mirror) {
    col_idx = (ScalarIntPtr)col_idx_;
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
        int rank = 0;
        for (int q = 0; q < nblk; ++q) {
          const int nq = __builtin_amdgcn_readlane(n, q);
          rank += (nq > n || (nq == n && q < tid)) ? 1 : 0;
        }
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
  }
  // k is wave-uniform; so are the results, and they are made scalar registers
  __device__ __forceinline__ int blk(int k) const { return __builtin_amdgcn_readfirstlane(tab[k]); }
  __device__ __forceinline__ int rs(int k) const {
    return __builtin_amdgcn_readfirstlane(tab[kRMax + k]);
  }
  __device__ __forceinline__ int n(int k) const {
    return __builtin_amdgcn_readfirstlane(tab[2 * kRMax + k]);
  }
  __device__ __forceinline__ int head(int k) const {
    return __builtin_amdgcn_readfirstlane(tab[3 * kRMax + k]);
  }
  // listed block `it` of slot k (both wave-uniform, it < n(k))
  __device__ __forceinline__ int col(int k, int it) const { return col_idx[rs(k) + it]; }
  // first slot >= k with a non-empty list, kRMax if none
  __device__ __forceinline__ int next_row(int k) const {
    while (k < kRMax && n(k) == 0) ++k;
    return k;
  }
};

// Walk over all listed blocks of the row set as one double-buffered stream.  issue(stage, k, col)
// starts the transfer of the tiles of block `col` of the row in slot k into stage 0/1; comp(stage, col) consumes
// them; row_begin(k) loads the per-row state, row_end(k, stage) combines and stores it and may
// use the LDS of `stage` (the one just consumed) after a barrier of its own.  The transfer of
// the next block, which may belong to the next row, is issued before the current one is
// computed, and the list entry after that one is fetched at the same time.  A wave first waits
// for its own transfers (vmcnt), the barrier then makes the whole stage visible and retires the
// reads of the stage about to be refilled.  All control flow is workgroup-uniform.
// With OWN_PF the per-row state comes from tiles that prefetch(k) transfers into an LDS area of
// the kernel's own (one row ahead: right after the barrier that follows row_begin of the
// current row, when no wavefront reads the area any more), so row_begin reads LDS instead of
// waiting for global memory at every row; a row of a single block, whose successor's tiles were
// requested in the same step, waits for them before it hands over.
template <bool OWN_PF, class RowBegin, class Prefetch, class Issue, class Comp, class RowEnd>
__device__ __forceinline__ void walk_rows(const RowSet& rows, RowBegin row_begin, Prefetch prefetch,
                                          Issue issue, Comp comp, RowEnd row_end) {
  int ki = rows.next_row(0), iti = 0;
  if (ki >= kRMax) return;
  int ni = rows.n(ki);                 // length of the list the issue side is in
  int coli = rows.col(ki, 0);          // block whose transfer is issued next
  issue(0, ki, coli);
  int kc = ki, itc = 0, colc = coli, nc = ni;
  auto advance = [&]() {
    if (++iti == ni) {
      ki = rows.next_row(ki + 1);
      iti = 0;
      if (ki < kRMax) ni = rows.n(ki);
    }
    if (ki < kRMax) coli = rows.col(ki, iti);
  };
  advance();
  if (OWN_PF) {
    prefetch(kc);
    wait_vmcnt<0>();
    lds_barrier();
  }
  row_begin(kc);
  bool want_pf = OWN_PF;               // the row after kc still has to be requested
  int t_pf = -1;                       // step in which the last request was made
  for (int t = 0;; ++t) {
    wait_vmcnt<0>();
    lds_barrier();
    const bool more = ki < kRMax;
    if (OWN_PF && want_pf) {
      const int kn = rows.next_row(kc + 1);
      if (kn < kRMax) {
        prefetch(kn);
        t_pf = t;
      }
      want_pf = false;
    }
    if (more) issue((t + 1) & 1, ki, coli);
    comp(t & 1, colc);
    const bool last = itc + 1 == nc;
    if (last) row_end(kc, t & 1);
    if (!more) break;
    if (last) {
      if (OWN_PF && t_pf == t) {
        wait_vmcnt<0>();
        lds_barrier();
      }
      row_begin(ki);
      want_pf = OWN_PF;
      nc = ni;
    }
    kc = ki;
    itc = iti;
    colc = coli;
    advance();
  }
}

// ---------------------------------------------------------------------------
// forward: O, LSE for the query blocks of one workgroup
// ---------------------------------------------------------------------------
template <int D, int DT>
__global__ __launch_bounds__(kAT, D == 64 ? kFwdOcc64 : 2) void attn_fwd_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t st[2][2 * 64 * D];   // stage: K tile, V tile
  __shared__ float xstat[2][2][2][64];   // [part][own][max, sum][lane]
  __shared__ int rowtab[4 * kRMax];
  const int nqb = a.S / 64;
  const int h0 = blockIdx.x * a.vheads, b = blockIdx.y;   // first head of the group, batch entry
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int own = wave % 2, part = wave / 2;   // own query half, key half of every block
  const int ql = 32 * own + lane % 32, h2 = lane / 32;
  // element offset of head hh's tensors, and of its per-row statistics
  auto base_of = [&](int hh) { return (long long)b * a.sb + (long long)hh * a.sh; };
  auto stat_of = [&](int hh) { return ((long long)b * a.Hh + hh) * a.S; };
  const uint32_t st_addr = lds_addr(&st[0][0]);

  RowSet rows;
  rows.init(rowtab, a.row_ptr, a.col_idx, a.nnz_cap, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h0) * nqb, nqb,
            a.vheads, h0, a.head_active, blockIdx.z, gridDim.z, a.rows_per_wg, true);
  // rows without a listed block (or of an inactive head): O = 0, LSE = -inf, nothing to read
  if (part == 0) {
    for (int j = 0; j < kRMax; ++j)
      if (rows.blk(j) >= 0 && rows.n(j) == 0) {
        f32x16 z[D / 32];
        zero(z);
        const int hh = rows.head(j);
        store_acc<D, DT>(z, 0.f, a.Out + base_of(hh) + (long long)(rows.blk(j) * 64 + ql) * a.ss);
        if (h2 == 0) a.LSE[stat_of(hh) + rows.blk(j) * 64 + ql] = -INFINITY;
      }
  }

  TileDma<D> dma;
  dma.init(a.ss);
  LaneOff<D> lo;
  lo.init(part);
  const float sc = a.scale * kLog2e;
  // state of the row being computed (this wavefront's part of it)
  int qb = 0;
  long long qoff = 0, soff = 0;      // this lane's row of Q / O, and of the statistics
  uint4 qf[D / 16];
  f32x16 o_acc[D / 32];
  float m = -INFINITY, lsum = 0.f;   // running maximum (scaled log2 units) and sum

  auto row_begin = [&](int k) {
    qb = rows.blk(k);
    const int hh = rows.head(k);
    qoff = base_of(hh) + (long long)(qb * 64 + ql) * a.ss;
    soff = stat_of(hh) + qb * 64 + ql;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      qf[s] = *reinterpret_cast<const uint4*>(a.Q + qoff + 16 * s + 8 * h2);
    zero(o_acc);
    m = -INFINITY;
    lsum = 0.f;
  };
  auto issue = [&](int stage, int k, int col) {
    const long long t0 = base_of(rows.head(k)) + (long long)col * 64 * a.ss;
    const uint32_t dst = st_addr + stage * (4 * 64 * D);
    dma.issue(dst, a.K + t0);
    dma.issue(dst + 2 * 64 * D, a.V + t0);
  };
  // diag: the diagonal block of a causal mask, where keys after the query are excluded.  Only
  // the scores are touched inside that branch, so the accumulators have one definition on
  // every path and stay in place.
  auto comp = [&](int stage, int col) {
    const uint32_t stg = st_addr + stage * (4 * 64 * D);
    f32x16 s_acc;
    mma_rows<D, DT>(stg, lo, qf, s_acc);       // S^T[key][q]
    // the V^T operands do not depend on the scores; reading them now hides their LDS latency
    // behind the softmax arithmetic
    TrOps<D> vt;
    load_tr<D>(stg + 2 * 64 * D, lo, vt);
    __builtin_amdgcn_sched_barrier(0);
    if (a.causal && col >= qb) mask_diag(s_acc, own, part, col > qb);
    float mloc = s_acc[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mloc = fmaxf(mloc, s_acc[v]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    // The reference point m of the running sums only has to bound the scores from above up to
    // a factor that fp32 holds comfortably: it follows the running maximum only when that has
    // moved by more than kSlack (then exp2(score - m) <= 2^kSlack), so most blocks need no
    // rescaling of the accumulators.  Sums, output and LSE do not depend on the choice.
    const float cand = mloc * sc;
    const float m_new = cand > m + kSlack ? cand : m;
    // a query none of whose keys so far is allowed keeps m = -inf; subtracting 0 instead keeps
    // the exponentials below at exp2(-inf) = 0 rather than exp2(-inf + inf)
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_use);
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float p = __builtin_amdgcn_exp2f(fmaf(s_acc[v], sc, -m_use));
      s_acc[v] = p;
      psum += p;
    }
    psum += __shfl_xor(psum, 32);
    lsum = lsum * alpha + psum;
    // (where m was -inf the accumulators are still zero: nothing to rescale.  Whole-vector
    // products under a wave-uniform branch: a lane-wise branch around element updates can send
    // the accumulators to scratch.)
    const bool rescale = __any(alpha != 1.f && m != -INFINITY);
    m = m_new;
    if (rescale) {
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct) o_acc[ct] *= alpha;
    }
    mma_tr<D, DT>(vt, s_acc, o_acc);          // O^T += V^T P^T
  };
  // combine the two key halves: (m, l, O) = (m0, l0, O0) (+) (m1, l1, O1)
  auto row_end = [&](int, int stage) {
    float* area = reinterpret_cast<float*>(st[stage]);
    lds_barrier();                       // every wavefront is done with the tiles of this stage
    if (part == 0)
      put_half<D, 0>(area, own, o_acc);
    else
      put_half<D, 1>(area, own, o_acc);
    xstat[part][own][0][lane] = m;
    xstat[part][own][1][lane] = lsum;
    lds_barrier();
    const float m1 = xstat[1 - part][own][0][lane], l1 = xstat[1 - part][own][1][lane];
    const float mt = fmaxf(m, m1);
    const float mu = mt == -INFINITY ? 0.f : mt;
    const float a0 = __builtin_amdgcn_exp2f(m - mu), a1 = __builtin_amdgcn_exp2f(m1 - mu);
    const float l = lsum * a0 + l1 * a1;
    const bool any = l > 0.f;
    const float inv = any ? 1.f / l : 0.f;
    if (part == 0) {
      merge_half<D, 0>(area, own, a0 * inv, a1 * inv, o_acc);
      store_acc<D, DT, 0, D / 64>(o_acc, 1.f, a.Out + qoff);
      if (h2 == 0)
        a.LSE[soff] = any ? (mt + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
    } else {
      merge_half<D, 1>(area, own, a0 * inv, a1 * inv, o_acc);
      store_acc<D, DT, D / 64, D / 64>(o_acc, 1.f, a.Out + qoff);
    }
  };
  walk_rows<false>(rows, row_begin, [](int) {}, issue, comp, row_end);
}

// ---------------------------------------------------------------------------
// backward, query side: Delta and dQ for the query blocks of one workgroup
// ---------------------------------------------------------------------------
template <int D, int DT>
__global__ __launch_bounds__(kAT, D == 64 ? kDqOcc64 : 2) void attn_bwd_dq_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t st[2][2 * 64 * D];   // stage: K tile, V tile
  // Q and dO tiles of a row, brought in one row ahead (head size 64 only: with 128 the area would
  // halve the number of resident workgroups)
  constexpr bool kOwnPf = D == 64;
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t ownt[kOwnPf ? 2 : 1][kOwnPf ? 64 * D : 8];
  __shared__ int rowtab[4 * kRMax];
  const int nqb = a.S / 64;
  const int h0 = blockIdx.x * a.vheads, b = blockIdx.y;   // first head of the group, batch entry
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int own = wave % 2, part = wave / 2;   // own query half, key half of every block
  const int ql = 32 * own + lane % 32, h2 = lane / 32;
  auto base_of = [&](int hh) { return (long long)b * a.sb + (long long)hh * a.sh; };
  auto stat_of = [&](int hh) { return ((long long)b * a.Hh + hh) * a.S; };
  const uint32_t st_addr = lds_addr(&st[0][0]), own_addr = lds_addr(&ownt[0][0]);
  const uint32_t own_off = tile_off<D>(ql, 8 * h2);   // this lane's fragments inside an own tile

  RowSet rows;
  rows.init(rowtab, a.row_ptr, a.col_idx, a.nnz_cap, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h0) * nqb, nqb,
            a.vheads, h0, a.head_active, blockIdx.z, gridDim.z, a.rows_per_wg, true);
  // rows without a listed block (or of an inactive head): O = 0, hence Delta = 0 and dQ = 0
  if (part == 0) {
    for (int j = 0; j < kRMax; ++j)
      if (rows.blk(j) >= 0 && rows.n(j) == 0) {
        f32x16 z[D / 32];
        zero(z);
        const int hh = rows.head(j);
        store_acc<D, DT>(z, 0.f, a.dQ + base_of(hh) + (long long)(rows.blk(j) * 64 + ql) * a.ss);
        if (h2 == 0) {
          a.Delta[stat_of(hh) + rows.blk(j) * 64 + ql] = 0.f;
          a.NegLse2[stat_of(hh) + rows.blk(j) * 64 + ql] = INFINITY;
        }
      }
  }

  TileDma<D> dma;
  dma.init(a.ss);
  LaneOff<D> lo;
  lo.init(part);
  const float sc = a.scale * kLog2e;
  int qb = 0;
  long long qoff = 0, soff = 0;      // this lane's row of Q / O / dO / dQ, and of the statistics
  uint4 qf[D / 16], dof[D / 16];
  float delta = 0.f, lse2 = 0.f;
  f32x16 dq_acc[D / 32];

  // the row's Q and dO tiles have been brought into LDS (prefetch below) or are read from
  // global memory; O is only needed for Delta and always comes straight from global memory
  // (computing Delta for all rows of the workgroup up front was measured slower)
  auto row_begin = [&](int k) {
    qb = rows.blk(k);
    const int hh = rows.head(k);
    qoff = base_of(hh) + (long long)(qb * 64 + ql) * a.ss;
    soff = stat_of(hh) + qb * 64 + ql;
    uint4 ofr[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      ofr[s] = *reinterpret_cast<const uint4*>(a.O + qoff + 16 * s + 8 * h2);
    // a row whose listed blocks hold no allowed key has LSE = -inf: +inf here makes every
    // probability exp2(score - inf) = 0, also for excluded scores (-inf), which -(-inf) would not
    const float lse_in = a.LSEin[soff];
    lse2 = lse_in == -INFINITY ? INFINITY : lse_in * kLog2e;
    float sum = 0.f;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      if (kOwnPf) {
        qf[s] = lds_read16((own_addr | own_off) ^ tile_off<D>(0, 16 * s));
        dof[s] = lds_read16((own_addr + 2 * 64 * D) | (own_off ^ tile_off<D>(0, 16 * s)));
      } else {
        qf[s] = *reinterpret_cast<const uint4*>(a.Q + qoff + 16 * s + 8 * h2);
        dof[s] = *reinterpret_cast<const uint4*>(a.dO + qoff + 16 * s + 8 * h2);
      }
    }
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const uint4 of = ofr[s];
      const uint32_t x[4] = {dof[s].x, dof[s].y, dof[s].z, dof[s].w};
      const uint32_t y[4] = {of.x, of.y, of.z, of.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        sum += to_f32<DT>(x[e] & 0xFFFFu) * to_f32<DT>(y[e] & 0xFFFFu) + to_f32<DT>(x[e] >> 16) * to_f32<DT>(y[e] >> 16);
    }
    delta = sum + __shfl_xor(sum, 32);
    if (part == 0 && h2 == 0) {        // for the key-side kernel: Delta and -LSE in log2 units
      a.Delta[soff] = delta;
      a.NegLse2[soff] = -lse2;
    }
    zero(dq_acc);
  };
  auto prefetch = [&](int k) {
    const long long t0 = base_of(rows.head(k)) + (long long)rows.blk(k) * 64 * a.ss;
    dma.issue(own_addr, a.Q + t0);
    dma.issue(own_addr + 2 * 64 * D, a.dO + t0);
  };
  auto issue = [&](int stage, int k, int col) {
    const long long t0 = base_of(rows.head(k)) + (long long)col * 64 * a.ss;
    const uint32_t dst = st_addr + stage * (4 * 64 * D);
    dma.issue(dst, a.K + t0);
    dma.issue(dst + 2 * 64 * D, a.V + t0);
  };
  auto comp = [&](int stage, int col) {
    const uint32_t stg = st_addr + stage * (4 * 64 * D);
    f32x16 s_acc, dp_acc;
    mma_rows<D, DT>(stg, lo, qf, s_acc);                    // S^T[key][q]
    mma_rows<D, DT>(stg + 2 * 64 * D, lo, dof, dp_acc);     // dP^T[key][q]
    if (a.causal && col >= qb) mask_diag(s_acc, own, part, col > qb);   // excluded keys: P = exp2(-inf) = 0
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float p = __builtin_amdgcn_exp2f(fmaf(s_acc[v], sc, -lse2));
      s_acc[v] = p * (dp_acc[v] - delta);   // dS^T
    }
    // registers are what limits the number of resident wavefronts here, so the K^T operands
    // are read only now; the other wavefronts of the SIMD cover the latency
    __builtin_amdgcn_sched_barrier(0);
    TrOps<D> kt;
    load_tr<D>(stg, lo, kt);
    mma_tr<D, DT>(kt, s_acc, dq_acc);           // dQ^T += K^T dS^T
  };
  auto row_end = [&](int, int stage) {     // dQ = sum over the two key halves
    float* area = reinterpret_cast<float*>(st[stage]);
    lds_barrier();
    if (part == 0)
      put_half<D, 0>(area, own, dq_acc);
    else
      put_half<D, 1>(area, own, dq_acc);
    lds_barrier();
    if (part == 0) {
      merge_half<D, 0>(area, own, 1.f, 1.f, dq_acc);
      store_acc<D, DT, 0, D / 64>(dq_acc, a.scale, a.dQ + qoff);
    } else {
      merge_half<D, 1>(area, own, 1.f, 1.f, dq_acc);
      store_acc<D, DT, D / 64, D / 64>(dq_acc, a.scale, a.dQ + qoff);
    }
  };
  walk_rows<kOwnPf>(rows, row_begin, prefetch, issue, comp, row_end);
}

// ---------------------------------------------------------------------------
// backward, key side: dK and dV for the key blocks of one workgroup
// ---------------------------------------------------------------------------
// WHICH = 0: dK and dV in one walk (head size 64).  At head size 128 the two gradients together need
// 406 registers, i.e. one workgroup per CU and nothing to hide a wavefront's latency behind, so the
// launcher runs the kernel twice there: WHICH = 1 computes dV only (S, P, dV += dO^T P), WHICH = 2
// dK only (S, dP, dS, dK += Q^T dS), each with two workgroups per CU; the tiles of a block are
// transferred and its scores computed twice, which costs less than the idle SIMDs did.
template <int D, int DT, int WHICH>
__global__ __launch_bounds__(kAT, D == 64 ? kDkvOcc64 : (WHICH == 0 ? 1 : 2)) void attn_bwd_dkv_bf16(
    const AttnArgs a) {
  constexpr bool kDV = WHICH != 2, kDK = WHICH != 1;
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t st[2][2 * 64 * D];   // stage: Q tile, dO tile
  // K and V tiles of a row, brought in one row ahead (head size 64 only: with 128 the kernel is
  // at its register limit and the extra addressing spills)
  constexpr bool kOwnPf = D == 64;
  __shared__ __attribute__((aligned(2 * 64 * D))) uint16_t ownt[kOwnPf ? 2 : 1][kOwnPf ? 64 * D : 8];
  __shared__ __attribute__((aligned(256))) float sstat[2][128];   // stage: -LSE*log2e [64], Delta [64]
  __shared__ int rowtab[4 * kRMax];
  const int nkb = a.S / 64;
  const int h0 = blockIdx.x * a.vheads, b = blockIdx.y;   // first head of the group, batch entry
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int own = wave % 2, part = wave / 2;   // own key half, query half of every block
  const int kl = 32 * own + lane % 32, h2 = lane / 32;
  auto base_of = [&](int hh) { return (long long)b * a.sb + (long long)hh * a.sh; };
  auto stat_of = [&](int hh) { return ((long long)b * a.Hh + hh) * a.S; };
  const uint32_t st_addr = lds_addr(&st[0][0]), sstat_addr = lds_addr(&sstat[0][0]);
  const uint32_t own_addr = lds_addr(&ownt[0][0]);
  const uint32_t own_off = tile_off<D>(kl, 8 * h2);   // this lane's fragments inside an own tile

  RowSet rows;
  rows.init(rowtab, a.crow_ptr, a.ccol_idx, a.cnnz_cap, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h0) * nkb, nkb,
            a.vheads, h0, a.head_active, blockIdx.z, gridDim.z, a.rows_per_wg, false);
  // key blocks used by no query block: zero gradients, nothing to read
  if (part == 0) {
    for (int j = 0; j < kRMax; ++j)
      if (rows.blk(j) >= 0 && rows.n(j) == 0) {
        f32x16 z[D / 32];
        zero(z);
        const long long koff = base_of(rows.head(j)) + (long long)(rows.blk(j) * 64 + kl) * a.ss;
        if (kDV) store_acc<D, DT>(z, 0.f, a.dV + koff);
        if (kDK) store_acc<D, DT>(z, 0.f, a.dK + koff);
      }
  }

  TileDma<D> dma;
  dma.init(a.ss);
  LaneOff<D> lo;
  lo.init(part);
  const float sc = a.scale * kLog2e;
  const float* stat_src = wave == 0 ? a.NegLse2 : a.Delta;  // wave 0: -LSE*log2(e), wave 1: Delta
  int kb = 0;
  long long koff = 0;
  uint4 kf[D / 16], vf[D / 16];
  f32x16 dk_acc[D / 32], dv_acc[D / 32];

  auto row_begin = [&](int k) {       // the row's K and V tiles are in LDS (prefetch below) or read directly
    kb = rows.blk(k);
    koff = base_of(rows.head(k)) + (long long)(kb * 64 + kl) * a.ss;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      if (kOwnPf) {
        kf[s] = lds_read16((own_addr | own_off) ^ tile_off<D>(0, 16 * s));
        vf[s] = lds_read16((own_addr + 2 * 64 * D) | (own_off ^ tile_off<D>(0, 16 * s)));
      } else {
        kf[s] = *reinterpret_cast<const uint4*>(a.K + koff + 16 * s + 8 * h2);
        if (kDK) vf[s] = *reinterpret_cast<const uint4*>(a.V + koff + 16 * s + 8 * h2);
      }
    }
    if (kDK) zero(dk_acc);
    if (kDV) zero(dv_acc);
  };
  auto prefetch = [&](int k) {
    const long long t0 = base_of(rows.head(k)) + (long long)rows.blk(k) * 64 * a.ss;
    dma.issue(own_addr, a.K + t0);
    dma.issue(own_addr + 2 * 64 * D, a.V + t0);
  };
  auto issue = [&](int stage, int k, int qb) {
    const int hh = rows.head(k);
    const long long t0 = base_of(hh) + (long long)qb * 64 * a.ss;
    const uint32_t dst = st_addr + stage * (4 * 64 * D);
    dma.issue(dst, a.Q + t0);
    dma.issue(dst + 2 * 64 * D, a.dO + t0);
    if (wave < 2) dma4(stat_src + stat_of(hh) + qb * 64 + lane, sstat_addr + stage * 512 + wave * 256);
  };
  auto comp = [&](int stage, int col) {
    const uint32_t stg = st_addr + stage * (4 * 64 * D);
    const float* stt = sstat[stage];
    f32x16 s_acc, dp_acc;
    mma_rows<D, DT>(stg, lo, kf, s_acc);                   // S[q][key]
    if (kDK) mma_rows<D, DT>(stg + 2 * 64 * D, lo, vf, dp_acc);     // dP[q][key]
    // diagonal block: here the rows of the score tile are queries and the lane is the key
    if (a.causal && col <= kb) mask_diag_t(s_acc, own, part, col < kb);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int q0 = 8 * g + 4 * h2;                 // four consecutive queries of this half
      const float4 nl = *reinterpret_cast<const float4*>(stt + 32 * part + q0);
      const float nls[4] = {nl.x, nl.y, nl.z, nl.w};
      float dls[4] = {0.f, 0.f, 0.f, 0.f};
      if (kDK) {
        const float4 dl = *reinterpret_cast<const float4*>(stt + 64 + 32 * part + q0);
        dls[0] = dl.x; dls[1] = dl.y; dls[2] = dl.z; dls[3] = dl.w;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = 4 * g + e;
        const float p = __builtin_amdgcn_exp2f(fmaf(s_acc[v], sc, nls[e]));
        s_acc[v] = p;                                         // P
        if (kDK) dp_acc[v] = p * (dp_acc[v] - dls[e]);        // dS
      }
    }
    // registers are what limits the number of resident wavefronts here, so the transposed
    // operands are read only when they are needed
    __builtin_amdgcn_sched_barrier(0);
    if (kDV) {
      TrOps<D> dot;
      load_tr<D>(stg + 2 * 64 * D, lo, dot);
      mma_tr<D, DT>(dot, s_acc, dv_acc);            // dV^T += dO^T P
    }
    if (kDK) {
      TrOps<D> qt;
      load_tr<D>(stg, lo, qt);
      __builtin_amdgcn_sched_barrier(0);
      mma_tr<D, DT>(qt, dp_acc, dk_acc);            // dK^T += Q^T dS
    }
  };
  // dV and dK = sums over the two query halves, exchanged one after the other through the
  // same LDS area
  auto row_end = [&](int, int stage) {
    float* area = reinterpret_cast<float*>(st[stage]);
    if (D == 128) {      // the one-sided exchange (the symmetric one costs registers this size lacks)
      if (kDV) {
        lds_barrier();
        if (part == 1) put_all<D>(area, own, dv_acc);
        lds_barrier();
        if (part == 0) {
          merge_all<D>(area, own, dv_acc);
          store_acc<D, DT>(dv_acc, 1.f, a.dV + koff);
        }
      }
      if (kDK) {
        lds_barrier();
        if (part == 1) put_all<D>(area, own, dk_acc);
        lds_barrier();
        if (part == 0) {
          merge_all<D>(area, own, dk_acc);
          store_acc<D, DT>(dk_acc, a.scale, a.dK + koff);
        }
      }
      return;
    }
    lds_barrier();
    if (part == 0)
      put_half<D, 0>(area, own, dv_acc);
    else
      put_half<D, 1>(area, own, dv_acc);
    lds_barrier();
    if (part == 0)
      merge_half<D, 0>(area, own, 1.f, 1.f, dv_acc);
    else
      merge_half<D, 1>(area, own, 1.f, 1.f, dv_acc);
    lds_barrier();
    if (part == 0)
      put_half<D, 0>(area, own, dk_acc);
    else
      put_half<D, 1>(area, own, dk_acc);
    lds_barrier();
    if (part == 0) {
      merge_half<D, 0>(area, own, 1.f, 1.f, dk_acc);
      store_acc<D, DT, 0, D / 64>(dv_acc, 1.f, a.dV + koff);
      store_acc<D, DT, 0, D / 64>(dk_acc, a.scale, a.dK + koff);
    } else {
      merge_half<D, 1>(area, own, 1.f, 1.f, dk_acc);
      store_acc<D, DT, D / 64, D / 64>(dv_acc, 1.f, a.dV + koff);
      store_acc<D, DT, D / 64, D / 64>(dk_acc, a.scale, a.dK + koff);
    }
  };
  walk_rows<kOwnPf>(rows, row_begin, prefetch, issue, comp, row_end);
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

template <int D, int DT>
static hipError_t launch_fwd(AttnArgs a, int B, hipStream_t st) {
  ProfScope ps(kKAttnFwd, st);
  const int nblk = a.S / 64;
  a.vheads = heads_per_group(nblk, a.Hh);
  a.rows_per_wg = rows_per_wg(nblk, a.Hh, B, kCUs * (D == 64 ? kFwdOcc64 : 2));
  const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
  hipLaunchKernelGGL((attn_fwd_bf16<D, DT>), dim3(a.Hh / a.vheads, B, G * a.vheads), dim3(kAT), 0, st, a);
  return hipGetLastError();
}

template <int D, int DT>
static hipError_t launch_bwd(AttnArgs a, int B, hipStream_t st) {
  const int nblk = a.S / 64;
  a.vheads = heads_per_group(nblk, a.Hh);
  {
    ProfScope ps(kKAttnDq, st);
    a.rows_per_wg = rows_per_wg(nblk, a.Hh, B, kCUs * (D == 64 ? kDqOcc64 : 2));
    const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
    hipLaunchKernelGGL((attn_bwd_dq_bf16<D, DT>), dim3(a.Hh / a.vheads, B, G * a.vheads), dim3(kAT), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKAttnDkv, st);
    a.rows_per_wg = rows_per_wg(nblk, a.Hh, B, kCUs * (D == 64 ? kDkvOcc64 : 2));
    const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
    const dim3 grid(a.Hh / a.vheads, B, G * a.vheads);
    if constexpr (D == 64) {
      hipLaunchKernelGGL((attn_bwd_dkv_bf16<D, DT, 0>), grid, dim3(kAT), 0, st, a);
    } else {      // head size 128: dV and dK in a launch each (see the kernel)
      hipLaunchKernelGGL((attn_bwd_dkv_bf16<D, DT, 1>), grid, dim3(kAT), 0, st, a);
      hipLaunchKernelGGL((attn_bwd_dkv_bf16<D, DT, 2>), grid, dim3(kAT), 0, st, a);
    }
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
