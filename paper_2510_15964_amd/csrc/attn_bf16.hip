// Block-sparse attention for gfx950 (Sec. VI-A).  The two block-sparse products
// of the paper -- SDD (scores on listed blocks) and DSD (probabilities times
// V) -- are fused with the softmax in flash style, so the score blocks live
// only in registers; the unit of work is the listed block, which is what keeps
// heads with different patterns balanced (Sec. VI-A, online combination).
//
// Layout of one workgroup (128 threads = 2 wavefronts): a 64-row query block
// (forward, dQ) or a 64-row key block (dK/dV) at a time; each wavefront owns 32
// of the rows and walks the block list of its row of the mask.  All products
// run on the 32x32x16 bf16 MFMA with fp32 accumulators.
//
// At the block densities of the paper a row of the mask lists only a few
// blocks, so a workgroup that handled one row would spend most of its life in
// the chain of dependent loads that starts it (row pointer -> list -> tiles).
// A workgroup therefore owns up to four rows of one (batch, head) and walks
// their lists as ONE stream of blocks: the metadata of all its rows is read up
// front, and the tile transfer of the next block -- of the same row or of the
// next one -- is always in flight while the current block is computed.  The
// rows are picked k, 2G-1-k, 2G+k, 4G-1-k (G = groups per head), which gives
// every workgroup the same number of blocks under a causal mask.
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

#define LX_AS1 __attribute__((address_space(1)))
#define LX_AS3 __attribute__((address_space(3)))

constexpr int kAT = 128;                 // threads per workgroup
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef short short4v __attribute__((ext_vector_type(4)));
struct TrueTag { static constexpr bool value = true; };
struct FalseTag { static constexpr bool value = false; };

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
  static constexpr int kPerWave = 64 / kRowsPer / 2;
  long long off[kPerWave];
  __device__ __forceinline__ void init(long long ld) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int g = wave + 2 * u;
      const int row = kRowsPer * g + lane / kSlots;
      const int slot = (lane % kSlots) ^ tswz<D>(row);
      off[u] = (long long)row * ld + slot * 8;
    }
  }
  // tile_addr: LDS byte address of the destination tile
  __device__ __forceinline__ void issue(uint32_t tile_addr, const uint16_t* g0) const {
    const int wave = threadIdx.x / kWave;
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) dma16(g0 + off[u], tile_addr + (wave + 2 * u) * 1024);
  }
};

// acc[half] += R[rows 32*half + lane%32][:] . F^T   where R is a row-major tile in LDS and F the
// per-lane register fragments (column index = lane%32).  Result register v of a lane is element
// (row 32*half + 8*(v/4) + 4*(lane/32) + v%4, column lane%32).
template <int D>
__device__ __forceinline__ void mma_rows(const uint16_t* tile, const uint4 (&frag)[D / 16],
                                         f32x16 (&acc)[2]) {
  const int lane = threadIdx.x % kWave, r = lane % 32, h2 = lane / 32;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // The operand reads are issued ahead of the MFMAs that use them (all 2 * D/16 of them for
  // D = 64, one half at a time for D = 128, where registers are short), so their LDS latency is
  // paid once instead of once per k16 slice.
  constexpr int kGroup = D == 64 ? 2 : 1;   // halves per group of reads
#pragma unroll
  for (int h0 = 0; h0 < 2; h0 += kGroup) {
    uint4 a[kGroup][D / 16];
#pragma unroll
    for (int hh = 0; hh < kGroup; ++hh) {
      const int row = 32 * (h0 + hh) + r;
#pragma unroll
      for (int s = 0; s < D / 16; ++s)
        a[hh][s] =
            *reinterpret_cast<const uint4*>(tile + row * D + (((2 * s + h2) ^ tswz<D>(row)) << 3));
    }
    __builtin_amdgcn_sched_barrier(0);   // keep the reads above: the scheduler would sink them
#pragma unroll
    for (int hh = 0; hh < kGroup; ++hh)
#pragma unroll
      for (int s = 0; s < D / 16; ++s)
        // the first product starts from a literal zero (no register clearing)
        acc[h0 + hh] = mfma32(a[hh][s], frag[s], s == 0 ? zero16 : acc[h0 + hh]);
  }
}

// One row of a block list, kept in a register (entry it of the row sits in lane it % 64), so the
// walk over the list issues no memory loads: a load inside the pipelined loop would have to wait
// on vmcnt and with it on the tile DMA that is deliberately left in flight.
struct ListRow {
  const int* p;
  int n, chunk, cur;
  __device__ __forceinline__ void init(const int* list, int n_) {
    p = list;
    n = n_;
    chunk = -1;
    cur = 0;
  }
  __device__ __forceinline__ int get(int it) {        // it is wave-uniform
    if ((it >> 6) != chunk) {                         // only for rows longer than 64 entries
      chunk = it >> 6;
      const int i = chunk * 64 + (int)(threadIdx.x % kWave);
      cur = i < n ? p[i] : 0;
    }
    return __builtin_amdgcn_readlane(cur, it & 63);
  }
};

// Operands of out[ct] += T^T . P for the k-slices s2 = S0 .. S0+NS2-1 (16 rows of T each), read
// from the row-major [64 x D] tile T in LDS with the transposing read.
template <int D, int NS2>
struct TrOps {
  uint4 a[NS2][D / 32];
};
template <int D, int NS2>
__device__ __forceinline__ void load_tr(const uint16_t* tile, int s2_0, TrOps<D, NS2>& t) {
  const int lane = threadIdx.x % kWave, h2 = lane / 32;
  const int j = lane % 16, e = j / 4, q = j % 4;
  const int cbase = 16 * ((lane / 16) % 2) + 4 * q;      // + 32*ct
#pragma unroll
  for (int i = 0; i < NS2; ++i) {
    const int r_lo = 16 * (s2_0 + i) + 4 * h2 + e, r_hi = r_lo + 8;
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) {
      const int col = 32 * ct + cbase;
      const uint16_t* p_lo = tile + r_lo * D + (((col >> 3) ^ tswz<D>(r_lo)) << 3) + (col & 7);
      const uint16_t* p_hi = tile + r_hi * D + (((col >> 3) ^ tswz<D>(r_hi)) << 3) + (col & 7);
      const uint2 lo = __builtin_bit_cast(
          uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LX_AS3 short4v*)p_lo));
      const uint2 hi = __builtin_bit_cast(
          uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LX_AS3 short4v*)p_hi));
      t.a[i][ct] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
  }
}
// p[half][v]: accumulator-layout values of the [64 x 32] factor P (rounded to bf16 here).
template <int D, int NS2>
__device__ __forceinline__ void mma_tr(const TrOps<D, NS2>& t, int s2_0, const f32x16 (&p)[2],
                                       f32x16 (&out)[D / 32]) {
#pragma unroll
  for (int i = 0; i < NS2; ++i) {
    const int s2 = s2_0 + i, half = s2 / 2, g0 = 2 * (s2 % 2);
    uint4 b;
    b.x = pack2bf(p[half][4 * g0 + 0], p[half][4 * g0 + 1]);
    b.y = pack2bf(p[half][4 * g0 + 2], p[half][4 * g0 + 3]);
    b.z = pack2bf(p[half][4 * g0 + 4], p[half][4 * g0 + 5]);
    b.w = pack2bf(p[half][4 * g0 + 6], p[half][4 * g0 + 7]);
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) out[ct] = mfma32(t.a[i][ct], b, out[ct]);
  }
}
// out[ct] += T^T . P with the reads of two k-slices grouped ahead of their MFMAs.
template <int D>
__device__ __forceinline__ void mma_transposed(const uint16_t* tile, const f32x16 (&p)[2],
                                               f32x16 (&out)[D / 32]) {
#pragma unroll
  for (int s2 = 0; s2 < 4; s2 += 2) {
    TrOps<D, 2> t;
    load_tr<D, 2>(tile, s2, t);
    __builtin_amdgcn_sched_barrier(0);
    mma_tr<D, 2>(t, s2, p, out);
  }
}

template <int N>
__device__ __forceinline__ void zero(f32x16 (&a)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) a[i][v] = 0.f;
}

// accumulator layout [c-tile][v] (c = 32ct + 8(v/4) + 4(lane/32) + v%4, row = lane%32) -> global
template <int D>
__device__ __forceinline__ void store_acc(const f32x16 (&acc)[D / 32], float mul,
                                          uint16_t* __restrict__ dst_row) {
  const int h2 = (threadIdx.x % kWave) / 32;
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 o;
      o.x = pack2bf(acc[ct][4 * g] * mul, acc[ct][4 * g + 1] * mul);
      o.y = pack2bf(acc[ct][4 * g + 2] * mul, acc[ct][4 * g + 3] * mul);
      *reinterpret_cast<uint2*>(dst_row + 32 * ct + 8 * g + 4 * h2) = o;
    }
}

// ---------------------------------------------------------------------------
// rows of a workgroup and the walk over their blocks
// ---------------------------------------------------------------------------
constexpr int kRMax = 4;   // rows of the mask per workgroup, at most

// Wave-uniform selection from a small array by a run-time index (stays in scalar registers).
__device__ __forceinline__ int pick(const int (&v)[kRMax], int k) {
  int r = v[0];
#pragma unroll
  for (int j = 1; j < kRMax; ++j) r = k == j ? v[j] : r;
  return r;
}

// The rows (query blocks, or key blocks for dK/dV) of one (batch, head) that workgroup g of G
// owns: slot j holds block j*G + g for even j and (j+1)*G - 1 - g for odd j.  All metadata is
// fetched here, before the walk, so the walk itself issues no dependent metadata loads.
struct RowSet {
  int blk[kRMax];   // block index of the slot, -1 = slot not used
  int n[kRMax];     // listed blocks of that row (0 for an inactive head)
  ListRow list[kRMax];
  __device__ __forceinline__ void init(const int* __restrict__ row_ptr,
                                       const int* __restrict__ col_idx, int head_row0, int nblk,
                                       int g, int G, int R, bool head_on) {
    int rs[kRMax];
#pragma unroll
    for (int j = 0; j < kRMax; ++j) {
      const int bj = (j & 1) ? (j + 1) * G - 1 - g : j * G + g;
      const bool used = j < R && bj < nblk;
      blk[j] = used ? bj : -1;
      rs[j] = 0;
      n[j] = 0;
      if (used) {
        rs[j] = row_ptr[head_row0 + bj];
        n[j] = head_on ? row_ptr[head_row0 + bj + 1] - rs[j] : 0;
      }
      // wave-uniform by construction; say so, to keep the walk's control flow scalar
      rs[j] = __builtin_amdgcn_readfirstlane(rs[j]);
      n[j] = __builtin_amdgcn_readfirstlane(n[j]);
    }
#pragma unroll
    for (int j = 0; j < kRMax; ++j) {
      list[j].init(col_idx + rs[j], n[j]);
      if (n[j] > 0) list[j].get(0);   // fetch the first 64 entries now
    }
  }
  // listed block `it` of slot k (both wave-uniform)
  __device__ __forceinline__ int col(int k, int it) {
    int c = 0;
#pragma unroll
    for (int j = 0; j < kRMax; ++j)
      if (k == j) c = list[j].get(it);
    return c;
  }
  // first slot >= k with a non-empty list, kRMax if none
  __device__ __forceinline__ int next_row(int k) const {
    int r = kRMax;
#pragma unroll
    for (int j = kRMax - 1; j >= 0; --j) r = (j >= k && n[j] > 0) ? j : r;
    return r;
  }
};

// Walk over all listed blocks of the row set as one double-buffered stream.  issue(stage, k, it)
// starts the transfer of block `it` of slot k into stage 0/1; comp(stage, k, it) consumes it;
// row_begin(k) / row_end(k) load and store the per-row state.  The transfer of the next block,
// which may belong to the next row, is issued before the current one is computed.  A wave first
// waits for its own transfers (vmcnt), the barrier then makes the whole stage visible and
// retires the reads of the stage about to be refilled.  All control flow is workgroup-uniform.
template <class RowBegin, class Issue, class Comp, class RowEnd>
__device__ __forceinline__ void walk_rows(RowSet& rows, RowBegin row_begin, Issue issue, Comp comp,
                                          RowEnd row_end) {
  int ki = __builtin_amdgcn_readfirstlane(rows.next_row(0)), iti = 0;
  if (ki >= kRMax) return;
  issue(0, ki, iti);
  int kc = ki, itc = 0, nc = pick(rows.n, kc);
  auto advance = [&]() {
    if (++iti == pick(rows.n, ki)) {
      ki = __builtin_amdgcn_readfirstlane(rows.next_row(ki + 1));
      iti = 0;
    }
  };
  advance();
  row_begin(kc);
  for (int t = 0;; ++t) {
    wait_vmcnt<0>();
    lds_barrier();
    const bool more = ki < kRMax;
    if (more) issue((t + 1) & 1, ki, iti);
    comp(t & 1, kc, itc);
    const bool last = itc + 1 == nc;
    if (last) row_end(kc);
    if (!more) break;
    if (last) {
      row_begin(ki);
      nc = pick(rows.n, ki);
    }
    kc = ki;
    itc = iti;
    advance();
  }
}

// ---------------------------------------------------------------------------
// forward: O, LSE for the query blocks of one workgroup
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT, D == 64 ? 2 : 1) void attn_fwd_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t st[2][2 * 64 * D];   // stage: K tile, V tile
  const int nqb = a.S / 64;
  const int h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int ql = 32 * wave + lane % 32, h2 = lane / 32;
  const long long base = (long long)b * a.sb + (long long)h * a.sh;
  const long long stat_base = ((long long)b * a.Hh + h) * a.S;
  const uint32_t st_addr = lds_addr(&st[0][0]);

  RowSet rows;
  rows.init(a.row_ptr, a.col_idx, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nqb, nqb, blockIdx.x,
            gridDim.x, a.rows_per_wg, !(a.head_active && !a.head_active[h]));
  // rows without a listed block (or of an inactive head): O = 0, LSE = -inf, nothing to read
#pragma unroll
  for (int j = 0; j < kRMax; ++j)
    if (rows.blk[j] >= 0 && rows.n[j] == 0) {
      f32x16 z[D / 32];
      zero(z);
      store_acc<D>(z, 0.f, a.Out + base + (long long)(rows.blk[j] * 64 + ql) * a.ss);
      if (h2 == 0) a.LSE[stat_base + rows.blk[j] * 64 + ql] = -INFINITY;
    }

  TileDma<D> dma;
  dma.init(a.ss);
  const float sc = a.scale * kLog2e;
  // state of the row being computed
  int qb = 0;
  long long qoff = 0;
  uint4 qf[D / 16];
  f32x16 o_acc[D / 32];
  float m = -INFINITY, lsum = 0.f;

  auto row_begin = [&](int k) {
    qb = pick(rows.blk, k);
    qoff = base + (long long)(qb * 64 + ql) * a.ss;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      qf[s] = *reinterpret_cast<const uint4*>(a.Q + qoff + 16 * s + 8 * h2);
    zero(o_acc);
    m = -INFINITY;
    lsum = 0.f;
  };
  auto issue = [&](int stage, int k, int it) {
    const long long t0 = base + (long long)rows.col(k, it) * 64 * a.ss;
    const uint32_t dst = st_addr + stage * (4 * 64 * D);
    dma.issue(dst, a.K + t0);
    dma.issue(dst + 2 * 64 * D, a.V + t0);
  };
  // DIAG: the diagonal block of a causal mask, where keys after the query are excluded.  Two
  // separate instantiations (instead of a branch in the middle) keep the 32 score registers in
  // place on both paths.
  auto comp_body = [&](const uint16_t* stg, auto diag_tag) {
    constexpr bool DIAG = decltype(diag_tag)::value;
    f32x16 s_acc[2];
    mma_rows<D>(stg, qf, s_acc);           // S^T[key][q]
    // D = 64: the V^T operands do not depend on the scores; reading them now hides their LDS
    // latency behind the softmax arithmetic
    TrOps<D, D == 64 ? 4 : 1> vt;
    if (D == 64) {
      load_tr<D, D == 64 ? 4 : 1>(stg + 64 * D, 0, vt);
      __builtin_amdgcn_sched_barrier(0);
    }
    float mloc = -INFINITY;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (DIAG) {
          const int kl = 32 * half + 8 * (v / 4) + 4 * h2 + v % 4;
          if (kl > ql) s_acc[half][v] = -INFINITY;
        }
        mloc = fmaxf(mloc, s_acc[half][v]);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m, mloc * sc);          // running max in scaled log2 units
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    float psum = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s_acc[half][v], sc, -m_new));
        s_acc[half][v] = p;
        psum += p;
      }
    psum += __shfl_xor(psum, 32);
    lsum = lsum * alpha + psum;
    m = m_new;
    if (__any(alpha != 1.f)) {            // the running maximum moved for some query
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[ct][v] *= alpha;
    }
    if (D == 64)                                     // O^T += V^T P^T
      mma_tr<D, D == 64 ? 4 : 1>(vt, 0, s_acc, o_acc);
    else
      mma_transposed<D>(stg + 64 * D, s_acc, o_acc);
  };
  auto comp = [&](int stage, int k, int it) {
    if (a.causal && rows.col(k, it) == qb)
      comp_body(st[stage], TrueTag{});
    else
      comp_body(st[stage], FalseTag{});
  };
  auto row_end = [&](int) {
    const bool any = lsum > 0.f;
    const float inv = any ? 1.f / lsum : 0.f;
    store_acc<D>(o_acc, inv, a.Out + qoff);
    if (h2 == 0)
      a.LSE[stat_base + qb * 64 + ql] = any ? (m + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
  };
  walk_rows(rows, row_begin, issue, comp, row_end);
}

// ---------------------------------------------------------------------------
// backward, query side: Delta and dQ for the query blocks of one workgroup
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT, D == 64 ? 2 : 1) void attn_bwd_dq_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t st[2][2 * 64 * D];   // stage: K tile, V tile
  const int nqb = a.S / 64;
  const int h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int ql = 32 * wave + lane % 32, h2 = lane / 32;
  const long long base = (long long)b * a.sb + (long long)h * a.sh;
  const long long stat_base = ((long long)b * a.Hh + h) * a.S;
  const uint32_t st_addr = lds_addr(&st[0][0]);

  RowSet rows;
  rows.init(a.row_ptr, a.col_idx, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nqb, nqb, blockIdx.x,
            gridDim.x, a.rows_per_wg, !(a.head_active && !a.head_active[h]));
  // rows without a listed block (or of an inactive head): O = 0, hence Delta = 0 and dQ = 0
#pragma unroll
  for (int j = 0; j < kRMax; ++j)
    if (rows.blk[j] >= 0 && rows.n[j] == 0) {
      f32x16 z[D / 32];
      zero(z);
      store_acc<D>(z, 0.f, a.dQ + base + (long long)(rows.blk[j] * 64 + ql) * a.ss);
      if (h2 == 0) {
        a.Delta[stat_base + rows.blk[j] * 64 + ql] = 0.f;
        a.NegLse2[stat_base + rows.blk[j] * 64 + ql] = INFINITY;
      }
    }

  TileDma<D> dma;
  dma.init(a.ss);
  const float sc = a.scale * kLog2e;
  int qb = 0;
  long long qoff = 0;
  uint4 qf[D / 16], dof[D / 16];
  float delta = 0.f, lse2 = 0.f;
  f32x16 dq_acc[D / 32];

  auto row_begin = [&](int k) {
    qb = pick(rows.blk, k);
    qoff = base + (long long)(qb * 64 + ql) * a.ss;
    float part = 0.f;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      qf[s] = *reinterpret_cast<const uint4*>(a.Q + qoff + 16 * s + 8 * h2);
      dof[s] = *reinterpret_cast<const uint4*>(a.dO + qoff + 16 * s + 8 * h2);
      const uint4 of = *reinterpret_cast<const uint4*>(a.O + qoff + 16 * s + 8 * h2);
      const uint32_t x[4] = {dof[s].x, dof[s].y, dof[s].z, dof[s].w};
      const uint32_t y[4] = {of.x, of.y, of.z, of.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        part += bf2f(x[e] & 0xFFFFu) * bf2f(y[e] & 0xFFFFu) + bf2f(x[e] >> 16) * bf2f(y[e] >> 16);
    }
    delta = part + __shfl_xor(part, 32);
    lse2 = a.LSEin[stat_base + qb * 64 + ql] * kLog2e;
    if (h2 == 0) {                     // for the key-side kernel: Delta and -LSE in log2 units
      a.Delta[stat_base + qb * 64 + ql] = delta;
      a.NegLse2[stat_base + qb * 64 + ql] = -lse2;
    }
    zero(dq_acc);
  };
  auto issue = [&](int stage, int k, int it) {
    const long long t0 = base + (long long)rows.col(k, it) * 64 * a.ss;
    const uint32_t dst = st_addr + stage * (4 * 64 * D);
    dma.issue(dst, a.K + t0);
    dma.issue(dst + 2 * 64 * D, a.V + t0);
  };
  auto comp_body = [&](const uint16_t* stg, auto diag_tag) {
    constexpr bool DIAG = decltype(diag_tag)::value;
    f32x16 s_acc[2], dp_acc[2];
    mma_rows<D>(stg, qf, s_acc);              // S^T[key][q]
    mma_rows<D>(stg + 64 * D, dof, dp_acc);   // dP^T[key][q]
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float p = __builtin_amdgcn_exp2f(fmaf(s_acc[half][v], sc, -lse2));
        if (DIAG) {
          const int kl = 32 * half + 8 * (v / 4) + 4 * h2 + v % 4;
          if (kl > ql) p = 0.f;
        }
        s_acc[half][v] = p * (dp_acc[half][v] - delta);   // dS^T
      }
    mma_transposed<D>(stg, s_acc, dq_acc);    // dQ^T += K^T dS^T
  };
  auto comp = [&](int stage, int k, int it) {
    if (a.causal && rows.col(k, it) == qb)
      comp_body(st[stage], TrueTag{});
    else
      comp_body(st[stage], FalseTag{});
  };
  auto row_end = [&](int) { store_acc<D>(dq_acc, a.scale, a.dQ + qoff); };
  walk_rows(rows, row_begin, issue, comp, row_end);
}

// ---------------------------------------------------------------------------
// backward, key side: dK and dV for the key blocks of one workgroup
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT, D == 64 ? 2 : 1) void attn_bwd_dkv_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t st[2][2 * 64 * D];   // stage: Q tile, dO tile
  __shared__ __attribute__((aligned(256))) float sstat[2][128];   // stage: -LSE*log2e [64], Delta [64]
  const int nkb = a.S / 64;
  const int h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int kl = 32 * wave + lane % 32, h2 = lane / 32;
  const long long base = (long long)b * a.sb + (long long)h * a.sh;
  const long long stat_base = ((long long)b * a.Hh + h) * a.S;
  const uint32_t st_addr = lds_addr(&st[0][0]), sstat_addr = lds_addr(&sstat[0][0]);

  RowSet rows;
  rows.init(a.crow_ptr, a.ccol_idx, ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nkb, nkb,
            blockIdx.x, gridDim.x, a.rows_per_wg, !(a.head_active && !a.head_active[h]));
  // key blocks used by no query block: zero gradients, nothing to read
#pragma unroll
  for (int j = 0; j < kRMax; ++j)
    if (rows.blk[j] >= 0 && rows.n[j] == 0) {
      f32x16 z[D / 32];
      zero(z);
      const long long koff = base + (long long)(rows.blk[j] * 64 + kl) * a.ss;
      store_acc<D>(z, 0.f, a.dV + koff);
      store_acc<D>(z, 0.f, a.dK + koff);
    }

  TileDma<D> dma;
  dma.init(a.ss);
  const float sc = a.scale * kLog2e;
  const float* stat_src = wave == 0 ? a.NegLse2 : a.Delta;  // wave 0: -LSE*log2(e), wave 1: Delta
  int kb = 0;
  long long koff = 0;
  uint4 kf[D / 16], vf[D / 16];
  f32x16 dk_acc[D / 32], dv_acc[D / 32];

  auto row_begin = [&](int k) {
    kb = pick(rows.blk, k);
    koff = base + (long long)(kb * 64 + kl) * a.ss;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      kf[s] = *reinterpret_cast<const uint4*>(a.K + koff + 16 * s + 8 * h2);
      vf[s] = *reinterpret_cast<const uint4*>(a.V + koff + 16 * s + 8 * h2);
    }
    zero(dk_acc);
    zero(dv_acc);
  };
  auto issue = [&](int stage, int k, int it) {
    const int qb = rows.col(k, it);
    const long long t0 = base + (long long)qb * 64 * a.ss;
    const uint32_t dst = st_addr + stage * (4 * 64 * D);
    dma.issue(dst, a.Q + t0);
    dma.issue(dst + 2 * 64 * D, a.dO + t0);
    dma4(stat_src + stat_base + qb * 64 + lane, sstat_addr + stage * 512 + wave * 256);
  };
  auto comp_body = [&](const uint16_t* stg, const float* stt, auto diag_tag) {
    constexpr bool DIAG = decltype(diag_tag)::value;
    f32x16 s_acc[2], dp_acc[2];
    mma_rows<D>(stg, kf, s_acc);               // S[q][key]
    mma_rows<D>(stg + 64 * D, vf, dp_acc);     // dP[q][key]
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int q0 = 32 * half + 8 * g + 4 * h2;            // four consecutive queries
        const float4 nl = *reinterpret_cast<const float4*>(stt + q0);
        const float4 dl = *reinterpret_cast<const float4*>(stt + 64 + q0);
        const float nls[4] = {nl.x, nl.y, nl.z, nl.w}, dls[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * g + e;
          float p = __builtin_amdgcn_exp2f(fmaf(s_acc[half][v], sc, nls[e]));
          if (DIAG && kl > q0 + e) p = 0.f;
          s_acc[half][v] = p;                                   // P
          dp_acc[half][v] = p * (dp_acc[half][v] - dls[e]);     // dS
        }
      }
    mma_transposed<D>(stg + 64 * D, s_acc, dv_acc);   // dV^T += dO^T P
    mma_transposed<D>(stg, dp_acc, dk_acc);           // dK^T += Q^T dS
  };
  auto comp = [&](int stage, int k, int it) {
    if (a.causal && rows.col(k, it) == kb)
      comp_body(st[stage], sstat[stage], TrueTag{});
    else
      comp_body(st[stage], sstat[stage], FalseTag{});
  };
  auto row_end = [&](int) {
    store_acc<D>(dv_acc, 1.f, a.dV + koff);
    store_acc<D>(dk_acc, a.scale, a.dK + koff);
  };
  walk_rows(rows, row_begin, issue, comp, row_end);
}

// Rows per workgroup: as many (up to kRMax) as still leave enough workgroups to fill the chip,
// unless the caller fixed the number.
static int g_rows_per_wg = 0;
hipError_t set_attn_rows_per_wg(int r) {
  if (r < 0 || r > kRMax) return hipErrorInvalidValue;
  g_rows_per_wg = r;
  return hipSuccess;
}
static int rows_per_wg(int nblk, int heads, int B) {
  const long long total = (long long)nblk * heads * B;
  int r = g_rows_per_wg > 0 ? g_rows_per_wg : (int)(total / 1024);
  r = r < 1 ? 1 : (r > kRMax ? kRMax : r);
  return r > nblk ? nblk : r;
}

template <int D>
static hipError_t launch_fwd(AttnArgs a, int B, hipStream_t st) {
  ProfScope ps(kKAttnFwd, st);
  const int nblk = a.S / 64;
  a.rows_per_wg = rows_per_wg(nblk, a.Hh, B);
  const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
  hipLaunchKernelGGL(attn_fwd_bf16<D>, dim3(G, a.Hh, B), dim3(kAT), 0, st, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd(AttnArgs a, int B, hipStream_t st) {
  const int nblk = a.S / 64;
  a.rows_per_wg = rows_per_wg(nblk, a.Hh, B);
  const int G = (nblk + a.rows_per_wg - 1) / a.rows_per_wg;
  {
    ProfScope ps(kKAttnDq, st);
    hipLaunchKernelGGL(attn_bwd_dq_bf16<D>, dim3(G, a.Hh, B), dim3(kAT), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKAttnDkv, st);
    hipLaunchKernelGGL(attn_bwd_dkv_bf16<D>, dim3(G, a.Hh, B), dim3(kAT), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_attn_fwd_bf16(int D, int B, const AttnArgs& a, hipStream_t st) {
  return D == 64 ? launch_fwd<64>(a, B, st) : launch_fwd<128>(a, B, st);
}
hipError_t launch_attn_bwd_bf16(int D, int B, const AttnArgs& a, hipStream_t st) {
  return D == 64 ? launch_bwd<64>(a, B, st) : launch_bwd<128>(a, B, st);
}

}  // namespace lx
