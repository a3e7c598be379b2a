// Block-sparse attention for gfx950 (Sec. VI-A).  The two block-sparse products
// of the paper -- SDD (scores on listed blocks) and DSD (probabilities times
// V) -- are fused with the softmax in flash style, so the score blocks live
// only in registers; the unit of work is the listed block, which is what keeps
// heads with different patterns balanced (Sec. VI-A, online combination).
//
// Layout of one workgroup (128 threads = 2 wavefronts): a 64-row query block
// (forward, dQ) or a 64-row key block (dK/dV); each wavefront owns 32 of the
// rows and walks the block list of its row of the mask.  All products run on
// the 32x32x16 bf16 MFMA with fp32 accumulators.
//
// Data movement: the [64 x D] tiles of the listed blocks go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane), double buffered: the
// tiles of list entry it+1 are in flight while entry it is computed.  The two
// stages are separate LDS arrays so that the compiler's LDS-DMA tracking does
// not wait for the in-flight stage.  Tiles are row-major, unpadded, with the
// 16-byte slots of a row XOR-swizzled by the row index (bank spreading).
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
  __device__ __forceinline__ void issue(uint16_t* tile, const uint16_t* g0) const {
    const int wave = threadIdx.x / kWave;
#pragma unroll
    for (int u = 0; u < kPerWave; ++u)
      __builtin_amdgcn_global_load_lds((const LX_AS1 void*)(g0 + off[u]),
                                       (LX_AS3 void*)(tile + (wave + 2 * u) * 512), 16, 0, 0);
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
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int row = 32 * half + r;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const uint4 a = *reinterpret_cast<const uint4*>(tile + row * D +
                                                      (((2 * s + h2) ^ tswz<D>(row)) << 3));
      // the first product starts from a literal zero (no register clearing); acc is overwritten
      acc[half] = mfma32(a, frag[s], s == 0 ? zero16 : acc[half]);
    }
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

// out[ct] += T^T . P   where T is a row-major [64 x D] tile in LDS (read transposed) and
// p[half][v] the accumulator-layout values of the [64 x 32] factor (rounded to bf16 here).
template <int D>
__device__ __forceinline__ void mma_transposed(const uint16_t* tile, const f32x16 (&p)[2],
                                               f32x16 (&out)[D / 32]) {
  const int lane = threadIdx.x % kWave, h2 = lane / 32;
  const int j = lane % 16, e = j / 4, q = j % 4;
  const int cbase = 16 * ((lane / 16) % 2) + 4 * q;      // + 32*ct
#pragma unroll
  for (int s2 = 0; s2 < 4; ++s2) {
    const int half = s2 / 2, g0 = 2 * (s2 % 2);
    uint4 b;
    b.x = pack2bf(p[half][4 * g0 + 0], p[half][4 * g0 + 1]);
    b.y = pack2bf(p[half][4 * g0 + 2], p[half][4 * g0 + 3]);
    b.z = pack2bf(p[half][4 * g0 + 4], p[half][4 * g0 + 5]);
    b.w = pack2bf(p[half][4 * g0 + 6], p[half][4 * g0 + 7]);
    const int r_lo = 16 * s2 + 4 * h2 + e, r_hi = r_lo + 8;
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) {
      const int col = 32 * ct + cbase;
      const uint16_t* p_lo = tile + r_lo * D + (((col >> 3) ^ tswz<D>(r_lo)) << 3) + (col & 7);
      const uint16_t* p_hi = tile + r_hi * D + (((col >> 3) ^ tswz<D>(r_hi)) << 3) + (col & 7);
      const uint2 lo = __builtin_bit_cast(
          uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LX_AS3 short4v*)p_lo));
      const uint2 hi = __builtin_bit_cast(
          uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LX_AS3 short4v*)p_hi));
      out[ct] = mfma32(make_uint4(lo.x, lo.y, hi.x, hi.y), b, out[ct]);
    }
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

// Double-buffered walk over n list entries: issue0/issue1 start the DMA of an entry into
// stage 0/1, comp0/comp1 consume it.  A wave first waits for its own DMA (vmcnt), the barrier
// then makes the whole stage visible and retires the reads of the stage about to be refilled.
template <class I0, class I1, class C0, class C1>
__device__ __forceinline__ void walk2(int n, I0 issue0, I1 issue1, C0 comp0, C1 comp1) {
  if (n > 0) issue0(0);
  for (int it = 0; it < n; it += 2) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (it + 1 < n) issue1(it + 1);
    comp0(it);
    if (it + 1 < n) {
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      if (it + 2 < n) issue0(it + 2);
      comp1(it + 1);
    }
  }
}

// ---------------------------------------------------------------------------
// forward: O, LSE for one (batch, head, query block)
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT, D == 64 ? 2 : 1) void attn_fwd_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t st0[2 * 64 * D];   // K tile, V tile
  __shared__ __attribute__((aligned(1024))) uint16_t st1[2 * 64 * D];
  const int nqb = a.S / 64;
  const int qb = nqb - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int ql = 32 * wave + lane % 32, h2 = lane / 32;
  const int row = ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nqb + qb;
  const int rs = a.row_ptr[row];
  int n = a.row_ptr[row + 1] - rs;
  if (a.head_active && !a.head_active[h]) n = 0;
  const long long base = (long long)b * a.sb + (long long)h * a.sh;
  const long long qoff = base + (long long)(qb * 64 + ql) * a.ss;
  if (n == 0) {   // no listed block (or inactive head): O = 0, LSE = -inf, nothing to read
    f32x16 z[D / 32];
    zero(z);
    store_acc<D>(z, 0.f, a.Out + qoff);
    if (h2 == 0) a.LSE[((long long)b * a.Hh + h) * a.S + qb * 64 + ql] = -INFINITY;
    return;
  }

  uint4 qf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qf[s] = *reinterpret_cast<const uint4*>(a.Q + qoff + 16 * s + 8 * h2);

  TileDma<D> dma;
  dma.init(a.ss);
  f32x16 o_acc[D / 32];
  zero(o_acc);
  float m = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  ListRow list;
  list.init(a.col_idx + rs, n);
  auto issue = [&](uint16_t* st, int it) {
    const long long t0 = base + (long long)list.get(it) * 64 * a.ss;
    dma.issue(st, a.K + t0);
    dma.issue(st + 64 * D, a.V + t0);
  };
  // DIAG: the diagonal block of a causal mask, where keys after the query are excluded.  Two
  // separate instantiations (instead of a branch in the middle) keep the 32 score registers in
  // place on both paths.
  auto comp_body = [&](const uint16_t* st, auto diag_tag) {
    constexpr bool DIAG = decltype(diag_tag)::value;
    f32x16 s_acc[2];
    mma_rows<D>(st, qf, s_acc);           // S^T[key][q]
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
    mma_transposed<D>(st + 64 * D, s_acc, o_acc);   // O^T += V^T P^T
  };
  auto comp = [&](const uint16_t* st, int it) {
    if (a.causal && list.get(it) == qb)
      comp_body(st, TrueTag{});
    else
      comp_body(st, FalseTag{});
  };
  walk2(n, [&](int it) { issue(st0, it); }, [&](int it) { issue(st1, it); },
        [&](int it) { comp(st0, it); }, [&](int it) { comp(st1, it); });

  const bool any = lsum > 0.f;
  const float inv = any ? 1.f / lsum : 0.f;
  store_acc<D>(o_acc, inv, a.Out + qoff);
  if (h2 == 0)
    a.LSE[((long long)b * a.Hh + h) * a.S + qb * 64 + ql] =
        any ? (m + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
}

// ---------------------------------------------------------------------------
// backward, query side: Delta and dQ for one (batch, head, query block)
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT, D == 64 ? 2 : 1) void attn_bwd_dq_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t st0[2 * 64 * D];   // K tile, V tile
  __shared__ __attribute__((aligned(1024))) uint16_t st1[2 * 64 * D];
  const int nqb = a.S / 64;
  const int qb = nqb - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int ql = 32 * wave + lane % 32, h2 = lane / 32;
  const int row = ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nqb + qb;
  const int rs = a.row_ptr[row];
  int n = a.row_ptr[row + 1] - rs;
  if (a.head_active && !a.head_active[h]) n = 0;
  const long long base = (long long)b * a.sb + (long long)h * a.sh;
  const long long qoff = base + (long long)(qb * 64 + ql) * a.ss;
  const long long stat = ((long long)b * a.Hh + h) * a.S + qb * 64 + ql;
  if (n == 0) {   // no listed block (or inactive head): O = 0, hence Delta = 0 and dQ = 0
    f32x16 z[D / 32];
    zero(z);
    store_acc<D>(z, 0.f, a.dQ + qoff);
    if (h2 == 0) {
      a.Delta[stat] = 0.f;
      a.NegLse2[stat] = INFINITY;
    }
    return;
  }

  uint4 qf[D / 16], dof[D / 16];
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
  const float delta = part + __shfl_xor(part, 32);
  const float lse2 = a.LSEin[stat] * kLog2e;
  if (h2 == 0) {                     // for the key-side kernel: Delta and -LSE in log2 units
    a.Delta[stat] = delta;
    a.NegLse2[stat] = -lse2;
  }
  const float sc = a.scale * kLog2e;

  TileDma<D> dma;
  dma.init(a.ss);
  f32x16 dq_acc[D / 32];
  zero(dq_acc);

  ListRow list;
  list.init(a.col_idx + rs, n);
  auto issue = [&](uint16_t* st, int it) {
    const long long t0 = base + (long long)list.get(it) * 64 * a.ss;
    dma.issue(st, a.K + t0);
    dma.issue(st + 64 * D, a.V + t0);
  };
  auto comp_body = [&](const uint16_t* st, auto diag_tag) {
    constexpr bool DIAG = decltype(diag_tag)::value;
    f32x16 s_acc[2], dp_acc[2];
    mma_rows<D>(st, qf, s_acc);              // S^T[key][q]
    mma_rows<D>(st + 64 * D, dof, dp_acc);   // dP^T[key][q]
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
    mma_transposed<D>(st, s_acc, dq_acc);    // dQ^T += K^T dS^T
  };
  auto comp = [&](const uint16_t* st, int it) {
    if (a.causal && list.get(it) == qb)
      comp_body(st, TrueTag{});
    else
      comp_body(st, FalseTag{});
  };
  walk2(n, [&](int it) { issue(st0, it); }, [&](int it) { issue(st1, it); },
        [&](int it) { comp(st0, it); }, [&](int it) { comp(st1, it); });
  store_acc<D>(dq_acc, a.scale, a.dQ + qoff);
}

// ---------------------------------------------------------------------------
// backward, key side: dK and dV for one (batch, head, key block)
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT, D == 64 ? 2 : 1) void attn_bwd_dkv_bf16(const AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t st0[2 * 64 * D];   // Q tile, dO tile
  __shared__ __attribute__((aligned(1024))) uint16_t st1[2 * 64 * D];
  __shared__ __attribute__((aligned(256))) float stat0[128];            // -LSE*log2e [64], Delta [64]
  __shared__ __attribute__((aligned(256))) float stat1[128];
  const int nkb = a.S / 64;
  const int kb = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int kl = 32 * wave + lane % 32, h2 = lane / 32;
  const int row = ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nkb + kb;
  const int rs = a.crow_ptr[row];
  int n = a.crow_ptr[row + 1] - rs;
  if (a.head_active && !a.head_active[h]) n = 0;
  const long long base = (long long)b * a.sb + (long long)h * a.sh;
  const long long koff = base + (long long)(kb * 64 + kl) * a.ss;
  const long long stat_base = ((long long)b * a.Hh + h) * a.S;
  if (n == 0) {   // key block used by no query block: zero gradients, nothing to read
    f32x16 z[D / 32];
    zero(z);
    store_acc<D>(z, 0.f, a.dV + koff);
    store_acc<D>(z, 0.f, a.dK + koff);
    return;
  }

  uint4 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    kf[s] = *reinterpret_cast<const uint4*>(a.K + koff + 16 * s + 8 * h2);
    vf[s] = *reinterpret_cast<const uint4*>(a.V + koff + 16 * s + 8 * h2);
  }
  const float sc = a.scale * kLog2e;
  TileDma<D> dma;
  dma.init(a.ss);
  f32x16 dk_acc[D / 32], dv_acc[D / 32];
  zero(dk_acc);
  zero(dv_acc);
  const float* stat_src = wave == 0 ? a.NegLse2 : a.Delta;  // wave 0: -LSE*log2(e), wave 1: Delta

  ListRow list;
  list.init(a.ccol_idx + rs, n);
  auto issue = [&](uint16_t* st, float* sstat, int it) {
    const int qb = list.get(it);
    const long long t0 = base + (long long)qb * 64 * a.ss;
    dma.issue(st, a.Q + t0);
    dma.issue(st + 64 * D, a.dO + t0);
    __builtin_amdgcn_global_load_lds((const LX_AS1 void*)(stat_src + stat_base + qb * 64 + lane),
                                     (LX_AS3 void*)(sstat + 64 * wave), 4, 0, 0);
  };
  auto comp_body = [&](const uint16_t* st, const float* sstat, auto diag_tag) {
    constexpr bool DIAG = decltype(diag_tag)::value;
    f32x16 s_acc[2], dp_acc[2];
    mma_rows<D>(st, kf, s_acc);               // S[q][key]
    mma_rows<D>(st + 64 * D, vf, dp_acc);     // dP[q][key]
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int q0 = 32 * half + 8 * g + 4 * h2;            // four consecutive queries
        const float4 nl = *reinterpret_cast<const float4*>(sstat + q0);
        const float4 dl = *reinterpret_cast<const float4*>(sstat + 64 + q0);
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
    mma_transposed<D>(st + 64 * D, s_acc, dv_acc);   // dV^T += dO^T P
    mma_transposed<D>(st, dp_acc, dk_acc);           // dK^T += Q^T dS
  };
  auto comp = [&](const uint16_t* st, const float* sstat, int it) {
    if (a.causal && list.get(it) == kb)
      comp_body(st, sstat, TrueTag{});
    else
      comp_body(st, sstat, FalseTag{});
  };
  walk2(n, [&](int it) { issue(st0, stat0, it); }, [&](int it) { issue(st1, stat1, it); },
        [&](int it) { comp(st0, stat0, it); }, [&](int it) { comp(st1, stat1, it); });
  store_acc<D>(dv_acc, 1.f, a.dV + koff);
  store_acc<D>(dk_acc, a.scale, a.dK + koff);
}

template <int D>
static hipError_t launch_fwd(const AttnArgs& a, int B, hipStream_t st) {
  ProfScope ps(kKAttnFwd, st);
  hipLaunchKernelGGL(attn_fwd_bf16<D>, dim3(a.S / 64, a.Hh, B), dim3(kAT), 0, st, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd(const AttnArgs& a, int B, hipStream_t st) {
  {
    ProfScope ps(kKAttnDq, st);
    hipLaunchKernelGGL(attn_bwd_dq_bf16<D>, dim3(a.S / 64, a.Hh, B), dim3(kAT), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKAttnDkv, st);
    hipLaunchKernelGGL(attn_bwd_dkv_bf16<D>, dim3(a.S / 64, a.Hh, B), dim3(kAT), 0, st, a);
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
