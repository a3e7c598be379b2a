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
// Trick used throughout: the first product is computed transposed (S^T = K Q^T)
// so that every lane holds scores of ONE query and the accumulator registers
// can be fed straight back as the B operand of the second product; the MFMA's
// k index may be permuted freely as long as both operands agree, so the A
// operand (V^T, K^T, Q^T, dO^T from LDS) is read in the matching order
// { 16s+4h .. +3, 16s+8+4h .. +3 }.  Operands needed "k-major" are written to
// LDS transposed, two rows packed per 32-bit store.
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kAT = 128;                 // threads per workgroup
constexpr int kTP = 68;                  // pitch (elements) of transposed tiles [D][64]
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int D>
struct Tile {                            // a [64 x D] bf16 tile held across the workgroup
  static constexpr int kTasks = D / 32;  // per thread: (row pair, 8-column group) tasks
  uint4 lo[kTasks], hi[kTasks];          // row 2rp and row 2rp+1
};

template <int D>
__device__ __forceinline__ void tile_fetch(Tile<D>& t, const uint16_t* __restrict__ g,
                                           long long ld) {
#pragma unroll
  for (int u = 0; u < Tile<D>::kTasks; ++u) {
    const int task = threadIdx.x + kAT * u;
    const int cg = task % (D / 8), rp = task / (D / 8);
    t.lo[u] = *reinterpret_cast<const uint4*>(g + (long long)(2 * rp) * ld + cg * 8);
    t.hi[u] = *reinterpret_cast<const uint4*>(g + (long long)(2 * rp + 1) * ld + cg * 8);
  }
}

// row-major copy: lds[row][c], pitch D+8
template <int D>
__device__ __forceinline__ void tile_store_rows(const Tile<D>& t, uint16_t* lds) {
#pragma unroll
  for (int u = 0; u < Tile<D>::kTasks; ++u) {
    const int task = threadIdx.x + kAT * u;
    const int cg = task % (D / 8), rp = task / (D / 8);
    *reinterpret_cast<uint4*>(lds + (2 * rp) * (D + 8) + cg * 8) = t.lo[u];
    *reinterpret_cast<uint4*>(lds + (2 * rp + 1) * (D + 8) + cg * 8) = t.hi[u];
  }
}

// transposed copy: lds[c][row], pitch kTP; rows 2rp, 2rp+1 share one 32-bit word
template <int D>
__device__ __forceinline__ void tile_store_transposed(const Tile<D>& t, uint16_t* lds) {
  uint32_t* w = reinterpret_cast<uint32_t*>(lds);
#pragma unroll
  for (int u = 0; u < Tile<D>::kTasks; ++u) {
    const int task = threadIdx.x + kAT * u;
    const int cg = task % (D / 8), rp = task / (D / 8);
    const uint32_t a[4] = {t.lo[u].x, t.lo[u].y, t.lo[u].z, t.lo[u].w};
    const uint32_t b[4] = {t.hi[u].x, t.hi[u].y, t.hi[u].z, t.hi[u].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int c = cg * 8 + 2 * e;
      w[(c * kTP) / 2 + rp] = (a[e] & 0xFFFFu) | (b[e] << 16);
      w[((c + 1) * kTP) / 2 + rp] = (a[e] >> 16) | (b[e] & 0xFFFF0000u);
    }
  }
}

// acc[half] += R[rows 32*half + lane%32][:] . F^T   where R is a row-major LDS tile and
// F the per-lane register fragments (column index = lane%32).  Result register v of a lane is
// element (row 32*half + 8*(v/4) + 4*(lane/32) + v%4, column lane%32).
template <int D>
__device__ __forceinline__ void mma_rows(const uint16_t* lds, const uint4 (&frag)[D / 16],
                                         f32x16 (&acc)[2]) {
  const int lane = threadIdx.x % kWave, r = lane % 32, kq = (lane / 32) * 8;
#pragma unroll
  for (int half = 0; half < 2; ++half)
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const uint4 a = *reinterpret_cast<const uint4*>(lds + (32 * half + r) * (D + 8) + 16 * s + kq);
      acc[half] = mfma32(a, frag[s], acc[half]);
    }
}

// out[ct] += T^T-tile . P   where lds holds the transposed tile [D][64] and p[half][v] are the
// fp32 accumulator-layout values of the [64 x 32] factor (rounded to bf16 here).
template <int D>
__device__ __forceinline__ void mma_transposed(const uint16_t* lds, const f32x16 (&p)[2],
                                               f32x16 (&out)[D / 32]) {
  const int lane = threadIdx.x % kWave, r = lane % 32, h2 = lane / 32;
#pragma unroll
  for (int s2 = 0; s2 < 4; ++s2) {
    const int half = s2 / 2, g0 = 2 * (s2 % 2);
    uint4 b;
    b.x = pack2bf(p[half][4 * g0 + 0], p[half][4 * g0 + 1]);
    b.y = pack2bf(p[half][4 * g0 + 2], p[half][4 * g0 + 3]);
    b.z = pack2bf(p[half][4 * g0 + 4], p[half][4 * g0 + 5]);
    b.w = pack2bf(p[half][4 * g0 + 6], p[half][4 * g0 + 7]);
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) {
      const uint16_t* row = lds + (32 * ct + r) * kTP + 16 * s2 + 4 * h2;
      const uint2 lo = *reinterpret_cast<const uint2*>(row);
      const uint2 hi = *reinterpret_cast<const uint2*>(row + 8);
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


// ---------------------------------------------------------------------------
// forward: O, LSE for one (batch, head, query block)
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT) void attn_fwd_bf16(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* Ks = smem;                    // [64][D+8]
  uint16_t* Vt = smem + 64 * (D + 8);     // [D][kTP]
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

  uint4 qf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qf[s] = *reinterpret_cast<const uint4*>(a.Q + qoff + 16 * s + 8 * h2);

  f32x16 o_acc[D / 32];
  zero(o_acc);
  float m = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  for (int it = 0; it < n; ++it) {
    const int kb = a.col_idx[rs + it];
    if (a.causal && kb > qb) continue;
    Tile<D> tk, tv;
    tile_fetch<D>(tk, a.K + base + (long long)kb * 64 * a.ss, a.ss);
    tile_fetch<D>(tv, a.V + base + (long long)kb * 64 * a.ss, a.ss);
    __syncthreads();
    tile_store_rows<D>(tk, Ks);
    tile_store_transposed<D>(tv, Vt);
    __syncthreads();

    f32x16 s_acc[2];
    zero(s_acc);
    mma_rows<D>(Ks, qf, s_acc);
    const bool diag = a.causal && kb == qb;
    float mloc = -INFINITY;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float x = s_acc[half][v] * sc;
        const int kl = 32 * half + 8 * (v / 4) + 4 * h2 + v % 4;
        if (diag && kl > ql) x = -INFINITY;
        s_acc[half][v] = x;
        mloc = fmaxf(mloc, x);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m, mloc);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    float psum = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(s_acc[half][v] - m_new);
        s_acc[half][v] = p;
        psum += p;
      }
    psum += __shfl_xor(psum, 32);
    lsum = lsum * alpha + psum;
    m = m_new;
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
      for (int v = 0; v < 16; ++v) o_acc[ct][v] *= alpha;
    mma_transposed<D>(Vt, s_acc, o_acc);
  }

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
__global__ __launch_bounds__(kAT) void attn_bwd_dq_bf16(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* Ks = smem;                          // [64][D+8]
  uint16_t* Vs = Ks + 64 * (D + 8);             // [64][D+8]
  uint16_t* Kt = Vs + 64 * (D + 8);             // [D][kTP]
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
  if (h2 == 0) a.Delta[stat] = delta;
  const float lse2 = a.LSEin[stat] * kLog2e;
  const float sc = a.scale * kLog2e;

  f32x16 dq_acc[D / 32];
  zero(dq_acc);
  for (int it = 0; it < n; ++it) {
    const int kb = a.col_idx[rs + it];
    if (a.causal && kb > qb) continue;
    Tile<D> tk, tv;
    tile_fetch<D>(tk, a.K + base + (long long)kb * 64 * a.ss, a.ss);
    tile_fetch<D>(tv, a.V + base + (long long)kb * 64 * a.ss, a.ss);
    __syncthreads();
    tile_store_rows<D>(tk, Ks);
    tile_store_transposed<D>(tk, Kt);
    tile_store_rows<D>(tv, Vs);
    __syncthreads();

    f32x16 s_acc[2], dp_acc[2];
    zero(s_acc);
    zero(dp_acc);
    mma_rows<D>(Ks, qf, s_acc);     // S^T[key][q]
    mma_rows<D>(Vs, dof, dp_acc);   // dP^T[key][q]
    const bool diag = a.causal && kb == qb;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int kl = 32 * half + 8 * (v / 4) + 4 * h2 + v % 4;
        float p = __builtin_amdgcn_exp2f(s_acc[half][v] * sc - lse2);
        if (diag && kl > ql) p = 0.f;
        s_acc[half][v] = p * (dp_acc[half][v] - delta);   // dS^T
      }
    mma_transposed<D>(Kt, s_acc, dq_acc);
  }
  store_acc<D>(dq_acc, a.scale, a.dQ + qoff);
}

// ---------------------------------------------------------------------------
// backward, key side: dK and dV for one (batch, head, key block)
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAT) void attn_bwd_dkv_bf16(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* Qs = smem;                          // [64][D+8]
  uint16_t* dOs = Qs + 64 * (D + 8);            // [64][D+8]
  uint16_t* Qt = dOs + 64 * (D + 8);            // [D][kTP]
  uint16_t* dOt = Qt + D * kTP;                 // [D][kTP]
  float* lse_s = reinterpret_cast<float*>(dOt + D * kTP);  // [64] (log2 units)
  float* del_s = lse_s + 64;                               // [64]
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
  const long long stat0 = ((long long)b * a.Hh + h) * a.S;

  uint4 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    kf[s] = *reinterpret_cast<const uint4*>(a.K + koff + 16 * s + 8 * h2);
    vf[s] = *reinterpret_cast<const uint4*>(a.V + koff + 16 * s + 8 * h2);
  }
  const float sc = a.scale * kLog2e;
  f32x16 dk_acc[D / 32], dv_acc[D / 32];
  zero(dk_acc);
  zero(dv_acc);

  for (int it = 0; it < n; ++it) {
    const int qb = a.ccol_idx[rs + it];
    if (a.causal && qb < kb) continue;
    Tile<D> tq, tdo;
    tile_fetch<D>(tq, a.Q + base + (long long)qb * 64 * a.ss, a.ss);
    tile_fetch<D>(tdo, a.dO + base + (long long)qb * 64 * a.ss, a.ss);
    float stat_v = 0.f;
    if (threadIdx.x < 64) stat_v = a.LSEin[stat0 + qb * 64 + threadIdx.x] * kLog2e;
    else stat_v = a.Delta[stat0 + qb * 64 + threadIdx.x - 64];
    __syncthreads();
    tile_store_rows<D>(tq, Qs);
    tile_store_transposed<D>(tq, Qt);
    tile_store_rows<D>(tdo, dOs);
    tile_store_transposed<D>(tdo, dOt);
    lse_s[threadIdx.x] = stat_v;   // threads 64..127 land in del_s
    __syncthreads();

    f32x16 s_acc[2], dp_acc[2];
    zero(s_acc);
    zero(dp_acc);
    mma_rows<D>(Qs, kf, s_acc);     // S[q][key]
    mma_rows<D>(dOs, vf, dp_acc);   // dP[q][key]
    const bool diag = a.causal && kb == qb;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ql = 32 * half + 8 * (v / 4) + 4 * h2 + v % 4;
        float p = __builtin_amdgcn_exp2f(s_acc[half][v] * sc - lse_s[ql]);
        if (diag && kl > ql) p = 0.f;
        s_acc[half][v] = p;                                   // P
        dp_acc[half][v] = p * (dp_acc[half][v] - del_s[ql]);  // dS
      }
    mma_transposed<D>(dOt, s_acc, dv_acc);
    mma_transposed<D>(Qt, dp_acc, dk_acc);
  }
  store_acc<D>(dv_acc, 1.f, a.dV + koff);
  store_acc<D>(dk_acc, a.scale, a.dK + koff);
}

template <int D>
static size_t fwd_lds() { return (64 * (D + 8) + D * kTP) * 2; }
template <int D>
static size_t dq_lds() { return (2 * 64 * (D + 8) + D * kTP) * 2; }
template <int D>
static size_t dkv_lds() { return (2 * 64 * (D + 8) + 2 * D * kTP) * 2 + 128 * 4; }

template <int D>
static hipError_t launch_fwd(const AttnArgs& a, int B, hipStream_t st) {
  ProfScope ps(kKAttnFwd, st);
  hipLaunchKernelGGL(attn_fwd_bf16<D>, dim3(a.S / 64, a.Hh, B), dim3(kAT), fwd_lds<D>(), st, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd(const AttnArgs& a, int B, hipStream_t st) {
  static bool attr_set = false;   // raise the dynamic LDS limit once (above 64 KiB for D = 128)
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dkv_bf16<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)dkv_lds<D>());
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  {
    ProfScope ps(kKAttnDq, st);
    hipLaunchKernelGGL(attn_bwd_dq_bf16<D>, dim3(a.S / 64, a.Hh, B), dim3(kAT), dq_lds<D>(), st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(kKAttnDkv, st);
    hipLaunchKernelGGL(attn_bwd_dkv_bf16<D>, dim3(a.S / 64, a.Hh, B), dim3(kAT), dkv_lds<D>(), st, a);
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
