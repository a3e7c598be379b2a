// fp32 block-sparse attention (Sec. VI-A: SDD, softmax, DSD over a block list; Sec. V-C for the
// backward pass): the correctness configuration of the attention operator, as ffn_f32.hip is for
// the FFN.  Plain multiply-adds from fp32 LDS tiles, no matrix unit; not tuned.  Tensors, the
// score / probability tile and the statistics handed from kernel to kernel are fp32; every SUM
// (dot products over the head dimension, sums over keys or queries, Delta) is accumulated in
// double.  With fp32 sums the outputs stay within 1e-5 of the fp64 definition on the largest
// error, but not element by element: a row's O carries the ~1e-6 of its accumulation as a whole,
// Delta = rowsum(dO (.) O) inherits it, and dQ of that row moves by (error of Delta) * scale * P K,
// which reads up to 2e-5 against the row's own small gradients.
//
// One workgroup of 256 threads per 64-row block of its OWN rows: a query block in the forward and
// query-side backward kernels (it walks the row list), a key block in the key-side backward
// kernel (it walks the column list).  Thread (r, p) = (tid % 64, tid / 64) works for own row r:
// in the score phase on the 16 rows 16p .. 16p+15 of the streamed block, in the accumulation
// phase on the D/4 output columns p*D/4 ..; the 64 x 64 tile of probabilities (or score
// gradients) passes through LDS in between.  Tiles are stored with a row stride of D + 1 floats,
// which spreads the rows that the 64 threads of a wavefront read at the same column over the banks.
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kFT = 256;   // threads per workgroup

template <int D>
struct F32Tiles {
  static constexpr int kLd = D + 1;            // row stride of a [64 x D] tile in LDS (floats)
  static constexpr int kTile = 64 * kLd;
  static constexpr int kSc = 64 * 65;          // a [64 x 64] score tile, row stride 65
};

// [64 x D] rows row0.. of a tensor (row stride ss elements) -> LDS tile
template <int D>
__device__ __forceinline__ void load_tile(float* __restrict__ dst, const float* __restrict__ src,
                                          long long ss) {
  for (int e = threadIdx.x; e < 64 * D; e += kFT) {
    const int r = e / D, c = e % D;
    dst[r * F32Tiles<D>::kLd + c] = src[(long long)r * ss + c];
  }
}

struct F32Head {
  long long base;     // element offset of the head's tensors
  long long stat;     // offset of its per-row statistics
  int list_row0;      // first row of the head in the block list
  bool on;
};
__device__ __forceinline__ F32Head head_of(const AttnArgs& a, int b, int h, int nblk) {
  F32Head hd;
  hd.base = (long long)b * a.sb + (long long)h * a.sh;
  hd.stat = ((long long)b * a.Hh + h) * a.S;
  hd.list_row0 = ((a.mask_batch == 1 ? 0 : b) * a.Hh + h) * nblk;
  hd.on = !a.head_active || a.head_active[h] != 0;
  return hd;
}

// forward: O and LSE of one query block.  grid (query block, head, batch)
template <int D>
__global__ __launch_bounds__(kFT) void attn_fwd_f32(const AttnArgs a, const float* __restrict__ Q,
                                                    const float* __restrict__ K, const float* __restrict__ V,
                                                    float* __restrict__ O) {
  using T = F32Tiles<D>;
  extern __shared__ float lds[];
  float* q_t = lds;                 // own queries
  float* k_t = q_t + T::kTile;
  float* v_t = k_t + T::kTile;
  float* s_t = v_t + T::kTile;      // [query][key] scores, then probabilities
  const int nblk = a.S / 64, qb = blockIdx.x;
  const F32Head hd = head_of(a, blockIdx.z, blockIdx.y, nblk);
  const int r = threadIdx.x % 64, p = threadIdx.x / 64;
  const int rs = a.row_ptr[hd.list_row0 + qb];
  const int n = hd.on ? max(min(a.row_ptr[hd.list_row0 + qb + 1], a.nnz_cap) - rs, 0) : 0;
  constexpr int kC = D / 4;                     // output columns of this thread
  double o[kC];
#pragma unroll
  for (int c = 0; c < kC; ++c) o[c] = 0.0;
  float m = -INFINITY;                          // running maximum of query r (same in all four p)
  double l = 0.0;                               // ... and sum
  if (n > 0) load_tile<D>(q_t, Q + hd.base + (long long)qb * 64 * a.ss, a.ss);
  for (int it = 0; it < n; ++it) {
    const int kb = a.col_idx[rs + it];
    __syncthreads();                            // the previous block's tiles are no longer read
    load_tile<D>(k_t, K + hd.base + (long long)kb * 64 * a.ss, a.ss);
    load_tile<D>(v_t, V + hd.base + (long long)kb * 64 * a.ss, a.ss);
    __syncthreads();
#pragma unroll 1
    for (int j = 0; j < 16; ++j) {              // scores of query r against keys 16p + j
      const int k = 16 * p + j;
      double acc = 0.0;
#pragma unroll 8
      for (int c = 0; c < D; ++c) acc += (double)q_t[r * T::kLd + c] * (double)k_t[k * T::kLd + c];
      float s = (float)(acc * (double)a.scale);
      if (a.causal && kb * 64 + k > qb * 64 + r) s = -INFINITY;   // a key after the query
      s_t[r * 65 + k] = s;
    }
    __syncthreads();
    float mb = -INFINITY;
#pragma unroll 4
    for (int k = 0; k < 64; ++k) mb = fmaxf(mb, s_t[r * 65 + k]);
    const float m_new = fmaxf(m, mb);
    if (m_new != -INFINITY) {                   // else: no allowed key so far, nothing to add
      const double alpha = exp((double)m - (double)m_new);    // exp(-inf) = 0 where m was -inf
      double sum = 0.0;
#pragma unroll
      for (int c = 0; c < kC; ++c) o[c] *= alpha;
#pragma unroll 2
      for (int k = 0; k < 64; ++k) {
        const double pr = exp((double)s_t[r * 65 + k] - (double)m_new);
        sum += pr;
        const float* vrow = v_t + k * T::kLd + p * kC;
#pragma unroll
        for (int c = 0; c < kC; ++c) o[c] += pr * (double)vrow[c];
      }
      l = l * alpha + sum;
      m = m_new;
    }
  }
  const double inv = l > 0.0 ? 1.0 / l : 0.0;
  float* orow = O + hd.base + (long long)(qb * 64 + r) * a.ss + p * kC;
#pragma unroll
  for (int c = 0; c < kC; ++c) orow[c] = (float)(o[c] * inv);
  if (p == 0) a.LSE[hd.stat + qb * 64 + r] = l > 0.0 ? (float)((double)m + log(l)) : -INFINITY;
}

// backward, query side: Delta = rowsum(dO (.) O) and dQ of one query block
template <int D>
__global__ __launch_bounds__(kFT) void attn_bwd_dq_f32(const AttnArgs a, const float* __restrict__ Q,
                                                       const float* __restrict__ K, const float* __restrict__ V,
                                                       const float* __restrict__ O, const float* __restrict__ dO,
                                                       float* __restrict__ dQ) {
  using T = F32Tiles<D>;
  extern __shared__ float lds[];
  float* q_t = lds;
  float* do_t = q_t + T::kTile;
  float* k_t = do_t + T::kTile;
  float* v_t = k_t + T::kTile;
  float* s_t = v_t + T::kTile;      // [query][key] dS
  const int nblk = a.S / 64, qb = blockIdx.x;
  const F32Head hd = head_of(a, blockIdx.z, blockIdx.y, nblk);
  const int r = threadIdx.x % 64, p = threadIdx.x / 64;
  const int rs = a.row_ptr[hd.list_row0 + qb];
  const int n = hd.on ? max(min(a.row_ptr[hd.list_row0 + qb + 1], a.nnz_cap) - rs, 0) : 0;
  constexpr int kC = D / 4;
  double g[kC];
#pragma unroll
  for (int c = 0; c < kC; ++c) g[c] = 0.0;
  const long long row = hd.base + (long long)(qb * 64 + r) * a.ss;
  const float lse = a.LSEin[hd.stat + qb * 64 + r];
  double delta = 0.0;
  if (n > 0) {
    load_tile<D>(q_t, Q + hd.base + (long long)qb * 64 * a.ss, a.ss);
    load_tile<D>(do_t, dO + hd.base + (long long)qb * 64 * a.ss, a.ss);
    for (int c = 0; c < D; ++c) delta += (double)dO[row + c] * (double)O[row + c];
  }
  if (p == 0) a.Delta[hd.stat + qb * 64 + r] = (float)delta;      // for the key-side kernel
  for (int it = 0; it < n; ++it) {
    const int kb = a.col_idx[rs + it];
    __syncthreads();
    load_tile<D>(k_t, K + hd.base + (long long)kb * 64 * a.ss, a.ss);
    load_tile<D>(v_t, V + hd.base + (long long)kb * 64 * a.ss, a.ss);
    __syncthreads();
#pragma unroll 1
    for (int j = 0; j < 16; ++j) {
      const int k = 16 * p + j;
      double s = 0.0, dp = 0.0;
#pragma unroll 8
      for (int c = 0; c < D; ++c) {
        s += (double)q_t[r * T::kLd + c] * (double)k_t[k * T::kLd + c];
        dp += (double)do_t[r * T::kLd + c] * (double)v_t[k * T::kLd + c];
      }
      const bool allowed = !(a.causal && kb * 64 + k > qb * 64 + r) && lse != -INFINITY;
      const double pr = allowed ? exp(s * (double)a.scale - (double)lse) : 0.0;
      s_t[r * 65 + k] = (float)(pr * (dp - delta));
    }
    __syncthreads();
#pragma unroll 2
    for (int k = 0; k < 64; ++k) {
      const double ds = s_t[r * 65 + k];
      const float* krow = k_t + k * T::kLd + p * kC;
#pragma unroll
      for (int c = 0; c < kC; ++c) g[c] += ds * (double)krow[c];
    }
  }
  float* grow = dQ + row + p * kC;
#pragma unroll
  for (int c = 0; c < kC; ++c) grow[c] = (float)(g[c] * (double)a.scale);
}

// backward, key side: dK and dV of one key block (walks the column list: entries = query blocks)
template <int D>
__global__ __launch_bounds__(kFT) void attn_bwd_dkv_f32(const AttnArgs a, const float* __restrict__ Q,
                                                        const float* __restrict__ K, const float* __restrict__ V,
                                                        const float* __restrict__ dO, float* __restrict__ dK,
                                                        float* __restrict__ dV) {
  using T = F32Tiles<D>;
  extern __shared__ float lds[];
  float* k_t = lds;                 // own keys
  float* v_t = k_t + T::kTile;
  float* q_t = v_t + T::kTile;
  float* do_t = q_t + T::kTile;
  float* s_t = do_t + T::kTile;     // [key][query]: P, then dS
  const int nblk = a.S / 64, kb = blockIdx.x;
  const F32Head hd = head_of(a, blockIdx.z, blockIdx.y, nblk);
  const int r = threadIdx.x % 64, p = threadIdx.x / 64;     // own key r
  const int rs = a.crow_ptr[hd.list_row0 + kb];
  const int n = hd.on ? max(min(a.crow_ptr[hd.list_row0 + kb + 1], a.cnnz_cap) - rs, 0) : 0;
  constexpr int kC = D / 4;
  double gk[kC], gv[kC];
#pragma unroll
  for (int c = 0; c < kC; ++c) gk[c] = gv[c] = 0.0;
  if (n > 0) {
    load_tile<D>(k_t, K + hd.base + (long long)kb * 64 * a.ss, a.ss);
    load_tile<D>(v_t, V + hd.base + (long long)kb * 64 * a.ss, a.ss);
  }
  for (int it = 0; it < n; ++it) {
    const int qb = a.ccol_idx[rs + it];
    __syncthreads();
    load_tile<D>(q_t, Q + hd.base + (long long)qb * 64 * a.ss, a.ss);
    load_tile<D>(do_t, dO + hd.base + (long long)qb * 64 * a.ss, a.ss);
    __syncthreads();
    float ds_keep[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {              // key r against queries 16p + j
      const int q = 16 * p + j;
      double s = 0.0, dp = 0.0;
#pragma unroll 8
      for (int c = 0; c < D; ++c) {
        s += (double)q_t[q * T::kLd + c] * (double)k_t[r * T::kLd + c];
        dp += (double)do_t[q * T::kLd + c] * (double)v_t[r * T::kLd + c];
      }
      const float lse = a.LSEin[hd.stat + qb * 64 + q];
      const bool allowed = !(a.causal && kb * 64 + r > qb * 64 + q) && lse != -INFINITY;
      const double pr = allowed ? exp(s * (double)a.scale - (double)lse) : 0.0;
      s_t[r * 65 + q] = (float)pr;
      ds_keep[j] = (float)(pr * (dp - (double)a.Delta[hd.stat + qb * 64 + q]));
    }
    __syncthreads();
#pragma unroll 2
    for (int q = 0; q < 64; ++q) {              // dV += P^T dO
      const double pr = s_t[r * 65 + q];
      const float* drow = do_t + q * T::kLd + p * kC;
#pragma unroll
      for (int c = 0; c < kC; ++c) gv[c] += pr * (double)drow[c];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) s_t[r * 65 + 16 * p + j] = ds_keep[j];
    __syncthreads();
#pragma unroll 2
    for (int q = 0; q < 64; ++q) {              // dK += dS^T Q
      const double ds = s_t[r * 65 + q];
      const float* qrow = q_t + q * T::kLd + p * kC;
#pragma unroll
      for (int c = 0; c < kC; ++c) gk[c] += ds * (double)qrow[c];
    }
  }
  const long long row = hd.base + (long long)(kb * 64 + r) * a.ss + p * kC;
#pragma unroll
  for (int c = 0; c < kC; ++c) {
    dV[row + c] = (float)gv[c];
    dK[row + c] = (float)(gk[c] * (double)a.scale);
  }
}

template <int D>
static hipError_t launch_f32_fwd(const AttnArgs& a, int B, hipStream_t st) {
  using T = F32Tiles<D>;
  const size_t lds = (3 * T::kTile + T::kSc) * sizeof(float);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd_f32<D>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  ProfScope ps(kKAttnFwd, st);
  hipLaunchKernelGGL(attn_fwd_f32<D>, dim3(a.S / 64, a.Hh, B), dim3(kFT), lds, st, a, (const float*)a.Q,
                     (const float*)a.K, (const float*)a.V, (float*)a.Out);
  return hipGetLastError();
}
template <int D>
static hipError_t launch_f32_bwd(const AttnArgs& a, int B, hipStream_t st) {
  using T = F32Tiles<D>;
  const size_t lds = (4 * T::kTile + T::kSc) * sizeof(float);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dq_f32<D>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv_f32<D>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  const dim3 grid(a.S / 64, a.Hh, B);
  {
    ProfScope ps(kKAttnDq, st);
    hipLaunchKernelGGL(attn_bwd_dq_f32<D>, grid, dim3(kFT), lds, st, a, (const float*)a.Q, (const float*)a.K,
                       (const float*)a.V, (const float*)a.O, (const float*)a.dO, (float*)a.dQ);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfScope ps(kKAttnDkv, st);
  hipLaunchKernelGGL(attn_bwd_dkv_f32<D>, grid, dim3(kFT), lds, st, a, (const float*)a.Q, (const float*)a.K,
                     (const float*)a.V, (const float*)a.dO, (float*)a.dK, (float*)a.dV);
  return hipGetLastError();
}

// The tensor pointers of AttnArgs are typed for the 16-bit kernels; the fp32 calls pass float
// tensors through them (strides in elements either way).
hipError_t launch_attn_fwd_f32(int D, int B, const AttnArgs& a, hipStream_t st) {
  return D == 64 ? launch_f32_fwd<64>(a, B, st) : launch_f32_fwd<128>(a, B, st);
}
hipError_t launch_attn_bwd_f32(int D, int B, const AttnArgs& a, hipStream_t st) {
  return D == 64 ? launch_f32_bwd<64>(a, B, st) : launch_f32_bwd<128>(a, B, st);
}

}  // namespace lx
