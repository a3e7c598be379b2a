// fp32 sparse FFN kernels (Sec. VI-B neuron-centric tiled products), used for
// the fp32 correctness configuration.  Plain LDS-tiled FMA kernels: on gfx950
// the fp32 vector rate equals the fp32 matrix rate, so there is nothing to gain
// from MFMA here and the straightforward tiling keeps fp32 rounding behaviour
// easy to reason about (one fused multiply-add per term, ascending k).
//
// Two kernel shapes serve all four products:
//   sdd: out block (i, j) = A_i [TT x K] . B_j [BN x K]^T for every listed
//        (token tile i, neuron block j); epilogue ReLU (+bias) or gating by the
//        stored activation sign.          (up-projection, dH)
//   dsd: out tile  = sum over listed j of Act_ij [TT x BN] . B[:, j-block]^T
//        (down-projection, dX), the contraction runs over active blocks only.
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kF32Threads = 256;
constexpr int kF32BK = 32;

// acc[a][b] += sum_k A[ty + 16a][k] * B[tx + 16b][k], k in [0, klen), klen % 32 == 0.
template <int TM, int TN>
__device__ __forceinline__ void gemm_nt_f32(const float* __restrict__ A, long long lda,
                                            const float* __restrict__ B, long long ldb, int klen,
                                            float (&acc)[TM / 16][TN / 16], float* As, float* Bs) {
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  constexpr int P = kF32BK + 1;
  for (int k0 = 0; k0 < klen; k0 += kF32BK) {
    for (int idx = tid; idx < (TM + TN) * 8; idx += kF32Threads) {
      const int row = idx / 8, seg = idx % 8;
      const float* src = row < TM ? A + (long long)row * lda : B + (long long)(row - TM) * ldb;
      const float4 v = *reinterpret_cast<const float4*>(src + k0 + seg * 4);
      float* dst = (row < TM ? As + row * P : Bs + (row - TM) * P) + seg * 4;
      dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < kF32BK; ++kk) {
      float a[TM / 16], b[TN / 16];
#pragma unroll
      for (int i = 0; i < TM / 16; ++i) a[i] = As[(ty + 16 * i) * P + kk];
#pragma unroll
      for (int j = 0; j < TN / 16; ++j) b[j] = Bs[(tx + 16 * j) * P + kk];
#pragma unroll
      for (int i = 0; i < TM / 16; ++i)
#pragma unroll
        for (int j = 0; j < TN / 16; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
}

// MODE 0: out = max(acc + bias, 0).  MODE 1: out = gate > 0 ? acc : 0.
template <int TT, int BN, int MODE>
__global__ __launch_bounds__(kF32Threads) void ffn_sdd_f32(
    const float* __restrict__ A, const float* __restrict__ W, const float* __restrict__ bias,
    const int* __restrict__ row_ptr, const int* __restrict__ col_idx, int gt, int K, int nnz_cap,
    float* __restrict__ out_act, const float* __restrict__ gate_act) {
  __shared__ float As[TT * (kF32BK + 1)];
  __shared__ float Bs[BN * (kF32BK + 1)];
  const int i = blockIdx.y;
  // gt consecutive token tiles share row i / gt of the list; the activation blocks of a list
  // row are stored as [entry][tile within the group]
  const int rs = row_ptr[i / gt], n_i = row_ptr[i / gt + 1] - rs;
  if ((int)blockIdx.x >= n_i) return;
  const int lp = rs + blockIdx.x;
  if (lp >= nnz_cap) return;       // entries beyond the capacity of the list buffers are ignored
  const int j = col_idx[lp];
  const long long p = (long long)lp * gt + i % gt;
  float acc[TT / 16][BN / 16] = {};
  gemm_nt_f32<TT, BN>(A + (long long)i * TT * K, K, W + (long long)j * BN * K, K, K, acc, As, Bs);
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
#pragma unroll
  for (int a = 0; a < TT / 16; ++a)
#pragma unroll
    for (int b = 0; b < BN / 16; ++b) {
      const int t = ty + 16 * a, n = tx + 16 * b;
      const long long o = (long long)p * TT * BN + t * BN + n;
      float v = acc[a][b];
      if (MODE == 0) {
        if (bias) v += bias[j * BN + n];
        v = v > 0.f ? v : 0.f;
      } else {
        v = gate_act[o] > 0.f ? v : 0.f;
      }
      out_act[o] = v;
    }
}

// out[i-tile, n0..n0+31] = sum_s act[p_s] [TT x BN] . W[n0.., j_s*BN ..]^T  (+ bias)
template <int TT, int BN>
__global__ __launch_bounds__(kF32Threads) void ffn_dsd_f32(
    const float* __restrict__ act, const float* __restrict__ W, long long ldw,
    const float* __restrict__ bias, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int gt, int ncols_out, int nnz_cap,
    float* __restrict__ out) {
  constexpr int CT = 32;
  __shared__ float As[TT * (kF32BK + 1)];
  __shared__ float Bs[CT * (kF32BK + 1)];
  const int i = blockIdx.y, n0 = blockIdx.x * CT;
  const int rs = row_ptr[i / gt], n_i = min(row_ptr[i / gt + 1], nnz_cap) - rs;
  float acc[TT / 16][CT / 16] = {};
  for (int s = 0; s < n_i; ++s) {
    const int p = rs + s;
    const int j = col_idx[p];
    gemm_nt_f32<TT, CT>(act + ((long long)p * gt + i % gt) * TT * BN, BN, W + (long long)n0 * ldw + (long long)j * BN,
                        ldw, BN, acc, As, Bs);
  }
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
#pragma unroll
  for (int a = 0; a < TT / 16; ++a)
#pragma unroll
    for (int b = 0; b < CT / 16; ++b) {
      const int t = i * TT + ty + 16 * a, n = n0 + tx + 16 * b;
      out[(long long)t * ncols_out + n] = acc[a][b] + (bias ? bias[n] : 0.f);
    }
}

template <int TT, int BN>
static hipError_t launch_f32(int pass, int Tt, int gt, int Fb, int d, int F, const float* A, const float* W1,
                             const float* b1, const float* W2, const float* b2, const int* row_ptr,
                             const int* col_idx, int nnz_cap, float* act_out,
                             const float* act_gate, float* out, hipStream_t st) {
  // W1: [F, d] rows = neurons (contraction over d).  W2: [d, F] (contraction over active f).
  {
    ProfScope ps(pass == 0 ? kKFfnUp : kKFfnDh, st);
    if (pass == 0)
      hipLaunchKernelGGL((ffn_sdd_f32<TT, BN, 0>), dim3(Fb, Tt), dim3(kF32Threads), 0, st, A, W1,
                         b1, row_ptr, col_idx, gt, d, nnz_cap, act_out, (const float*)nullptr);
    else
      hipLaunchKernelGGL((ffn_sdd_f32<TT, BN, 1>), dim3(Fb, Tt), dim3(kF32Threads), 0, st, A, W1,
                         (const float*)nullptr, row_ptr, col_idx, gt, d, nnz_cap, act_out, act_gate);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfScope ps(pass == 0 ? kKFfnDown : kKFfnDx, st);
  hipLaunchKernelGGL((ffn_dsd_f32<TT, BN>), dim3(d / 32, Tt), dim3(kF32Threads), 0, st,
                     (const float*)act_out, W2, (long long)F, b2, row_ptr, col_idx, gt, d, nnz_cap, out);
  return hipGetLastError();
}

// pass 0 (forward):  A = X,  W1 = W_up [F,d],     W2 = W_down [d,F], act_out = H_act, out = Y
// pass 1 (backward): A = dY, W1 = W_down_t [F,d], W2 = W_up_t [d,F], act_out = dZ_act,
//                    act_gate = H_act, out = dX
hipError_t launch_ffn_f32(int pass, int tile, int Tt, int gt, int Fb, int d, int F, const float* A,
                          const float* W1, const float* b1, const float* W2, const float* b2,
                          const int* row_ptr, const int* col_idx, int nnz_cap, float* act_out,
                          const float* act_gate, float* out, hipStream_t st) {
  if (tile == 32)
    return launch_f32<32, 32>(pass, Tt, gt, Fb, d, F, A, W1, b1, W2, b2, row_ptr, col_idx, nnz_cap,
                              act_out, act_gate, out, st);
  return launch_f32<64, 64>(pass, Tt, gt, Fb, d, F, A, W1, b1, W2, b2, row_ptr, col_idx, nnz_cap,
                            act_out, act_gate, out, st);
}

// ---------------------------------------------------------------------------
// Transpose for the one-time weight repack: dst[c][r] = src[r][c].
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ src, int R, int C,
                                                        T* __restrict__ dst) {
  __shared__ T tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  for (int rr = ty; rr < 64; rr += 4)
    if (r0 + rr < R && c0 + tx < C) tile[rr][tx] = src[(long long)(r0 + rr) * C + c0 + tx];
  __syncthreads();
  for (int cc = ty; cc < 64; cc += 4)
    if (c0 + cc < C && r0 + tx < R) dst[(long long)(c0 + cc) * R + r0 + tx] = tile[tx][cc];
}

hipError_t launch_transpose(int elem_bytes, const void* src, int R, int C, void* dst,
                            hipStream_t st) {
  dim3 grid((C + 63) / 64, (R + 63) / 64);
  ProfScope ps(kKTranspose, st);
  if (elem_bytes == 4)
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, st, (const float*)src, R, C,
                       (float*)dst);
  else
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)src, R,
                       C, (uint16_t*)dst);
  return hipGetLastError();
}

}  // namespace lx
