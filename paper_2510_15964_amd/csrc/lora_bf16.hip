// The small products of the LoRA branch on the up-projection (Sec. II-C: z = W x + B A x;
// Sec. II-D: its gradients) for gfx950: U = X A^T, dB = dZ^T U over the listed blocks,
// dA = G^T X, and the transposes of the two matrices.  A_pad [64, d] and B_pad [F, 64] hold
// A [r, d] and B [F, r] zero-padded to rank 64.  The branch's steps inside the up-projection and
// the input-gradient product live in the FFN kernels themselves.
#include "ffn_ring.h"

namespace lx {

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

// out[t][q] = sum over steps of sum_k P_s[t][k] Q_s[q][k] for token tile blockIdx.x ([64 x 64], both
// operands read along their rows) over the range of steps of blockIdx.y.
// MODE 0, U = X A_pad^T (Sec. II-C: the inner factor A x of the branch): P = X, Q = A_pad, row
//   stride ld of both; the steps are the ld / 64 chunks of K.
// MODE 1, G = dZ B_pad (Sec. II-D: the gradient that reaches A x): P = the compact blocks dZ_ij of
//   the tile's list, Q = B_t [64, ld]; the steps are the list entries, step s takes the columns
//   64 j_s .. of B_t.
// gridDim.y == 1: out [T,64] is stored in the element type; otherwise fp32 partial sums
// part[y][T][64], which lora_u_reduce_kernel adds.
template <int DT, int MODE>
__global__ __launch_bounds__(kThreads) void lora_nt_kernel(
    const uint16_t* __restrict__ P, const uint16_t* __restrict__ Q, int ld,
    const int* __restrict__ row_ptr, const int* __restrict__ col_idx, int gt, int nnz_cap,
    uint16_t* __restrict__ U, float* __restrict__ part, long long part_stride) {
  __shared__ __attribute__((aligned(1024))) uint16_t ring[kPairStages * kPairElems];
  const int i = blockIdx.x;
  int rs = 0, nsteps = ld / kBK;
  if (MODE == 1) {
    rs = row_ptr[i / gt];
    nsteps = max(min(row_ptr[i / gt + 1], nnz_cap) - rs, 0);   // entries beyond the capacity are ignored
  }
  const int per = (nsteps + gridDim.y - 1) / gridDim.y;
  const int s_lo = blockIdx.y * per, s_hi = min(nsteps, s_lo + per);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int th = wave % 2, qh = (wave / 2) % 2, kh = wave / 4;
  const int r = lane % 32, h2 = lane / 32;
  const uint16_t* src[2];
  if (MODE == 0)
    pair_src(P + (long long)i * 64 * ld, ld, Q, ld, src);
  else
    pair_src(P, 64, Q, ld, src);
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  run_ring_of<kPairStages, 2, kPairElems>(
      s_hi - s_lo, src, NoAlt(),
      [=](int s, long long& ob, long long& oa) {
        if (MODE == 0) {
          ob = oa = (long long)(s_lo + s) * kBK;
        } else {
          const int e = rs + s_lo + s;
          ob = ((long long)e * gt + i % gt) * 4096;
          oa = (long long)col_idx[e] * 64;
        }
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
// U (or G) = the sum of the parts, in order, rounded to the element type; n4 = number of groups
// of four elements
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

// U = X A_pad^T [T,64].  u_part: lora_u_split(Tt, d) * T * 64 floats of scratch (unused for a
// split of 1).
template <int DT>
static hipError_t launch_lora_u_t(int Tt, int d, const uint16_t* X, const uint16_t* A_pad, uint16_t* U,
                                  float* u_part, hipStream_t st) {
  const int split = lora_u_split(Tt, d);
  const long long n = (long long)Tt * 4096;
  const int* none = nullptr;
  hipLaunchKernelGGL((lora_nt_kernel<DT, 0>), dim3(Tt, split), dim3(kThreads), 0, st, X, A_pad, d, none,
                     none, 1, 0, U, u_part, n);
  if (split > 1)
    hipLaunchKernelGGL(lora_u_reduce_kernel<DT>, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st,
                       (const float*)u_part, split, n / 4, U);
  return hipGetLastError();
}
hipError_t launch_lora_u(int dt, int Tt, int d, const uint16_t* X, const uint16_t* A_pad, uint16_t* U,
                         float* u_part, hipStream_t st) {
  return LX_BY_DT(launch_lora_u_t, Tt, d, X, A_pad, U, u_part, st);
}

// G = dZ B_pad [T,64] from the compact blocks dZ and B_t [64,F].  g_part: lora_g_split(Tt) * T * 64
// floats of scratch (unused for a split of 1).
template <int DT>
static hipError_t launch_lora_g_t(int Tt, int gt, int F, const uint16_t* dZ, const uint16_t* B_t,
                                  const int* row_ptr, const int* col_idx, int nnz_cap, uint16_t* G,
                                  float* g_part, hipStream_t st) {
  const int split = lora_g_split(Tt);
  const long long n = (long long)Tt * 4096;
  hipLaunchKernelGGL((lora_nt_kernel<DT, 1>), dim3(Tt, split), dim3(kThreads), 0, st, dZ, B_t, F, row_ptr,
                     col_idx, gt, nnz_cap, G, g_part, n);
  if (split > 1)
    hipLaunchKernelGGL(lora_u_reduce_kernel<DT>, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st,
                       (const float*)g_part, split, n / 4, G);
  return hipGetLastError();
}
hipError_t launch_lora_g(int dt, int Tt, int gt, int F, const uint16_t* dZ, const uint16_t* B_t,
                         const int* row_ptr, const int* col_idx, int nnz_cap, uint16_t* G,
                         float* g_part, hipStream_t st) {
  return LX_BY_DT(launch_lora_g_t, Tt, gt, F, dZ, B_t, row_ptr, col_idx, nnz_cap, G, g_part, st);
}

hipError_t launch_lora_transposes(int d, int F, const uint16_t* A_pad, uint16_t* A_t,
                                  const uint16_t* B_pad, uint16_t* B_t, hipStream_t st) {
  hipLaunchKernelGGL(lora_transpose_kernel, dim3(d / 64 + F / 64), dim3(256), 0, st, A_pad, d, A_t,
                     B_pad, F, B_t);
  return hipGetLastError();
}

// dB = dZ^T U over the listed blocks and dA = G^T X.  Scratch: da_part [lora_da_split][64][d] and
// db_part [lora_db_split][F][64] (each unused for a split of 1).
template <int DT>
static hipError_t launch_lora_grads_t(int Tt, int gt, int d, int F, const uint16_t* dZ,
                                      const uint16_t* U, const uint16_t* G, const uint16_t* X,
                                      const int* row_ptr, const int* col_idx, int nnz_cap,
                                      float* da_part, float* db_part, float* dA, float* dB,
                                      hipStream_t st) {
  const int sb = lora_db_split(Tt, F), sa = lora_da_split(Tt, d);
  const long long nb = (long long)F * 64, na = (long long)64 * d;
  hipLaunchKernelGGL((lora_tn_kernel<DT, 0>), dim3(F / 64, sb), dim3(kThreads), 0, st, dZ, U, 64ll,
                     row_ptr, col_idx, Tt, gt, nnz_cap, sb > 1 ? db_part : dB, nb, 64);
  hipLaunchKernelGGL((lora_tn_kernel<DT, 1>), dim3(d / 64, sa), dim3(kThreads), 0, st, G, X,
                     (long long)d, row_ptr, col_idx, Tt, gt, nnz_cap, sa > 1 ? da_part : dA, na, d);
  const long long n4b = sb > 1 ? nb / 4 : 0, n4a = sa > 1 ? na / 4 : 0;
  if (n4b + n4a > 0)
    hipLaunchKernelGGL(lora_grad_reduce_kernel, dim3((unsigned)((n4b + n4a + 255) / 256)), dim3(256), 0,
                       st, (const float*)db_part, sb, n4b, dB, (const float*)da_part, sa, n4a, dA);
  return hipGetLastError();
}
hipError_t launch_lora_grads(int dt, int Tt, int gt, int d, int F, const uint16_t* dZ,
                             const uint16_t* U, const uint16_t* G, const uint16_t* X,
                             const int* row_ptr, const int* col_idx, int nnz_cap, float* da_part,
                             float* db_part, float* dA, float* dB, hipStream_t st) {
  return LX_BY_DT(launch_lora_grads_t, Tt, gt, d, F, dZ, U, G, X, row_ptr, col_idx, nnz_cap, da_part,
                  db_part, dA, dB, st);
}

}  // namespace lx
