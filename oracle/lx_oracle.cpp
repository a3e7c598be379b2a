// CPU oracle for the Dynamic-aware Operator (Long Exposure, Sec. VI).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plainly
// written definition of what the operators compute.  It exists so that the GPU
// library can be checked against something that can be verified by eye; it is
// never part of the product path and shares no code, header, table or helper
// with the HIP sources.  Only tests, the smoke check and the benchmark's
// "cpu_baseline" leg may load it.
//
// Every function is the mathematical definition written out: inputs are fp32
// arrays (for bf16 runs they hold bf16-representable values), all arithmetic
// and all outputs are fp64, and no blocking, fusion or reordering is applied
// beyond the order of summation that the definition itself implies (ascending
// index).  The block masks are taken in their dense form (one byte per block,
// 0 = do not compute, 1 = compute: Sec. IV-B), exactly as the Exposer /
// Predictor would hand them over.
//
// Pinned by tests (none is "parity unpinned"): dense special case against
// library matmul / softmax attention, exact ReLU-support equivalence, empty
// mask, brute-force element-wise masks on tiny shapes, finite differences and
// autograd for the backward passes, closed forms, NaN poisoning of inactive
// blocks, popcount / scatter-back for the compaction, and for the MLP
// predictor brute force, the max-over-tokens closed form of the reduction and
// the threshold limits.

#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

extern "C" {

// ---------------------------------------------------------------------------
// Active-block list (Sec. VI-A "a list of data block indices", Sec. VI-B
// "indices of activated neuron blocks"): for every mask row the ascending
// column indices of its non-zero entries, rows concatenated; row_ptr[r] is
// where row r starts.  Strides are in bytes(=elements of uint8) so that the
// same routine yields the row-compressed or the column-compressed list.
// ---------------------------------------------------------------------------
void lxo_mask_compact(const uint8_t* mask, int32_t rows, int32_t cols,
                      int64_t row_stride, int64_t col_stride,
                      int32_t* row_ptr, int32_t* col_idx) {
  int32_t n = 0;
  row_ptr[0] = 0;
  for (int32_t r = 0; r < rows; ++r) {
    for (int32_t c = 0; c < cols; ++c) {
      if (mask[r * row_stride + c * col_stride] != 0) col_idx[n++] = c;
    }
    row_ptr[r + 1] = n;
  }
}

// ---------------------------------------------------------------------------
// Masked FFN forward (Sec. II-C forward equations with sigma = ReLU; Sec. II-D
// for the effect of an inactive neuron; Sec. VI-B: only active neuron blocks
// are computed).
//   Z[t,f] = sum_k X[t,k] W_up[f,k] + b_up[f]      where M[t/tile_t][f/blk_n]
//   H[t,f] = M ? max(Z,0) : 0
//   Y[t,n] = sum_f H[t,f] W_down[n,f] + b_down[n]
// X [T,d], W_up [F,d], W_down [d,F] row-major (torch.nn.Linear convention).
// b_up / b_down may be null.  M is [T/tile_t][F/blk_n] bytes.
// Outputs: H [T,F], Y [T,d] in fp64.
// ---------------------------------------------------------------------------
void lxo_ffn_fwd(int32_t T, int32_t d, int32_t F, int32_t tile_t, int32_t blk_n,
                 const float* X, const float* W_up, const float* b_up,
                 const float* W_down, const float* b_down, const uint8_t* M,
                 double* H, double* Y) {
  const int32_t Fb = F / blk_n;
  for (int32_t t = 0; t < T; ++t) {
    const uint8_t* Mrow = M + (int64_t)(t / tile_t) * Fb;
    for (int32_t f = 0; f < F; ++f) {
      double h = 0.0;
      if (Mrow[f / blk_n]) {
        double z = b_up ? (double)b_up[f] : 0.0;
        for (int32_t k = 0; k < d; ++k)
          z += (double)X[(int64_t)t * d + k] * (double)W_up[(int64_t)f * d + k];
        h = z > 0.0 ? z : 0.0;
      }
      H[(int64_t)t * F + f] = h;
    }
    for (int32_t n = 0; n < d; ++n) {
      double y = b_down ? (double)b_down[n] : 0.0;
      for (int32_t f = 0; f < F; ++f) {
        if (!Mrow[f / blk_n]) continue;  // inactive neurons are not touched
        y += H[(int64_t)t * F + f] * (double)W_down[(int64_t)n * F + f];
      }
      Y[(int64_t)t * d + n] = y;
    }
  }
}

// ---------------------------------------------------------------------------
// Masked FFN input gradient (Sec. II-D: dL/dz = ReLU' (.) dL/da, and inactive
// neurons are excluded from the backward pass; the mask is the forward one).
//   dH[t,f] = sum_n dY[t,n] W_down[n,f]             where M
//   dZ[t,f] = (M and act[t,f]) ? dH[t,f] : 0        act = [Z > 0] from forward
//   dX[t,k] = sum_f dZ[t,f] W_up[f,k]
// act is [T,F] bytes.  Outputs: dZ [T,F], dX [T,d] in fp64.
// ---------------------------------------------------------------------------
void lxo_ffn_bwd_dx(int32_t T, int32_t d, int32_t F, int32_t tile_t,
                    int32_t blk_n, const float* dY, const float* W_up,
                    const float* W_down, const uint8_t* M, const uint8_t* act,
                    double* dZ, double* dX) {
  const int32_t Fb = F / blk_n;
  for (int32_t t = 0; t < T; ++t) {
    const uint8_t* Mrow = M + (int64_t)(t / tile_t) * Fb;
    for (int32_t f = 0; f < F; ++f) {
      double g = 0.0;
      if (Mrow[f / blk_n] && act[(int64_t)t * F + f]) {
        for (int32_t n = 0; n < d; ++n)
          g += (double)dY[(int64_t)t * d + n] * (double)W_down[(int64_t)n * F + f];
      }
      dZ[(int64_t)t * F + f] = g;
    }
    for (int32_t k = 0; k < d; ++k) {
      double x = 0.0;
      for (int32_t f = 0; f < F; ++f) {
        if (!Mrow[f / blk_n]) continue;
        x += dZ[(int64_t)t * F + f] * (double)W_up[(int64_t)f * d + k];
      }
      dX[(int64_t)t * d + k] = x;
    }
  }
}

// ---------------------------------------------------------------------------
// Masked FFN with a LoRA branch on the up-projection (Sec. II-C: z = W x + B A x,
// a = sigma(z); Sec. II-D: the gradients of the trainable A and B, and the rule
// that a neuron which is inactive in the forward pass takes no part in the
// backward pass).  A [r,d], B [F,r].
//   U[t,q] = sum_k X[t,k] A[q,k]
//   Z[t,f] = sum_k X[t,k] W_up[f,k] + sum_q U[t,q] B[f,q]     where M
//   H = M ? max(Z,0) : 0;   Y[t,n] = sum_f H[t,f] W_down[n,f]
// Outputs: U [T,r], H [T,F], Y [T,d] in fp64.
// ---------------------------------------------------------------------------
void lxo_ffn_lora_fwd(int32_t T, int32_t d, int32_t F, int32_t r, int32_t tile_t, int32_t blk_n,
                      const float* X, const float* W_up, const float* A, const float* B,
                      const float* W_down, const uint8_t* M, double* U, double* H, double* Y) {
  const int32_t Fb = F / blk_n;
  for (int32_t t = 0; t < T; ++t) {
    const uint8_t* Mrow = M + (int64_t)(t / tile_t) * Fb;
    for (int32_t q = 0; q < r; ++q) {
      double u = 0.0;
      for (int32_t k = 0; k < d; ++k) u += (double)X[(int64_t)t * d + k] * (double)A[(int64_t)q * d + k];
      U[(int64_t)t * r + q] = u;
    }
    for (int32_t f = 0; f < F; ++f) {
      double h = 0.0;
      if (Mrow[f / blk_n]) {
        double z = 0.0;
        for (int32_t k = 0; k < d; ++k)
          z += (double)X[(int64_t)t * d + k] * (double)W_up[(int64_t)f * d + k];
        for (int32_t q = 0; q < r; ++q) z += U[(int64_t)t * r + q] * (double)B[(int64_t)f * r + q];
        h = z > 0.0 ? z : 0.0;
      }
      H[(int64_t)t * F + f] = h;
    }
    for (int32_t n = 0; n < d; ++n) {
      double y = 0.0;
      for (int32_t f = 0; f < F; ++f) {
        if (!Mrow[f / blk_n]) continue;
        y += H[(int64_t)t * F + f] * (double)W_down[(int64_t)n * F + f];
      }
      Y[(int64_t)t * d + n] = y;
    }
  }
}

// Backward of the above for the input and the trainable matrices.  Uin [T,r] is
// the forward's U as stored (the caller may have rounded it to the run dtype),
// act [T,F] the activation map [Z > 0].
//   dZ[t,f] = (M and act) ? sum_n dY[t,n] W_down[n,f] : 0
//   G[t,q]  = sum_f dZ[t,f] B[f,q]
//   dX[t,k] = sum_f dZ[t,f] W_up[f,k] + sum_q G[t,q] A[q,k]
//   dB[f,q] = sum_t dZ[t,f] Uin[t,q]        dA[q,k] = sum_t G[t,q] X[t,k]
// Outputs in fp64: dZ [T,F], G [T,r], dX [T,d], dA [r,d], dB [F,r].
void lxo_ffn_lora_bwd(int32_t T, int32_t d, int32_t F, int32_t r, int32_t tile_t, int32_t blk_n,
                      const float* X, const float* dY, const float* W_up, const float* A,
                      const float* B, const float* W_down, const uint8_t* M, const uint8_t* act,
                      const double* Uin, double* dZ, double* G, double* dX, double* dA,
                      double* dB) {
  const int32_t Fb = F / blk_n;
  for (int64_t i = 0; i < (int64_t)r * d; ++i) dA[i] = 0.0;
  for (int64_t i = 0; i < (int64_t)F * r; ++i) dB[i] = 0.0;
  for (int32_t t = 0; t < T; ++t) {
    const uint8_t* Mrow = M + (int64_t)(t / tile_t) * Fb;
    for (int32_t f = 0; f < F; ++f) {
      double g = 0.0;
      if (Mrow[f / blk_n] && act[(int64_t)t * F + f]) {
        for (int32_t n = 0; n < d; ++n)
          g += (double)dY[(int64_t)t * d + n] * (double)W_down[(int64_t)n * F + f];
      }
      dZ[(int64_t)t * F + f] = g;
    }
    for (int32_t q = 0; q < r; ++q) {
      double g = 0.0;
      for (int32_t f = 0; f < F; ++f) g += dZ[(int64_t)t * F + f] * (double)B[(int64_t)f * r + q];
      G[(int64_t)t * r + q] = g;
    }
    for (int32_t k = 0; k < d; ++k) {
      double x = 0.0;
      for (int32_t f = 0; f < F; ++f) x += dZ[(int64_t)t * F + f] * (double)W_up[(int64_t)f * d + k];
      for (int32_t q = 0; q < r; ++q) x += G[(int64_t)t * r + q] * (double)A[(int64_t)q * d + k];
      dX[(int64_t)t * d + k] = x;
    }
    for (int32_t f = 0; f < F; ++f) {
      const double z = dZ[(int64_t)t * F + f];
      if (z == 0.0) continue;
      for (int32_t q = 0; q < r; ++q) dB[(int64_t)f * r + q] += z * Uin[(int64_t)t * r + q];
    }
    for (int32_t q = 0; q < r; ++q)
      for (int32_t k = 0; k < d; ++k)
        dA[(int64_t)q * d + k] += G[(int64_t)t * r + q] * (double)X[(int64_t)t * d + k];
  }
}

// ---------------------------------------------------------------------------
// Block-masked attention forward, written as SDD -> softmax -> DSD (Sec. VI-A).
// Q,K,V are contiguous [B,Hh,S,D].  Mblk is [mask_batch][Hh][S/blk][S/blk]
// bytes with mask_batch 1 (shared over the batch, Sec. V-A) or B.
// A key k is allowed for query q iff its block is set and (not causal or
// k <= q).  Scores of keys that are not allowed are not computed: they take
// no part in the softmax (Sec. IV-B: 0 means non-computation).
// A row with no allowed key, or an inactive head, gives O = 0, LSE = -inf.
// Outputs: O [B,Hh,S,D], LSE [B,Hh,S] in fp64.
// ---------------------------------------------------------------------------
static inline bool key_allowed(const uint8_t* Mh, int32_t nb, int32_t blk,
                               int32_t causal, int32_t q, int32_t k) {
  if (causal && k > q) return false;
  return Mh[(int64_t)(q / blk) * nb + (k / blk)] != 0;
}

void lxo_attn_fwd(int32_t B, int32_t Hh, int32_t S, int32_t D, double scale,
                  int32_t causal, const float* Q, const float* K,
                  const float* V, int32_t blk, const uint8_t* Mblk,
                  int32_t mask_batch, const uint8_t* head_active, double* O,
                  double* LSE) {
  const int32_t nb = S / blk;
  const double ninf = -std::numeric_limits<double>::infinity();
  std::vector<double> s(S);
  for (int32_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < Hh; ++h) {
      const int64_t base = ((int64_t)b * Hh + h) * S;
      const uint8_t* Mh =
          Mblk + ((int64_t)(mask_batch == 1 ? 0 : b) * Hh + h) * nb * nb;
      const bool head_on = head_active ? head_active[h] != 0 : true;
      for (int32_t q = 0; q < S; ++q) {
        double* o = O + (base + q) * D;
        for (int32_t c = 0; c < D; ++c) o[c] = 0.0;
        // SDD: scores on allowed positions only
        double m = ninf;
        for (int32_t k = 0; k < S; ++k) {
          if (!head_on || !key_allowed(Mh, nb, blk, causal, q, k)) continue;
          double acc = 0.0;
          for (int32_t c = 0; c < D; ++c)
            acc += (double)Q[(base + q) * D + c] * (double)K[(base + k) * D + c];
          s[k] = scale * acc;
          if (s[k] > m) m = s[k];
        }
        if (m == ninf) {  // nothing allowed
          LSE[base + q] = ninf;
          continue;
        }
        // softmax over the allowed positions
        double l = 0.0;
        for (int32_t k = 0; k < S; ++k) {
          if (!key_allowed(Mh, nb, blk, causal, q, k)) continue;
          l += std::exp(s[k] - m);
        }
        LSE[base + q] = m + std::log(l);
        // DSD: O = P V
        for (int32_t k = 0; k < S; ++k) {
          if (!key_allowed(Mh, nb, blk, causal, q, k)) continue;
          const double p = std::exp(s[k] - m) / l;
          for (int32_t c = 0; c < D; ++c)
            o[c] += p * (double)V[(base + k) * D + c];
        }
      }
    }
}

// ---------------------------------------------------------------------------
// Block-masked attention backward (Sec. V-C: the backward pass mirrors the
// forward one; same mask).  Derivatives of O = softmax_allowed(scale Q K^T) V:
//   P[q,k]   as in the forward pass
//   Delta[q] = sum_c dO[q,c] O[q,c]
//   dV[k,:] += P[q,k] dO[q,:]
//   dP[q,k]  = sum_c dO[q,c] V[k,c]
//   dS[q,k]  = P[q,k] (dP[q,k] - Delta[q])
//   dQ[q,:] += scale dS[q,k] K[k,:]        dK[k,:] += scale dS[q,k] Q[q,:]
// Everything (P, O, Delta) is recomputed here in fp64; rows with no allowed key
// and inactive heads contribute nothing.  Outputs dQ,dK,dV [B,Hh,S,D] fp64.
// ---------------------------------------------------------------------------
void lxo_attn_bwd(int32_t B, int32_t Hh, int32_t S, int32_t D, double scale,
                  int32_t causal, const float* Q, const float* K,
                  const float* V, const float* dO, int32_t blk,
                  const uint8_t* Mblk, int32_t mask_batch,
                  const uint8_t* head_active, double* dQ, double* dK,
                  double* dV) {
  const int32_t nb = S / blk;
  const double ninf = -std::numeric_limits<double>::infinity();
  const int64_t total = (int64_t)B * Hh * S * D;
  for (int64_t i = 0; i < total; ++i) dQ[i] = dK[i] = dV[i] = 0.0;
  std::vector<double> s(S), p(S), o(D);
  for (int32_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < Hh; ++h) {
      if (head_active && !head_active[h]) continue;
      const int64_t base = ((int64_t)b * Hh + h) * S;
      const uint8_t* Mh =
          Mblk + ((int64_t)(mask_batch == 1 ? 0 : b) * Hh + h) * nb * nb;
      for (int32_t q = 0; q < S; ++q) {
        double m = ninf;
        for (int32_t k = 0; k < S; ++k) {
          if (!key_allowed(Mh, nb, blk, causal, q, k)) continue;
          double acc = 0.0;
          for (int32_t c = 0; c < D; ++c)
            acc += (double)Q[(base + q) * D + c] * (double)K[(base + k) * D + c];
          s[k] = scale * acc;
          if (s[k] > m) m = s[k];
        }
        if (m == ninf) continue;
        double l = 0.0;
        for (int32_t k = 0; k < S; ++k)
          if (key_allowed(Mh, nb, blk, causal, q, k)) l += std::exp(s[k] - m);
        for (int32_t c = 0; c < D; ++c) o[c] = 0.0;
        for (int32_t k = 0; k < S; ++k) {
          if (!key_allowed(Mh, nb, blk, causal, q, k)) continue;
          p[k] = std::exp(s[k] - m) / l;
          for (int32_t c = 0; c < D; ++c)
            o[c] += p[k] * (double)V[(base + k) * D + c];
        }
        double delta = 0.0;
        for (int32_t c = 0; c < D; ++c)
          delta += (double)dO[(base + q) * D + c] * o[c];
        for (int32_t k = 0; k < S; ++k) {
          if (!key_allowed(Mh, nb, blk, causal, q, k)) continue;
          double dp = 0.0;
          for (int32_t c = 0; c < D; ++c)
            dp += (double)dO[(base + q) * D + c] * (double)V[(base + k) * D + c];
          const double ds = p[k] * (dp - delta);
          for (int32_t c = 0; c < D; ++c) {
            dV[(base + k) * D + c] += p[k] * (double)dO[(base + q) * D + c];
            dQ[(base + q) * D + c] += scale * ds * (double)K[(base + k) * D + c];
            dK[(base + k) * D + c] += scale * ds * (double)Q[(base + q) * D + c];
          }
        }
      }
    }
}

// ---------------------------------------------------------------------------
// MLP predictor, inference side (Sec. V-A, "MLP Block"): approximate block
// scores S = X Wa with Wa [d, n_blk], binarised with a threshold (a block whose
// score exceeds it is kept), then reduced over the tokens of a group: a block
// is active for the group if it is active for any of its tokens (the final
// pattern must cover every token that needs the block; the paper reduces over
// batch and sequence, i.e. one group holding all tokens).
//   S[t,j]    = sum_k X[t,k] Wa[k,j]
//   M[g,j]    = OR over t in group g of (S[t,j] > thr)
// X [T,d], Wa [d,nblk] row-major; group_rows divides T.  Outputs: S [T,nblk]
// fp64 (may be null), M [T/group_rows][nblk] bytes (0/1).
// ---------------------------------------------------------------------------
void lxo_mlp_predict(int32_t T, int32_t d, int32_t nblk, int32_t group_rows,
                     const float* X, const float* Wa, double thr, double* S,
                     uint8_t* M) {
  for (int32_t g = 0; g < T / group_rows; ++g)
    for (int32_t j = 0; j < nblk; ++j) M[(int64_t)g * nblk + j] = 0;
  for (int32_t t = 0; t < T; ++t)
    for (int32_t j = 0; j < nblk; ++j) {
      double s = 0.0;
      for (int32_t k = 0; k < d; ++k)
        s += (double)X[(int64_t)t * d + k] * (double)Wa[(int64_t)k * nblk + j];
      if (S) S[(int64_t)t * nblk + j] = s;
      if (s > thr) M[(int64_t)(t / group_rows) * nblk + j] = 1;
    }
}

// ---------------------------------------------------------------------------
// Online pattern combination for multi-head attention (Sec. VI-A; the head's
// pattern is the pre-defined mask its predicted mask was categorised into,
// Sec. V-A).  pool: P dense block masks [nblk][nblk] (the atomic patterns whose
// layouts are pre-computed offline).  Head h of the Hm heads is assigned
// pattern head_pattern[h]; a negative value assigns no block at all.  The
// overall pattern of the multi-head attention is the per-head patterns side by
// side: out [Hm][nblk][nblk].  The block list the operator consumes is the
// compaction (lxo_mask_compact) of `out` viewed as Hm*nblk rows.
// ---------------------------------------------------------------------------
void lxo_attn_combine_patterns(int32_t P, int32_t nblk, const uint8_t* pool, int32_t Hm,
                               const int32_t* head_pattern, uint8_t* out) {
  const int64_t nn = (int64_t)nblk * nblk;
  for (int32_t h = 0; h < Hm; ++h) {
    const int32_t p = head_pattern[h];
    for (int32_t q = 0; q < nblk; ++q)
      for (int32_t k = 0; k < nblk; ++k)
        out[h * nn + (int64_t)q * nblk + k] =
            (p >= 0 && p < P && pool[p * nn + (int64_t)q * nblk + k] != 0) ? 1 : 0;
  }
}

}  // extern "C"
