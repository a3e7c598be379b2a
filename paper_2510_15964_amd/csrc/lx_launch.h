// Internal launch interface between the C-ABI host code and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lx {

constexpr int kCUs = 256;   // compute units of the chip
// element types of the 16-bit kernels (the `dt` argument of their launchers)
constexpr int kBf16 = 0, kF16 = 1;

// Kernel ids of the profiling aid (values are part of the C ABI: lx_kernel in lx.h).
enum KernelId {
  kKCompact = 0, kKFfnUp = 1, kKFfnDown = 2, kKFfnDh = 3, kKFfnDx = 4,
  kKAttnFwd = 5, kKAttnDq = 6, kKAttnDkv = 7, kKTranspose = 8, kKPredict = 9, kKCombine = 10, kKLora = 11, kKCount = 12
};
void prof_pre(int id, hipStream_t st);
void prof_post(int id, hipStream_t st);
// Brackets the launches issued while it is alive with a pair of events when kernel `id`
// is the one selected by lx_profile_begin; otherwise costs one integer compare.
struct ProfScope {
  int id;
  hipStream_t st;
  ProfScope(int id_, hipStream_t st_) : id(id_), st(st_) { prof_pre(id, st); }
  ~ProfScope() { prof_post(id, st); }
};

struct AttnArgs {
  const uint16_t *Q, *K, *V, *O, *dO;
  uint16_t *Out, *dQ, *dK, *dV;
  float *LSE, *Delta, *NegLse2;
  const float* LSEin;
  long long sb, sh, ss;
  const int *row_ptr, *col_idx;
  const int *crow_ptr, *ccol_idx;
  int nnz_cap, cnnz_cap;   // capacities of col_idx / ccol_idx: entries beyond them are ignored
  const uint8_t* head_active;
  int Hh, S, mask_batch, causal;
  float scale;
  int rows_per_wg;   // rows of the mask per workgroup, set by the launcher
  int vheads;        // consecutive heads whose rows one group of workgroups shares, set by the launcher
};

hipError_t launch_compact(const uint8_t*, int, int, int, long long, long long, long long, int*, int*,
                          int, hipStream_t);
// One compaction job: `batch` masks of rows x cols bytes -> one list (see lx_mask_compact).
struct CompactJob {
  const uint8_t* mask;
  int batch, rows, cols;
  long long bstride, rstride, cstride;
  int* row_ptr;
  int* col_idx;
  int cap;
};
hipError_t launch_compact_jobs(const CompactJob* jobs, int n, hipStream_t stream);
// One list built by the pattern combination: pool layout in, per-head layout out.
struct CombineList {
  const int* pool_row_ptr;   // [P*nblk + 1]
  const int* pool_col_idx;
  int pool_cap;
  int* row_ptr;              // [n_heads*nblk + 1]
  int* col_idx;
  int cap;
};
hipError_t launch_combine_patterns(const CombineList* lists, int n_lists, const int* head_pattern,
                                   int P, int nblk, int n_heads, hipStream_t stream);
hipError_t launch_compact_pair(const uint8_t*, int, int, int, long long, long long, long long, int*,
                               int*, int*, int*, int, hipStream_t);
hipError_t launch_ffn_f32(int pass, int tile, int Tt, int gt, int Fb, int d, int F, const float* A,
                          const float* W1, const float* b1, const float* W2, const float* b2,
                          const int* row_ptr, const int* col_idx, int nnz_cap, float* act_out,
                          const float* act_gate, float* out, hipStream_t st);
hipError_t launch_ffn_bf16(int dt, int pass, int Tt, int gt, int Fb, int d, int F, const uint16_t* A,
                           const uint16_t* W1, const uint16_t* b1, const uint16_t* W2,
                           const uint16_t* b2, const int* row_ptr, const int* col_idx, int nnz_cap,
                           uint16_t* act_out, const uint16_t* act_gate, uint16_t* out,
                           float* part, size_t part_bytes, hipStream_t st);
// bytes of partial sums with which the second product of a pass, given ONE list row of at most
// nnz_cap entries for all Tt token tiles, splits the lists of its last round of workgroups (0: never)
size_t ffn_dsd_split_bytes(int Tt, int d, int nnz_cap);
// Splits of the low-rank products of the LoRA branch over workgroups so that they fill the chip;
// the partial sums are added in a fixed order.  U = X A^T: over K; dB: over ranges of token
// tiles per neuron block; dA: over ranges of token tiles per 64-column chunk.
inline int lora_clamp(int s, int hi) { return s < 1 ? 1 : (s > hi ? (hi < 1 ? 1 : hi) : s); }
inline int lora_u_split(int Tt, int d) {
  const int by_k = d / 64 / 4;   // at least four K-steps per workgroup
  return lora_clamp((kCUs + Tt - 1) / Tt, by_k < 8 ? by_k : 8);
}
inline int lora_g_split(int Tt) { return lora_clamp((kCUs + Tt - 1) / Tt, 4); }   // over list entries
inline int lora_db_split(int Tt, int F) {
  const int s = lora_clamp((2 * kCUs + F / 64 - 1) / (F / 64), Tt < 16 ? Tt : 16);
  const int need = (Tt + 511) / 512;   // the kernel searches one tile of its range per thread
  return s > need ? s : need;
}
inline int lora_da_split(int Tt, int d) {
  return lora_clamp((kCUs + d / 64 - 1) / (d / 64), Tt < 32 ? Tt : 32);
}
// the small products of the LoRA branch (lora_bf16.hip); dt = kBf16 or kF16
hipError_t launch_lora_u(int dt, int Tt, int d, const uint16_t* X, const uint16_t* A_pad, uint16_t* U,
                         float* u_part, hipStream_t st);
hipError_t launch_lora_g(int dt, int Tt, int gt, int F, const uint16_t* dZ, const uint16_t* B_t,
                         const int* row_ptr, const int* col_idx, int nnz_cap, uint16_t* G,
                         float* g_part, hipStream_t st);
hipError_t launch_lora_transposes(int d, int F, const uint16_t* A_pad, uint16_t* A_t,
                                  const uint16_t* B_pad, uint16_t* B_t, hipStream_t st);
hipError_t launch_lora_grads(int dt, int Tt, int gt, int d, int F, const uint16_t* dZ,
                             const uint16_t* U, const uint16_t* G, const uint16_t* X,
                             const int* row_ptr, const int* col_idx, int nnz_cap, float* da_part,
                             float* db_part, float* dA, float* dB, hipStream_t st);
hipError_t launch_ffn_lora_fwd_bf16(int dt, int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* W_up, const uint16_t* A_pad,
                                    const uint16_t* B_pad, const uint16_t* W_down,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* U, uint16_t* H_act, uint16_t* Y, float* u_part,
                                    hipStream_t st);
hipError_t launch_ffn_lora_bwd_bf16(int dt, int Tt, int gt, int d, int F, const uint16_t* X,
                                    const uint16_t* dY, const uint16_t* H_act, const uint16_t* U,
                                    const uint16_t* W_down_t, const uint16_t* W_up_t,
                                    const uint16_t* A_pad, const uint16_t* B_pad,
                                    const int* row_ptr, const int* col_idx, int nnz_cap,
                                    uint16_t* dZ, uint16_t* B_t, uint16_t* A_t, uint16_t* G,
                                    float* g_part, float* da_part, float* db_part, uint16_t* dX,
                                    float* dA, float* dB, hipStream_t st);
hipError_t launch_predict_bf16(int dt, int T, int d, int nblk, int tiles_per_group, const uint16_t* X,
                               const uint16_t* Wa_t, float thr, uint8_t* mask, hipStream_t st);
hipError_t launch_transpose(int elem_bytes, const void* src, int R, int C, void* dst, hipStream_t st);
// Listed blocks of W [Fb][block_bytes] (device or device-addressable host memory) -> Wc, in the
// order of the one-row list; optionally the list of the compact matrix (see compact.hip).
hipError_t launch_gather_blocks(const void* W, int Fb, long long block_bytes, const int* row_ptr,
                                const int* col_idx, int cap, void* Wc, int* id_row_ptr,
                                int* id_col_idx, hipStream_t stream);
hipError_t launch_attn_fwd_bf16(int dt, int D, int B, const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_bwd_bf16(int dt, int D, int B, const AttnArgs& a, hipStream_t st);
// measurement aids (probe.hip)
hipError_t launch_probe_mfma(int iters, float* sink, hipStream_t st);
double probe_mfma_flops(int iters);
hipError_t launch_probe_copy(const void* src, void* dst, long long units16, hipStream_t st);
// fp32 attention (attn_f32.hip): AttnArgs' tensor pointers then hold float tensors
hipError_t launch_attn_fwd_f32(int D, int B, const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_bwd_f32(int D, int B, const AttnArgs& a, hipStream_t st);
hipError_t set_attn_rows_per_wg(int r);   // 0 = automatic
hipError_t set_ffn_tiles_per_wg(int n);   // 0 = automatic, 1, 2

}  // namespace lx
