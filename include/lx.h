/*
 * lx.h -- C ABI of the Dynamic-aware Operator for MI355X (gfx950).
 *
 * The library implements the sparse operators of Long Exposure, Sec. VI: a
 * frozen-weight transformer layer evaluated only on the blocks that a binary
 * block mask marks as active (Sec. IV-B: 1 = compute, 0 = do not compute), in
 * the forward pass and in the input-gradient backward pass (Sec. II-D: what is
 * inactive in the forward pass is excluded from the backward pass; Sec. V-C:
 * the backward savings mirror the forward ones).
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer unless its comment says HOST.
 *     lx_blocklist itself is a HOST struct holding DEVICE pointers.
 *   - The caller owns every buffer, including workspaces.  The library never
 *     allocates or frees device memory, never synchronises the host with the
 *     device, and enqueues work only on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream).  Calls return as soon as the work is
 *     enqueued.
 *   - All arguments are validated on the host BEFORE anything is launched;
 *     on any status other than LX_OK nothing has been enqueued and no output
 *     has been touched.  Contents of device-resident index lists are trusted
 *     (checking them would need a host synchronisation).
 *   - Outputs are fully overwritten: rows / heads without an active block are
 *     written as zeros (LSE as -inf), never left stale.
 *   - Matrices are row-major with the last dimension contiguous.  Data
 *     pointers must be 16-byte aligned.
 *   - bf16 runs keep fp32 accumulators; intermediates that feed a second
 *     matrix product (H, dZ, P, dS) are rounded to bf16 once.
 */
#ifndef LX_H_
#define LX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LX_OK = 0,
  LX_ERR_INVALID_ARG = 1, /* null pointer, non-positive or inconsistent size, misalignment */
  LX_ERR_UNSUPPORTED = 2, /* dtype / block size / head size not built */
  LX_ERR_WORKSPACE = 3,   /* workspace missing or smaller than the *_workspace_bytes query */
  LX_ERR_RUNTIME = 4      /* a HIP launch reported an error */
} lx_status;

/*
 * Element type of the tensors of a call.  LX_BF16 and LX_F16 (IEEE half, the parameter
 * precision of Sec. VII-A) run the same kernels: 16-bit operands, products accumulated in
 * fp32, outputs rounded to nearest even; softmax statistics and the gradients of the LoRA
 * matrices are fp32 for both.  LX_F32 is the correctness configuration of the FFN and of attention.
 */
typedef enum { LX_F32 = 0, LX_BF16 = 1, LX_F16 = 2 } lx_dtype;

/*
 * Row-compressed active-block list: the "list of data block indices" of
 * Sec. VI-A and the "indices of activated neuron blocks" of Sec. VI-B.
 * Row r owns col_idx[row_ptr[r] .. row_ptr[r+1]), ascending, no duplicates.
 *   FFN:        rows = T / tile_t (token tiles),      cols = F / blk_n (neuron blocks);
 *               rows may also be any divisor of T / tile_t: row r is then the
 *               list of the (T/tile_t)/rows consecutive token tiles of group r.
 *               rows = 1 is the paper's own case, one list reduced over batch
 *               and sequence (Sec. V-A) and shared by all tokens.
 *   attention:  rows = mask_batch * Hh * (S/64),      cols = S / 64
 *               (query-block rows for the row list; key-block rows for the
 *               column list used by the backward pass)
 * nnz_cap is a host-known upper bound on the number of active blocks (rows*cols
 * if nothing better is known); it sizes H_act and bounds launch grids, because
 * the true count lives only on the device.  If row_ptr counts more entries
 * than nnz_cap (a bound that was too small), every call ignores the entries
 * after the first nnz_cap in list order: the results are those of the
 * truncated list and nothing outside the stated buffers is read or written.
 * (The attention backward call takes two lists of the same mask; each is
 * truncated by itself, so dQ and dK/dV then belong to different truncations:
 * give both lists the capacity of the mask's true block count.)
 *
 * Setting the environment variable LX_LOG=1 makes every entry point that
 * enqueues work print one line with its name, sizes and status to stderr.
 */
typedef struct {
  int32_t rows;
  int32_t cols;
  const int32_t* row_ptr; /* DEVICE [rows + 1], row_ptr[0] == 0 */
  const int32_t* col_idx; /* DEVICE [>= nnz_cap] */
  int32_t nnz_cap;
} lx_blocklist;

/* Kernels that lx_profile_begin can select (one per step of the hot path). */
typedef enum {
  LX_K_COMPACT = 0,      /* mask compaction */
  LX_K_FFN_UP = 1,       /* H_ij = ReLU(X_i W_up_j^T) on listed blocks */
  LX_K_FFN_DOWN = 2,     /* Y_i = sum_j H_ij W_down_j^T */
  LX_K_FFN_DH = 3,       /* dZ_ij = (dY_i W_down_j) (.) [H_ij > 0] */
  LX_K_FFN_DX = 4,       /* dX_i = sum_j dZ_ij W_up_j */
  LX_K_ATTN_FWD = 5,     /* fused SDD + softmax + DSD */
  LX_K_ATTN_BWD_DQ = 6,  /* Delta and dQ, query side */
  LX_K_ATTN_BWD_DKV = 7, /* dK and dV, key side */
  LX_K_TRANSPOSE = 8,    /* weight repack */
  LX_K_PREDICT = 9,      /* MLP predictor: scores + threshold + OR over the tokens */
  LX_K_COMBINE = 10,     /* per-head pattern layouts -> multi-head block list */
  LX_K_LORA = 11         /* LoRA branch: U = X A^T, G = dZ B, dB, dA (the fused steps run in the FFN kernels) */
} lx_kernel;

/* Human-readable name of a status code (HOST string, static storage). */
const char* lx_status_string(lx_status s);

/*
 * Mask compaction (online step of Sec. VI-A; index list of Sec. VI-B).
 * Turns `batch` dense byte masks of rows x cols blocks into one row-compressed
 * list with batch*rows rows.  Entry (g, r, c) is read at
 * mask[g*batch_stride + r*row_stride + c*col_stride] (strides in bytes); any
 * non-zero byte counts as active.  Swapping row and column strides (and
 * rows/cols) yields the column-compressed list.
 *   row_ptr  out, int32[batch*rows + 1]
 *   col_idx  out, int32[col_idx_cap]; col_idx_cap must be >= batch*rows*cols
 *            unless the caller knows a tighter bound on the active count
 *            (entries beyond the capacity are dropped, row_ptr stays exact).
 * The result is unique (ascending columns), hence bit-exact reproducible.
 * Errors: INVALID_ARG for null pointers, non-positive sizes or capacity.
 */
lx_status lx_mask_compact(const uint8_t* mask, int32_t batch, int32_t rows, int32_t cols,
                          int64_t batch_stride, int64_t row_stride, int64_t col_stride,
                          int32_t* row_ptr, int32_t* col_idx, int32_t col_idx_cap, void* stream);

/*
 * The same compaction for the row-compressed AND the column-compressed list of
 * the same masks in a single launch (the attention backward pass walks both).
 * Row list: batch*rows rows of column indices into (row_ptr_r, col_idx_r);
 * column list: batch*cols rows of row indices into (row_ptr_c, col_idx_c).
 * col_idx_cap applies to each of the two index buffers.
 */
lx_status lx_mask_compact_pair(const uint8_t* mask, int32_t batch, int32_t rows, int32_t cols,
                               int64_t batch_stride, int64_t row_stride, int64_t col_stride,
                               int32_t* row_ptr_r, int32_t* col_idx_r, int32_t* row_ptr_c,
                               int32_t* col_idx_c, int32_t col_idx_cap, void* stream);

/*
 * Several independent compactions in ONE launch (all masks of a layer step: the
 * FFN token-tile masks and both attention lists), one workgroup per job.  Each
 * job has the meaning of one lx_mask_compact call.  `jobs` is a HOST array of
 * 1..8 entries holding DEVICE pointers; it is copied into the launch.
 */
typedef struct {
  const uint8_t* mask;
  int32_t batch, rows, cols;
  int64_t batch_stride, row_stride, col_stride;
  int32_t* row_ptr;
  int32_t* col_idx;
  int32_t col_idx_cap;
} lx_compact_job;
lx_status lx_mask_compact_batch(const lx_compact_job* jobs, int32_t n_jobs, void* stream);

/*
 * Online pattern combination for multi-head attention (Sec. VI-A).  Offline, the
 * pool: the layouts of n_patterns block patterns [nblk][nblk], i.e. the lists
 * lx_mask_compact builds from their dense masks with batch = n_patterns (pool_r,
 * rows = n_patterns*nblk, cols = nblk) and, for the backward pass, the
 * column-compressed lists of the same masks (pool_c, may be NULL together with
 * row_ptr_c and col_idx_c).  Online, per step: head h (of n_heads = mask_batch *
 * heads) is assigned pattern head_pattern[h] (DEVICE int32[n_heads]; a value
 * outside 0..n_patterns-1 assigns no block), and the call writes the list of
 * the whole attention, rows ordered (head, block row): the layout of each
 * head's pattern shifted by the number of blocks of the heads before it.  The
 * result equals lx_mask_compact on the dense mask [n_heads][nblk][nblk] whose
 * head h is a copy of its pattern; no mask is read or written.
 *   row_ptr_r / row_ptr_c  out, int32[n_heads*nblk + 1]
 *   col_idx_r / col_idx_c  out, int32[col_idx_cap] (entries beyond the capacity,
 *                          or beyond the pool's, are dropped; row_ptr stays exact)
 * Errors: INVALID_ARG for null pointers, non-positive sizes, or a pool whose
 * rows / cols do not match n_patterns and nblk.
 */
lx_status lx_attn_combine_patterns(const lx_blocklist* pool_r, const lx_blocklist* pool_c,
                                   int32_t n_patterns, int32_t nblk, const int32_t* head_pattern,
                                   int32_t n_heads, int32_t* row_ptr_r, int32_t* col_idx_r,
                                   int32_t* row_ptr_c, int32_t* col_idx_c, int32_t col_idx_cap,
                                   void* stream);

/*
 * One-time repack of the frozen weights (Sec. VI-B "memory coalescing": each
 * product reads its weights along the contiguous dimension).  Writes the
 * transposes W_up_t[d,F] = W_up[F,d]^T and W_down_t[F,d] = W_down[d,F]^T, which
 * the backward call uses.  Either output may be NULL to skip it.
 */
lx_status lx_ffn_pack_weights(lx_dtype dt, int32_t d, int32_t F, const void* W_up,
                              const void* W_down, void* W_up_t, void* W_down_t, void* stream);

/*
 * Weights kept in CPU memory (Sec. VII-B, memory footprint: with only the active
 * neurons computed, most of the MLP weights can stay on the CPU and only the
 * active ones are moved to the GPU).  Copies the listed neuron blocks of a
 * neuron-major matrix W [F,d] (the blk_n rows of a neuron block adjacent: W_up,
 * or W_down_t as lx_ffn_pack_weights writes it) into the compact matrix
 * Wc [nnz_cap*blk_n, d], entry k of the list becoming rows k*blk_n .. of Wc.
 *   W    [F,d]: DEVICE memory, or HOST memory that the device can address
 *        (allocated pinned, e.g. hipHostMalloc); read by the kernel on `stream`,
 *        so the caller keeps it unchanged until the stream has passed the call
 *   bl   DEVICE list with ONE row (the list shared by all token tiles),
 *        cols = F/blk_n
 *   Wc   out, DEVICE [bl->nnz_cap*blk_n, d]; rows of entries past the end of
 *        the list are left as they were
 *   compact_row_ptr / compact_col_idx   out, nullable: DEVICE int32[2] and
 *        int32[bl->nnz_cap], the one-row list {0, n}, 0 .. of the compact matrix:
 *        with it, Wc (and its transpose from lx_ffn_pack_weights) in place of the
 *        full matrices and F' = nnz_cap*blk_n, the FFN calls below compute
 *        exactly what they compute from the full matrices and bl.
 * Errors: INVALID_ARG for null pointers, sizes that do not match, a list with
 * more than one row, pointers not 16-byte aligned, or W in pageable host memory
 * (nothing is launched); UNSUPPORTED for an unknown element type.
 */
lx_status lx_ffn_gather_weight_blocks(lx_dtype dt, int32_t d, int32_t F, int32_t blk_n,
                                      const void* W, const lx_blocklist* bl, void* Wc,
                                      int32_t* compact_row_ptr, int32_t* compact_col_idx,
                                      void* stream);

/* Workspace (bytes) for lx_sparse_ffn_fwd / lx_sparse_ffn_bwd_dx.
 * nnz_cap: capacity of the activation buffers in blocks, i.e. bl->nnz_cap times
 *   the number of token tiles per list row ((T/tile_t)/bl->rows, 1 for a list
 *   row per tile).
 * have_h_act: the caller passes an H_act buffer to the forward call.
 * have_packed: the caller passes W_up_t and W_down_t to the backward call. */
size_t lx_sparse_ffn_fwd_workspace_bytes(lx_dtype dt, int32_t T, int32_t d, int32_t F,
                                         int32_t tile_t, int32_t blk_n, int32_t nnz_cap,
                                         int32_t have_h_act);
size_t lx_sparse_ffn_bwd_workspace_bytes(lx_dtype dt, int32_t T, int32_t d, int32_t F,
                                         int32_t tile_t, int32_t blk_n, int32_t nnz_cap,
                                         int32_t have_packed);

/*
 * Optional extra workspace of the two FFN calls (16-bit types).  With ONE list row for all token
 * tiles the second product of a pass (Y, dX) runs as (group of token tiles) x (256 output
 * columns) units, all equally long; when they make whole rounds of workgroups plus a small rest,
 * that rest would keep a fraction of the chip busy for a full round.  Given this many bytes
 * BEYOND what lx_sparse_ffn_fwd_workspace_bytes / lx_sparse_ffn_bwd_workspace_bytes return (the
 * same pointer, a larger workspace_bytes), the calls cut the lists of the rest's units into
 * pieces that fill the last round and add the pieces' fp32 partial sums in a fixed order
 * (reproducible; the outputs of those units then differ in the last bit from the unsplit sum).
 * Returns 0 where no split would be made (several list rows, units that fill their rounds, lists
 * whose bound bl->nnz_cap is too short to cut); a workspace without the extra bytes is always
 * valid and gives the unsplit sums.
 */
size_t lx_sparse_ffn_split_workspace_bytes(lx_dtype dt, int32_t T, int32_t d, int32_t tile_t,
                                           const lx_blocklist* bl);

/*
 * Sparse FFN forward (Sec. VI-B neuron-centric tiled products; forward
 * equations of Sec. II-C with ReLU).  For every listed (token tile i, neuron
 * block j):   H_ij = ReLU(X_i W_up[j,:]^T + b_up[j]);
 *             Y_i  = sum over listed j of H_ij W_down[:, j]^T + b_down.
 *   X      [T,d]   W_up [F,d]   W_down [d,F]   b_up [F] / b_down [d] nullable
 *   bl     rows = T/tile_t, cols = F/blk_n
 *   Y      out [T,d]
 *   H_act  out, compact activations, needed by the backward call; NULL keeps
 *          them in the workspace only.  With gt = (T/tile_t)/bl->rows token
 *          tiles per list row, the block of (tile i, entry k of its row r =
 *          i/gt) is block number row_ptr[r]*gt + k*gt + i%gt of tile_t x blk_n
 *          elements; the buffer holds nnz_cap*gt blocks (gt = 1: [nnz_cap]
 *          blocks in list order).
 * Supported: LX_F32 with (tile_t, blk_n) in {(32,32),(64,64)}, d % 32 == 0;
 *            LX_BF16 / LX_F16 with (64,64), d % 64 == 0.
 */
lx_status lx_sparse_ffn_fwd(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                            int32_t blk_n, const void* X, const void* W_up, const void* b_up,
                            const void* W_down, const void* b_down, const lx_blocklist* bl,
                            void* Y, void* H_act, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * Sparse FFN input gradient (Sec. II-D): for every listed (i, j)
 *   dZ_ij = (dY_i W_down[:, j]) (.) [H_ij > 0];   dX_i = sum_j dZ_ij W_up[j,:].
 *   dY [T,d]; H_act as written by the forward call (same list);
 *   W_up_t [d,F], W_down_t [F,d]: outputs of lx_ffn_pack_weights, or both NULL,
 *   in which case the transposes are rebuilt in the workspace on every call.
 *   dX out [T,d].
 */
lx_status lx_sparse_ffn_bwd_dx(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                               int32_t blk_n, const void* dY, const void* H_act,
                               const void* W_up, const void* W_down, const void* W_up_t,
                               const void* W_down_t, const lx_blocklist* bl, void* dX,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sparse FFN with a LoRA branch on the up-projection (Sec. II-C: z = W x + B A x,
 * a = ReLU(z); Sec. II-D: gradients of the trainable matrices, and no part in the
 * backward pass for what was inactive in the forward pass).  A [r,d] and B [F,r]
 * are handed over zero-padded to rank 64: A_pad [64,d] (rows r.. zero), B_pad
 * [F,64] (columns r.. zero); the padding costs nothing in accuracy and its
 * gradients come out zero.  LX_BF16 / LX_F16, 64 x 64 blocks only.
 *
 * Forward, for every listed (i, j):
 *   U = X A_pad^T [T,64];  H_ij = ReLU(X_i W_up_j^T + U_i B_pad_j^T);  Y_i = sum_j H_ij W_down_j^T
 *   U      out [T,64], needed by the backward call
 *   H_act  out, compact activations as in lx_sparse_ffn_fwd (required)
 *   workspace  >= lx_sparse_ffn_lora_fwd_workspace_bytes(T, d): fp32 partial sums of U when the
 *              product is split over K to fill the chip (few token tiles)
 * Backward:
 *   dZ_ij = (dY_i W_down[:, j]) (.) [H_ij > 0];   G = sum_j dZ_ij B_pad_j  [T,64]
 *   dX_i = sum_j dZ_ij W_up_j + G_i A_pad
 *   dB[j-th 64 rows] = sum_i dZ_ij^T U_i  (fp32 [F,64]; rows of blocks no tile lists are zero)
 *   dA = G^T X  (fp32 [64,d])
 *   W_up_t, W_down_t: outputs of lx_ffn_pack_weights (required here)
 *   workspace  >= lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, nnz_cap) with
 *              nnz_cap counted in activation blocks as for lx_sparse_ffn_bwd_workspace_bytes
 * U, dA and dB are summed over a number of ranges (of K, of token tiles) that depends
 * on the shape only, each range in ascending order and the ranges in a fixed order:
 * results are bit-reproducible.
 */
size_t lx_sparse_ffn_lora_fwd_workspace_bytes(int32_t T, int32_t d);
size_t lx_sparse_ffn_lora_bwd_workspace_bytes(int32_t T, int32_t d, int32_t F, int32_t nnz_cap);
lx_status lx_sparse_ffn_lora_fwd(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                                 int32_t blk_n, const void* X, const void* W_up, const void* A_pad,
                                 const void* B_pad, const void* W_down, const lx_blocklist* bl,
                                 void* Y, void* H_act, void* U, void* workspace,
                                 size_t workspace_bytes, void* stream);
lx_status lx_sparse_ffn_lora_bwd(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                                 int32_t blk_n, const void* X, const void* dY, const void* H_act,
                                 const void* U, const void* W_up_t, const void* W_down_t,
                                 const void* A_pad, const void* B_pad, const lx_blocklist* bl,
                                 void* dX, float* dA, float* dB, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * MLP predictor, inference side (Sec. V-A, "MLP Block"): block scores
 * S = X Wa [T, nblk], binarised with a threshold and reduced over the tokens of
 * a group: mask[g][n] = 1 if S[t][n] > thr for any token t of group g, else 0.
 * group_rows = T gives the paper's single mask reduced over batch and sequence;
 * group_rows = 64 one mask row per token tile.  The mask is what
 * lx_mask_compact takes (rows = T/group_rows, cols = nblk).
 *   X      [T,d]
 *   Wa_t   [nblk,d]: the predictor matrix of the paper ([d, nblk]) transposed,
 *          so that it is read along its contiguous dimension like the weights
 *   mask   out, uint8 [T/group_rows][nblk] (cleared and filled by the call,
 *          no workspace)
 * The comparison is made on fp32 sums of bf16 products; a score within rounding
 * distance of thr may fall on either side.
 * Supported: LX_BF16 / LX_F16, d % 64 == 0, nblk % 64 == 0, T % 64 == 0, group_rows a
 * multiple of 64 that divides T.
 */
lx_status lx_mlp_predict_mask(lx_dtype dt, int32_t T, int32_t d, int32_t nblk, int32_t group_rows,
                              const void* X, const void* Wa_t, float thr, uint8_t* mask,
                              void* stream);

/* Workspace (bytes) for lx_sparse_attn_bwd_dx (the forward call needs none). */
size_t lx_sparse_attn_bwd_workspace_bytes(lx_dtype dt, int32_t B, int32_t Hh, int32_t S,
                                          int32_t D);

/*
 * Block-sparse attention forward (Sec. VI-A: SDD, softmax, DSD over a block
 * list; here fused, the score matrix is never written).  For every batch b,
 * head h with head_active[h] != 0, query row q:
 *   allowed(q) = keys k whose 64x64 block (q/64, k/64) is listed for (b or 0, h)
 *                and, if causal, k <= q  (blocks above the diagonal must not be
 *                listed when causal);
 *   O[q,:] = softmax over allowed(q) of (scale Q[q,:] K[k,:]^T) times V;
 *   LSE[q] = log sum exp of the allowed scaled scores (natural log).
 * Rows with no allowed key and inactive heads give O = 0, LSE = -inf.
 *   Q,K,V,O  [B,Hh,S,D], element (b,h,s,c) at b*strides_bhs[0] + h*strides_bhs[1]
 *            + s*strides_bhs[2] + c (HOST array of 3 element strides, each a
 *            multiple of 8), all four tensors share the strides.
 *   bl       rows = mask_batch*Hh*(S/64) ordered (batch, head, query block);
 *            mask_batch is 1 (mask shared over the batch, Sec. V-A) or B.
 *   head_active  uint8[Hh] or NULL (all heads active)
 *   LSE      out float32 [B,Hh,S] contiguous
 * Supported: LX_BF16 / LX_F16 / LX_F32, D in {64, 128}, S % 64 == 0.  LX_F32 (float tensors,
 * fp32 arithmetic throughout) is the correctness configuration, like the fp32 FFN: plain
 * multiply-adds, not tuned.
 */
lx_status lx_sparse_attn_fwd(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                             float scale, int32_t causal, const void* Q, const void* K,
                             const void* V, const int64_t strides_bhs[3],
                             const lx_blocklist* bl, int32_t mask_batch,
                             const uint8_t* head_active, void* O, float* LSE, void* stream);

/*
 * Block-sparse attention backward over the same blocks (Sec. V-C).  With
 * P = exp(scale Q K^T - LSE) on allowed positions and Delta = rowsum(dO (.) O):
 *   dV = P^T dO;  dS = P (.) (dO V^T - Delta);  dQ = scale dS K;  dK = scale dS^T Q.
 *   dO, O, dQ, dK, dV share the layout and strides of Q.
 *   bl_rows  the forward list;  bl_cols  the same mask column-compressed:
 *            rows = mask_batch*Hh*(S/64) ordered (batch, head, key block),
 *            entries = query blocks.
 *   workspace  >= lx_sparse_attn_bwd_workspace_bytes (holds Delta and a rescaled LSE).
 */
lx_status lx_sparse_attn_bwd_dx(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                                float scale, int32_t causal, const void* Q, const void* K,
                                const void* V, const void* O, const float* LSE, const void* dO,
                                const int64_t strides_bhs[3], const lx_blocklist* bl_rows,
                                const lx_blocklist* bl_cols, int32_t mask_batch,
                                const uint8_t* head_active, void* dQ, void* dK, void* dV,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * lx_sparse_attn_bwd_dx for callers that cannot allocate device memory and have no workspace to
 * hand over (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same computation with Delta and the rescaled LSE kept in a buffer that is part
 * of the library's own device image (2 x 4 MiB per GPU, held until the process ends) instead of
 * a caller's workspace.  The call allocates and frees nothing and calls no allocating routine.
 * Arguments, layouts, results (bit for bit) and errors are those of lx_sparse_attn_bwd_dx, with
 *   LX_ERR_WORKSPACE  if B*Hh*S exceeds 1 048 576 rows, the capacity of that buffer;
 *   LX_ERR_RUNTIME    if the buffer's address on the current device cannot be obtained.
 * All calls on one GPU share the buffer (the current device's copy is used; its contents after a
 * call are unspecified): calls that overlap on one GPU -- different streams, or threads -- race;
 * calls on one stream, or otherwise ordered, do not.
 */
lx_status lx_sparse_attn_bwd_dx_noalloc(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                                        float scale, int32_t causal, const void* Q, const void* K,
                                        const void* V, const void* O, const float* LSE,
                                        const void* dO, const int64_t strides_bhs[3],
                                        const lx_blocklist* bl_rows, const lx_blocklist* bl_cols,
                                        int32_t mask_batch, const uint8_t* head_active, void* dQ,
                                        void* dK, void* dV, void* stream);

/*
 * Measurement aid for benchmarks (no part of the operators of Sec. VI; it lets a
 * harness time one kernel of the path in place).  After lx_profile_begin every
 * launch of `kernel` is bracketed by a pair of HIP events recorded on the
 * launch stream (at most max_launches launches; later ones are not timed).
 * lx_profile_end waits for those events, returns the summed kernel time in
 * milliseconds and the number of timed launches through HOST pointers, and
 * switches the bracketing off.  begin creates events (it allocates; call it
 * outside timed regions); not thread-safe.
 */
lx_status lx_profile_begin(int32_t kernel, int32_t max_launches);
lx_status lx_profile_end(float* total_ms, int32_t* launches);

/*
 * Measurement aids for benchmarks (no part of the operators of Sec. VI): what the chip sustains
 * on the two resources the operators are priced against, so that fractions of a MEASURED peak
 * can be stated next to fractions of the data-sheet one.  Both only enqueue one kernel on
 * `stream`; the caller times it (HIP events on that stream).
 *   lx_probe_mfma_rate    every wavefront of a chip-filling launch issues `iters` rounds of eight
 *                         independent 32x32x16 bf16 MFMAs on registers; *flops (HOST, out) = the
 *                         FLOP of the launch; sink: DEVICE float[1], never written in practice.
 *   lx_probe_stream_copy  dst[0..bytes) = src[0..bytes) with 16-byte accesses (bytes % 16 == 0,
 *                         both pointers 16-byte aligned, buffers must not overlap): the launch
 *                         moves 2 * bytes.
 * Errors: INVALID_ARG for null pointers, iters outside 1 .. 2^24, sizes or alignment as stated.
 */
lx_status lx_probe_mfma_rate(int32_t iters, float* sink, double* flops, void* stream);
lx_status lx_probe_stream_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Tuning knob of the attention kernels (Sec. VI-A leaves the launch shape open).
 * A workgroup walks the block lists of `rows` rows of the mask (query blocks in
 * the forward and dQ kernels, key blocks in the dK/dV kernel) of one (batch,
 * head) as one stream of blocks.  rows = 0 (the default) lets the library
 * choose from the problem size; 1..8 fixes it for all later calls of the
 * calling host thread (the setting is per thread: concurrent callers on other
 * threads keep theirs).  Results do not depend on it: it changes neither the
 * arithmetic of a row nor its order.  Returns LX_ERR_INVALID_ARG outside 0..8.
 */
lx_status lx_attn_set_rows_per_workgroup(int32_t rows);

/*
 * Tuning knob of the 16-bit FFN calls: how many token tiles one workgroup
 * multiplies with the weight rows it has staged.  Two or four tiles (possible
 * when list rows are shared by a multiple of that many consecutive tiles) cut
 * the weight bytes moved per product to 0.6 / 0.4 but also the number of
 * workgroups to a half / a quarter, so they pay for dense or large layers and
 * lose where one tile per workgroup just fills the chip.  tiles = 0 (the
 * default) lets the library choose: the largest group with which the work
 * items -- tile groups x groups of four list entries, counted from the list's
 * capacity nnz_cap -- still number at least one per CU; 1, 2 or 4 asks for at most that many for all later calls
 * of the calling host thread (per-thread setting; the library falls back to 2
 * or 1 where the list rows are not shared accordingly, and always uses 1 in the
 * LoRA calls).  The value governs the second product of a pass; the first
 * product takes that group size or a smaller one, whichever makes its rounds
 * of workgroups (one work item per CU) cheapest by the list's capacity.
 * Results are bit-identical for every value.  Returns LX_ERR_INVALID_ARG for
 * other values.
 */
lx_status lx_ffn_set_token_tiles_per_workgroup(int32_t tiles);

#ifdef __cplusplus
}
#endif
#endif /* LX_H_ */
