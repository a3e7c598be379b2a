// Host side of the C ABI declared in include/lx.h: argument validation,
// workspace layout and kernel dispatch.  Nothing here allocates device memory
// or synchronises; every check runs before the first launch so that the error
// paths can be exercised on a machine without a GPU.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <vector>

#include "../../include/lx.h"
#include "lx_launch.h"

namespace lx {

// ---- profiling aid (lx_profile_begin / lx_profile_end) -----------------------------------
static int g_prof_id = -1;
static int g_prof_n = 0;
static std::vector<hipEvent_t> g_prof_start, g_prof_stop;

void prof_pre(int id, hipStream_t st) {
  if (id != g_prof_id || g_prof_n >= (int)g_prof_start.size()) return;
  (void)hipEventRecord(g_prof_start[g_prof_n], st);
}
void prof_post(int id, hipStream_t st) {
  if (id != g_prof_id || g_prof_n >= (int)g_prof_start.size()) return;
  (void)hipEventRecord(g_prof_stop[g_prof_n], st);
  ++g_prof_n;
}
static void prof_clear() {
  for (hipEvent_t e : g_prof_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_prof_stop) (void)hipEventDestroy(e);
  g_prof_start.clear();
  g_prof_stop.clear();
  g_prof_id = -1;
  g_prof_n = 0;
}

// LX_LOG=1: one line per call on stderr (read once; any other value: silent)
static bool log_on() {
  static const bool on = [] {
    const char* v = std::getenv("LX_LOG");
    return v && v[0] == '1';
  }();
  return on;
}
#define LX_LOGF(...)                          \
  do {                                        \
    if (log_on()) {                           \
      std::fprintf(stderr, "[lx] " __VA_ARGS__); \
      std::fputc('\n', stderr);               \
    }                                         \
  } while (0)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline size_t esize(lx_dtype dt) { return dt == LX_F32 ? 4 : 2; }
static inline bool is16(lx_dtype dt) { return dt == LX_BF16 || dt == LX_F16; }
static inline int dt16(lx_dtype dt) { return dt == LX_F16 ? kF16 : kBf16; }   // element type of the 16-bit kernels

static lx_status check_ffn(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                           int32_t blk_n, const lx_blocklist* bl) {
  if (dt != LX_F32 && !is16(dt)) return LX_ERR_UNSUPPORTED;
  if (T <= 0 || d <= 0 || F <= 0 || tile_t <= 0 || blk_n <= 0) return LX_ERR_INVALID_ARG;
  if (dt == LX_F32) {
    if (!((tile_t == 32 && blk_n == 32) || (tile_t == 64 && blk_n == 64))) return LX_ERR_UNSUPPORTED;
    if (d % 32 != 0) return LX_ERR_UNSUPPORTED;
  } else {
    if (!(tile_t == 64 && blk_n == 64)) return LX_ERR_UNSUPPORTED;
    if (d % 64 != 0) return LX_ERR_UNSUPPORTED;
  }
  if (T % tile_t != 0 || F % blk_n != 0) return LX_ERR_UNSUPPORTED;
  if (!bl || !bl->row_ptr || !bl->col_idx) return LX_ERR_INVALID_ARG;
  if (bl->rows <= 0 || (T / tile_t) % bl->rows != 0 || bl->cols != F / blk_n)
    return LX_ERR_INVALID_ARG;
  if (bl->nnz_cap < 0 || (int64_t)bl->nnz_cap > (int64_t)bl->rows * bl->cols) return LX_ERR_INVALID_ARG;
  return LX_OK;
}

// ---- scratch of lx_sparse_attn_bwd_dx_noalloc ---------------------------------------------
// Delta and -LSE*log2(e) of up to kScratchRows (batch, head, token) rows: 2 x 4 MiB that every GPU
// the library runs on holds until the process ends.  `attn_scratch` is a host-side stand-in for
// the array, not a device address: host code uses the per-device address that
// hipGetSymbolAddress returns (each GPU holds its own copy of the array at its own address).
constexpr size_t kScratchRows = (size_t)1 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) float attn_scratch[2 * kScratchRows];
static float* g_scratch_dev[kMaxDevices] = {};
static std::mutex g_scratch_mutex;
// Address of the current device's copy of the array (looked up once per device); allocates nothing.
static hipError_t scratch_of_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_dev[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(attn_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_dev[dev] = (float*)p;
  }
  *out = g_scratch_dev[dev];
  return hipSuccess;
}

static size_t act_bytes(lx_dtype dt, int32_t tile_t, int32_t blk_n, int32_t nnz_cap) {
  return round256((size_t)(nnz_cap > 0 ? nnz_cap : 1) * tile_t * blk_n * esize(dt));
}

}  // namespace lx

using namespace lx;

extern "C" {

const char* lx_status_string(lx_status s) {
  switch (s) {
    case LX_OK: return "LX_OK";
    case LX_ERR_INVALID_ARG: return "LX_ERR_INVALID_ARG";
    case LX_ERR_UNSUPPORTED: return "LX_ERR_UNSUPPORTED";
    case LX_ERR_WORKSPACE: return "LX_ERR_WORKSPACE";
    case LX_ERR_RUNTIME: return "LX_ERR_RUNTIME";
  }
  return "LX_ERR_UNKNOWN";
}

lx_status lx_profile_begin(int32_t kernel, int32_t max_launches) {
  if (kernel < 0 || kernel >= kKCount || max_launches <= 0 || max_launches > (1 << 20))
    return LX_ERR_INVALID_ARG;
  prof_clear();
  g_prof_start.resize(max_launches);
  g_prof_stop.resize(max_launches);
  for (int i = 0; i < max_launches; ++i) {
    if (hipEventCreate(&g_prof_start[i]) != hipSuccess || hipEventCreate(&g_prof_stop[i]) != hipSuccess) {
      g_prof_start.resize(i);
      g_prof_stop.resize(i);
      prof_clear();
      return LX_ERR_RUNTIME;
    }
  }
  g_prof_id = kernel;
  return LX_OK;
}

lx_status lx_profile_end(float* total_ms, int32_t* launches) {
  if (!total_ms || !launches) return LX_ERR_INVALID_ARG;
  if (g_prof_id < 0) return LX_ERR_INVALID_ARG;
  float total = 0.f;
  lx_status rc = LX_OK;
  for (int i = 0; i < g_prof_n; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(g_prof_stop[i]) != hipSuccess ||
        hipEventElapsedTime(&ms, g_prof_start[i], g_prof_stop[i]) != hipSuccess) {
      rc = LX_ERR_RUNTIME;
      break;
    }
    total += ms;
  }
  *total_ms = total;
  *launches = g_prof_n;
  prof_clear();
  return rc;
}

lx_status lx_probe_mfma_rate(int32_t iters, float* sink, double* flops, void* stream) {
  if (iters <= 0 || iters > (1 << 24) || !sink || !flops) return LX_ERR_INVALID_ARG;
  *flops = probe_mfma_flops(iters);
  return launch_probe_mfma(iters, sink, (hipStream_t)stream) == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

lx_status lx_probe_stream_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst))
    return LX_ERR_INVALID_ARG;
  return launch_probe_copy(src, dst, (long long)(bytes / 16), (hipStream_t)stream) == hipSuccess
             ? LX_OK
             : LX_ERR_RUNTIME;
}

lx_status lx_attn_set_rows_per_workgroup(int32_t rows) {
  return set_attn_rows_per_wg(rows) == hipSuccess ? LX_OK : LX_ERR_INVALID_ARG;
}

lx_status lx_ffn_set_token_tiles_per_workgroup(int32_t tiles) {
  return set_ffn_tiles_per_wg(tiles) == hipSuccess ? LX_OK : LX_ERR_INVALID_ARG;
}

static lx_status mask_compact_impl(const uint8_t* mask, int32_t batch, int32_t rows, int32_t cols,
                          int64_t batch_stride, int64_t row_stride, int64_t col_stride,
                          int32_t* row_ptr, int32_t* col_idx, int32_t col_idx_cap, void* stream) {
  if (!mask || !row_ptr || !col_idx) return LX_ERR_INVALID_ARG;
  if (batch <= 0 || rows <= 0 || cols <= 0 || col_idx_cap <= 0) return LX_ERR_INVALID_ARG;
  if ((int64_t)batch * rows > (int64_t)1 << 30) return LX_ERR_INVALID_ARG;
  if (batch_stride < 0 || row_stride < 0 || col_stride < 0) return LX_ERR_INVALID_ARG;
  hipError_t e = launch_compact(mask, batch, rows, cols, batch_stride, row_stride, col_stride,
                                row_ptr, col_idx, col_idx_cap, (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

lx_status lx_mask_compact_pair(const uint8_t* mask, int32_t batch, int32_t rows, int32_t cols,
                               int64_t batch_stride, int64_t row_stride, int64_t col_stride,
                               int32_t* row_ptr_r, int32_t* col_idx_r, int32_t* row_ptr_c,
                               int32_t* col_idx_c, int32_t col_idx_cap, void* stream) {
  if (!mask || !row_ptr_r || !col_idx_r || !row_ptr_c || !col_idx_c) return LX_ERR_INVALID_ARG;
  if (batch <= 0 || rows <= 0 || cols <= 0 || col_idx_cap <= 0) return LX_ERR_INVALID_ARG;
  if ((int64_t)batch * rows > (int64_t)1 << 30 || (int64_t)batch * cols > (int64_t)1 << 30)
    return LX_ERR_INVALID_ARG;
  if (batch_stride < 0 || row_stride < 0 || col_stride < 0) return LX_ERR_INVALID_ARG;
  hipError_t e = launch_compact_pair(mask, batch, rows, cols, batch_stride, row_stride, col_stride,
                                     row_ptr_r, col_idx_r, row_ptr_c, col_idx_c, col_idx_cap,
                                     (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

static lx_status mask_compact_batch_impl(const lx_compact_job* jobs, int32_t n_jobs, void* stream) {
  if (!jobs || n_jobs <= 0 || n_jobs > 8) return LX_ERR_INVALID_ARG;
  CompactJob cj[8];
  for (int i = 0; i < n_jobs; ++i) {
    const lx_compact_job& j = jobs[i];
    if (!j.mask || !j.row_ptr || !j.col_idx) return LX_ERR_INVALID_ARG;
    if (j.batch <= 0 || j.rows <= 0 || j.cols <= 0 || j.col_idx_cap <= 0) return LX_ERR_INVALID_ARG;
    if ((int64_t)j.batch * j.rows > (int64_t)1 << 30) return LX_ERR_INVALID_ARG;
    if (j.batch_stride < 0 || j.row_stride < 0 || j.col_stride < 0) return LX_ERR_INVALID_ARG;
    cj[i] = {j.mask, j.batch, j.rows, j.cols, j.batch_stride, j.row_stride, j.col_stride,
             j.row_ptr, j.col_idx, j.col_idx_cap};
  }
  return launch_compact_jobs(cj, n_jobs, (hipStream_t)stream) == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

lx_status lx_attn_combine_patterns(const lx_blocklist* pool_r, const lx_blocklist* pool_c,
                                   int32_t n_patterns, int32_t nblk, const int32_t* head_pattern,
                                   int32_t n_heads, int32_t* row_ptr_r, int32_t* col_idx_r,
                                   int32_t* row_ptr_c, int32_t* col_idx_c, int32_t col_idx_cap,
                                   void* stream) {
  if (!pool_r || !head_pattern || !row_ptr_r || !col_idx_r) return LX_ERR_INVALID_ARG;
  if (n_patterns <= 0 || nblk <= 0 || n_heads <= 0 || col_idx_cap <= 0) return LX_ERR_INVALID_ARG;
  if ((int64_t)n_patterns * nblk > (int64_t)1 << 30 || (int64_t)n_heads * nblk > (int64_t)1 << 30)
    return LX_ERR_INVALID_ARG;
  const bool with_c = pool_c || row_ptr_c || col_idx_c;
  if (with_c && (!pool_c || !row_ptr_c || !col_idx_c)) return LX_ERR_INVALID_ARG;
  const lx_blocklist* pools[2] = {pool_r, pool_c};
  int32_t* rps[2] = {row_ptr_r, row_ptr_c};
  int32_t* cis[2] = {col_idx_r, col_idx_c};
  CombineList cl[2];
  const int n_lists = with_c ? 2 : 1;
  for (int i = 0; i < n_lists; ++i) {
    const lx_blocklist* pl = pools[i];
    if (!pl->row_ptr || !pl->col_idx || pl->nnz_cap <= 0) return LX_ERR_INVALID_ARG;
    if (pl->rows != n_patterns * nblk || pl->cols != nblk) return LX_ERR_INVALID_ARG;
    cl[i] = {pl->row_ptr, pl->col_idx, pl->nnz_cap, rps[i], cis[i], col_idx_cap};
  }
  return launch_combine_patterns(cl, n_lists, head_pattern, n_patterns, nblk, n_heads,
                                 (hipStream_t)stream) == hipSuccess
             ? LX_OK
             : LX_ERR_RUNTIME;
}

lx_status lx_ffn_pack_weights(lx_dtype dt, int32_t d, int32_t F, const void* W_up,
                              const void* W_down, void* W_up_t, void* W_down_t, void* stream) {
  if (dt != LX_F32 && !is16(dt)) return LX_ERR_UNSUPPORTED;
  if (d <= 0 || F <= 0) return LX_ERR_INVALID_ARG;
  if ((W_up_t && !W_up) || (W_down_t && !W_down)) return LX_ERR_INVALID_ARG;
  if (W_up_t) {
    if (launch_transpose((int)esize(dt), W_up, F, d, W_up_t, (hipStream_t)stream) != hipSuccess)
      return LX_ERR_RUNTIME;
  }
  if (W_down_t) {
    if (launch_transpose((int)esize(dt), W_down, d, F, W_down_t, (hipStream_t)stream) != hipSuccess)
      return LX_ERR_RUNTIME;
  }
  return LX_OK;
}

lx_status lx_ffn_gather_weight_blocks(lx_dtype dt, int32_t d, int32_t F, int32_t blk_n,
                                      const void* W, const lx_blocklist* bl, void* Wc,
                                      int32_t* compact_row_ptr, int32_t* compact_col_idx,
                                      void* stream) {
  if (dt != LX_F32 && !is16(dt)) return LX_ERR_UNSUPPORTED;
  if (d <= 0 || F <= 0 || blk_n <= 0 || F % blk_n != 0) return LX_ERR_INVALID_ARG;
  if (!W || !Wc || !bl || !bl->row_ptr || !bl->col_idx) return LX_ERR_INVALID_ARG;
  if (bl->rows != 1 || bl->cols != F / blk_n || bl->nnz_cap <= 0) return LX_ERR_INVALID_ARG;
  const long long block_bytes = (long long)blk_n * d * (long long)esize(dt);
  if (block_bytes % 16 != 0 || !aligned16(W) || !aligned16(Wc)) return LX_ERR_INVALID_ARG;
  // The kernel reads W through the pointer it is given: only memory the device can address is
  // accepted (device, managed, or host memory allocated pinned); for pinned host memory the
  // device-side alias of the allocation is what the kernel gets.
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, W) != hipSuccess) {
    (void)hipGetLastError();
    return LX_ERR_INVALID_ARG;
  }
  const void* src = W;
  if (at.type == hipMemoryTypeHost) {
    if (!at.devicePointer) return LX_ERR_INVALID_ARG;
    src = at.devicePointer;
  } else if (at.type != hipMemoryTypeDevice && at.type != hipMemoryTypeManaged) {
    return LX_ERR_INVALID_ARG;
  }
  if (launch_gather_blocks(src, F / blk_n, block_bytes, bl->row_ptr, bl->col_idx, bl->nnz_cap, Wc,
                           compact_row_ptr, compact_col_idx, (hipStream_t)stream) != hipSuccess)
    return LX_ERR_RUNTIME;
  return LX_OK;
}

size_t lx_sparse_ffn_fwd_workspace_bytes(lx_dtype dt, int32_t T, int32_t d, int32_t F,
                                         int32_t tile_t, int32_t blk_n, int32_t nnz_cap,
                                         int32_t have_h_act) {
  (void)T; (void)d; (void)F;
  return have_h_act ? 0 : act_bytes(dt, tile_t, blk_n, nnz_cap);
}

size_t lx_sparse_ffn_split_workspace_bytes(lx_dtype dt, int32_t T, int32_t d, int32_t tile_t,
                                          const lx_blocklist* bl) {
  if (!is16(dt) || T <= 0 || d <= 0 || tile_t != 64 || T % 64 != 0 || !bl || bl->rows != 1) return 0;
  return ffn_dsd_split_bytes(T / 64, d, bl->nnz_cap);
}

size_t lx_sparse_ffn_bwd_workspace_bytes(lx_dtype dt, int32_t T, int32_t d, int32_t F,
                                         int32_t tile_t, int32_t blk_n, int32_t nnz_cap,
                                         int32_t have_packed) {
  (void)T;
  size_t b = act_bytes(dt, tile_t, blk_n, nnz_cap);  // dZ_act
  if (!have_packed) b += 2 * round256((size_t)d * F * esize(dt));
  return b;
}

static lx_status ffn_fwd_impl(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                            int32_t blk_n, const void* X, const void* W_up, const void* b_up,
                            const void* W_down, const void* b_down, const lx_blocklist* bl,
                            void* Y, void* H_act, void* workspace, size_t workspace_bytes,
                            void* stream) {
  lx_status s = check_ffn(dt, T, d, F, tile_t, blk_n, bl);
  if (s != LX_OK) return s;
  if (!X || !W_up || !W_down || !Y) return LX_ERR_INVALID_ARG;
  if (!aligned16(X) || !aligned16(W_up) || !aligned16(W_down) || !aligned16(Y) ||
      !aligned16(H_act) || !aligned16(workspace) || !aligned16(b_up) || !aligned16(b_down))
    return LX_ERR_INVALID_ARG;
  const int gt = (T / tile_t) / bl->rows;     // token tiles per list row
  if ((int64_t)bl->nnz_cap * gt > (int64_t)1 << 30) return LX_ERR_INVALID_ARG;
  void* act = H_act;
  size_t used = 0;
  if (!act) {
    const size_t need = lx_sparse_ffn_fwd_workspace_bytes(dt, T, d, F, tile_t, blk_n, bl->nnz_cap * gt, 0);
    if (!workspace || workspace_bytes < need) return LX_ERR_WORKSPACE;
    act = workspace;
    used = need;
  }
  // whatever the workspace holds beyond that may take the partial sums of split lists
  float* part = workspace && workspace_bytes > used ? (float*)((char*)workspace + used) : nullptr;
  const size_t part_bytes = part ? workspace_bytes - used : 0;
  hipError_t e;
  if (dt == LX_F32)
    e = launch_ffn_f32(0, tile_t, T / tile_t, gt, bl->cols, d, F, (const float*)X, (const float*)W_up,
                       (const float*)b_up, (const float*)W_down, (const float*)b_down, bl->row_ptr,
                       bl->col_idx, bl->nnz_cap, (float*)act, nullptr, (float*)Y, (hipStream_t)stream);
  else
    e = launch_ffn_bf16(dt16(dt), 0, T / tile_t, gt, bl->cols, d, F, (const uint16_t*)X, (const uint16_t*)W_up,
                        (const uint16_t*)b_up, (const uint16_t*)W_down, (const uint16_t*)b_down,
                        bl->row_ptr, bl->col_idx, bl->nnz_cap, (uint16_t*)act, nullptr, (uint16_t*)Y,
                        part, part_bytes, (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

static lx_status ffn_bwd_dx_impl(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                               int32_t blk_n, const void* dY, const void* H_act,
                               const void* W_up, const void* W_down, const void* W_up_t,
                               const void* W_down_t, const lx_blocklist* bl, void* dX,
                               void* workspace, size_t workspace_bytes, void* stream) {
  lx_status s = check_ffn(dt, T, d, F, tile_t, blk_n, bl);
  if (s != LX_OK) return s;
  if (!dY || !H_act || !dX) return LX_ERR_INVALID_ARG;
  const bool packed = W_up_t && W_down_t;
  if (!packed && (W_up_t || W_down_t)) return LX_ERR_INVALID_ARG;  // both or neither
  if (!packed && (!W_up || !W_down)) return LX_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(H_act) || !aligned16(dX) || !aligned16(W_up) ||
      !aligned16(W_down) || !aligned16(W_up_t) || !aligned16(W_down_t) || !aligned16(workspace))
    return LX_ERR_INVALID_ARG;
  const int gt = (T / tile_t) / bl->rows;     // token tiles per list row
  if ((int64_t)bl->nnz_cap * gt > (int64_t)1 << 30) return LX_ERR_INVALID_ARG;
  const size_t need = lx_sparse_ffn_bwd_workspace_bytes(dt, T, d, F, tile_t, blk_n,
                                                        bl->nnz_cap * gt, packed ? 1 : 0);
  if (!workspace || workspace_bytes < need) return LX_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  void* dz = ws;
  ws += act_bytes(dt, tile_t, blk_n, bl->nnz_cap * gt);
  hipStream_t st = (hipStream_t)stream;
  if (!packed) {
    void* wut = ws;
    ws += round256((size_t)d * F * esize(dt));
    void* wdt = ws;
    if (launch_transpose((int)esize(dt), W_up, F, d, wut, st) != hipSuccess) return LX_ERR_RUNTIME;
    if (launch_transpose((int)esize(dt), W_down, d, F, wdt, st) != hipSuccess) return LX_ERR_RUNTIME;
    W_up_t = wut;
    W_down_t = wdt;
    ws += round256((size_t)d * F * esize(dt));
  }
  // whatever the workspace holds beyond the query's size may take the partial sums of split lists
  float* part = workspace_bytes > need ? (float*)((char*)workspace + need) : nullptr;
  const size_t part_bytes = part ? workspace_bytes - need : 0;
  hipError_t e;
  if (dt == LX_F32)
    e = launch_ffn_f32(1, tile_t, T / tile_t, gt, bl->cols, d, F, (const float*)dY,
                       (const float*)W_down_t, nullptr, (const float*)W_up_t, nullptr, bl->row_ptr,
                       bl->col_idx, bl->nnz_cap, (float*)dz, (const float*)H_act, (float*)dX, st);
  else
    e = launch_ffn_bf16(dt16(dt), 1, T / tile_t, gt, bl->cols, d, F, (const uint16_t*)dY,
                        (const uint16_t*)W_down_t, nullptr, (const uint16_t*)W_up_t, nullptr,
                        bl->row_ptr, bl->col_idx, bl->nnz_cap, (uint16_t*)dz, (const uint16_t*)H_act,
                        (uint16_t*)dX, part, part_bytes, st);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

size_t lx_sparse_ffn_lora_fwd_workspace_bytes(int32_t T, int32_t d) {
  if (T < 64 || d < 64) return 256;
  const int split = lora_u_split(T / 64, d);
  return 256 + (split > 1 ? round256((size_t)split * T * 64 * 4) : 0);
}

size_t lx_sparse_ffn_lora_bwd_workspace_bytes(int32_t T, int32_t d, int32_t F, int32_t nnz_cap) {
  if (T < 64 || d < 64 || F < 64) return 0;
  const int sa = lora_da_split(T / 64, d), sb = lora_db_split(T / 64, F), sg = lora_g_split(T / 64);
  return act_bytes(LX_BF16, 64, 64, nnz_cap) + round256((size_t)64 * F * 2) +
         round256((size_t)d * 64 * 2) + round256((size_t)T * 64 * 2) +
         (sg > 1 ? round256((size_t)sg * T * 64 * 4) : 0) +
         (sa > 1 ? round256((size_t)sa * 64 * d * 4) : 0) +
         (sb > 1 ? round256((size_t)sb * F * 64 * 4) : 0);
}

static lx_status check_lora(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                            int32_t blk_n, const lx_blocklist* bl) {
  if (!is16(dt)) return LX_ERR_UNSUPPORTED;
  lx_status s = check_ffn(dt, T, d, F, tile_t, blk_n, bl);
  if (s != LX_OK) return s;
  if ((int64_t)bl->nnz_cap * ((T / tile_t) / bl->rows) > (int64_t)1 << 30) return LX_ERR_INVALID_ARG;
  return LX_OK;
}

lx_status lx_sparse_ffn_lora_fwd(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                                 int32_t blk_n, const void* X, const void* W_up, const void* A_pad,
                                 const void* B_pad, const void* W_down, const lx_blocklist* bl,
                                 void* Y, void* H_act, void* U, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  lx_status s = check_lora(dt, T, d, F, tile_t, blk_n, bl);
  if (s != LX_OK) return s;
  if (!X || !W_up || !A_pad || !B_pad || !W_down || !Y || !H_act || !U) return LX_ERR_INVALID_ARG;
  if (!aligned16(X) || !aligned16(W_up) || !aligned16(A_pad) || !aligned16(B_pad) ||
      !aligned16(W_down) || !aligned16(Y) || !aligned16(H_act) || !aligned16(U) ||
      !aligned16(workspace))
    return LX_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < lx_sparse_ffn_lora_fwd_workspace_bytes(T, d)) return LX_ERR_WORKSPACE;
  const int gt = (T / tile_t) / bl->rows;
  hipError_t e = launch_ffn_lora_fwd_bf16(
      dt16(dt), T / 64, gt, d, F, (const uint16_t*)X, (const uint16_t*)W_up, (const uint16_t*)A_pad,
      (const uint16_t*)B_pad, (const uint16_t*)W_down, bl->row_ptr, bl->col_idx, bl->nnz_cap,
      (uint16_t*)U, (uint16_t*)H_act, (uint16_t*)Y, (float*)workspace, (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

lx_status lx_sparse_ffn_lora_bwd(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t,
                                 int32_t blk_n, const void* X, const void* dY, const void* H_act,
                                 const void* U, const void* W_up_t, const void* W_down_t,
                                 const void* A_pad, const void* B_pad, const lx_blocklist* bl,
                                 void* dX, float* dA, float* dB, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  lx_status s = check_lora(dt, T, d, F, tile_t, blk_n, bl);
  if (s != LX_OK) return s;
  if (!X || !dY || !H_act || !U || !W_up_t || !W_down_t || !A_pad || !B_pad || !dX || !dA || !dB)
    return LX_ERR_INVALID_ARG;
  if (!aligned16(X) || !aligned16(dY) || !aligned16(H_act) || !aligned16(U) || !aligned16(W_up_t) ||
      !aligned16(W_down_t) || !aligned16(A_pad) || !aligned16(B_pad) || !aligned16(dX) ||
      !aligned16(dA) || !aligned16(dB) || !aligned16(workspace))
    return LX_ERR_INVALID_ARG;
  const int gt = (T / tile_t) / bl->rows;
  const size_t need = lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, bl->nnz_cap * gt);
  if (!workspace || workspace_bytes < need) return LX_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  uint16_t* dz = (uint16_t*)ws;
  ws += act_bytes(LX_BF16, 64, 64, bl->nnz_cap * gt);
  uint16_t* bt = (uint16_t*)ws;
  ws += round256((size_t)64 * F * 2);
  uint16_t* at = (uint16_t*)ws;
  ws += round256((size_t)d * 64 * 2);
  uint16_t* g = (uint16_t*)ws;
  ws += round256((size_t)T * 64 * 2);
  float* part_g = (float*)ws;
  const int sg = lora_g_split(T / 64);
  if (sg > 1) ws += round256((size_t)sg * T * 64 * 4);
  float* part_a = (float*)ws;
  const int sa = lora_da_split(T / 64, d);
  if (sa > 1) ws += round256((size_t)sa * 64 * d * 4);
  float* part_b = (float*)ws;
  hipError_t e = launch_ffn_lora_bwd_bf16(
      dt16(dt), T / 64, gt, d, F, (const uint16_t*)X, (const uint16_t*)dY, (const uint16_t*)H_act,
      (const uint16_t*)U, (const uint16_t*)W_down_t, (const uint16_t*)W_up_t,
      (const uint16_t*)A_pad, (const uint16_t*)B_pad, bl->row_ptr, bl->col_idx, bl->nnz_cap, dz, bt,
      at, g, part_g, part_a, part_b, (uint16_t*)dX, dA, dB, (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

lx_status lx_mlp_predict_mask(lx_dtype dt, int32_t T, int32_t d, int32_t nblk, int32_t group_rows,
                              const void* X, const void* Wa_t, float thr, uint8_t* mask,
                              void* stream) {
  if (!is16(dt)) return LX_ERR_UNSUPPORTED;
  if (T <= 0 || d <= 0 || nblk <= 0 || group_rows <= 0) return LX_ERR_INVALID_ARG;
  if (T % 64 != 0 || d % 64 != 0 || nblk % 64 != 0) return LX_ERR_UNSUPPORTED;
  if (group_rows % 64 != 0 || T % group_rows != 0) return LX_ERR_INVALID_ARG;
  if (!X || !Wa_t || !mask || !aligned16(X) || !aligned16(Wa_t)) return LX_ERR_INVALID_ARG;
  if (thr != thr) return LX_ERR_INVALID_ARG;   // NaN
  if (2ll * nblk * d >= (1ll << 31) || (int64_t)(T / 64) * nblk >= (1ll << 31))
    return LX_ERR_INVALID_ARG;
  return launch_predict_bf16(dt16(dt), T, d, nblk, group_rows / 64, (const uint16_t*)X, (const uint16_t*)Wa_t,
                             thr, mask, (hipStream_t)stream) == hipSuccess
             ? LX_OK
             : LX_ERR_RUNTIME;
}

size_t lx_sparse_attn_bwd_workspace_bytes(lx_dtype dt, int32_t B, int32_t Hh, int32_t S,
                                          int32_t D) {
  (void)dt; (void)D;
  if (B <= 0 || Hh <= 0 || S <= 0) return 0;
  return 2 * round256((size_t)B * Hh * S * sizeof(float));   // Delta and -LSE*log2(e)
}

static lx_status check_attn(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                            const int64_t strides[3], const lx_blocklist* bl, int32_t mask_batch) {
  if (!is16(dt) && dt != LX_F32) return LX_ERR_UNSUPPORTED;
  if (B <= 0 || Hh <= 0 || S <= 0 || D <= 0) return LX_ERR_INVALID_ARG;
  if (D != 64 && D != 128) return LX_ERR_UNSUPPORTED;
  if (S % 64 != 0) return LX_ERR_UNSUPPORTED;
  if (B > 65535 || Hh > 65535) return LX_ERR_UNSUPPORTED;
  if (!strides) return LX_ERR_INVALID_ARG;
  for (int i = 0; i < 3; ++i)
    if (strides[i] < 0 || strides[i] % 8 != 0) return LX_ERR_INVALID_ARG;
  if (strides[2] < D) return LX_ERR_INVALID_ARG;
  if (mask_batch != 1 && mask_batch != B) return LX_ERR_INVALID_ARG;
  if (!bl || !bl->row_ptr || !bl->col_idx) return LX_ERR_INVALID_ARG;
  if ((int64_t)bl->rows != (int64_t)mask_batch * Hh * (S / 64) || bl->cols != S / 64)
    return LX_ERR_INVALID_ARG;
  return LX_OK;
}

static lx_status attn_fwd_impl(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                             float scale, int32_t causal, const void* Q, const void* K,
                             const void* V, const int64_t strides_bhs[3],
                             const lx_blocklist* bl, int32_t mask_batch,
                             const uint8_t* head_active, void* O, float* LSE, void* stream) {
  lx_status s = check_attn(dt, B, Hh, S, D, strides_bhs, bl, mask_batch);
  if (s != LX_OK) return s;
  if (!Q || !K || !V || !O || !LSE) return LX_ERR_INVALID_ARG;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return LX_ERR_INVALID_ARG;
  AttnArgs a = {};
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
  a.Out = (uint16_t*)O; a.LSE = LSE;
  a.sb = strides_bhs[0]; a.sh = strides_bhs[1]; a.ss = strides_bhs[2];
  a.row_ptr = bl->row_ptr; a.col_idx = bl->col_idx; a.nnz_cap = bl->nnz_cap;
  a.head_active = head_active;
  a.Hh = Hh; a.S = S; a.mask_batch = mask_batch; a.causal = causal ? 1 : 0; a.scale = scale;
  const hipError_t e = dt == LX_F32 ? launch_attn_fwd_f32(D, B, a, (hipStream_t)stream)
                                    : launch_attn_fwd_bf16(dt16(dt), D, B, a, (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

// Shared by the two backward entry points: everything but where Delta and -LSE*log2(e) live.
static lx_status attn_bwd_check(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                                const void* Q, const void* K, const void* V, const void* O,
                                const float* LSE, const void* dO, const int64_t strides_bhs[3],
                                const lx_blocklist* bl_rows, const lx_blocklist* bl_cols,
                                int32_t mask_batch, void* dQ, void* dK, void* dV) {
  lx_status s = check_attn(dt, B, Hh, S, D, strides_bhs, bl_rows, mask_batch);
  if (s != LX_OK) return s;
  s = check_attn(dt, B, Hh, S, D, strides_bhs, bl_cols, mask_batch);
  if (s != LX_OK) return s;
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV) return LX_ERR_INVALID_ARG;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
    return LX_ERR_INVALID_ARG;
  return LX_OK;
}
static lx_status attn_bwd_run(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D, float scale,
                              int32_t causal, const void* Q, const void* K, const void* V,
                              const void* O, const float* LSE, const void* dO,
                              const int64_t strides_bhs[3], const lx_blocklist* bl_rows,
                              const lx_blocklist* bl_cols, int32_t mask_batch,
                              const uint8_t* head_active, void* dQ, void* dK, void* dV,
                              float* delta, float* neg_lse2, void* stream) {
  AttnArgs a = {};
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
  a.O = (const uint16_t*)O; a.dO = (const uint16_t*)dO; a.LSEin = LSE;
  a.dQ = (uint16_t*)dQ; a.dK = (uint16_t*)dK; a.dV = (uint16_t*)dV;
  a.Delta = delta;
  a.NegLse2 = neg_lse2;
  a.sb = strides_bhs[0]; a.sh = strides_bhs[1]; a.ss = strides_bhs[2];
  a.row_ptr = bl_rows->row_ptr; a.col_idx = bl_rows->col_idx; a.nnz_cap = bl_rows->nnz_cap;
  a.crow_ptr = bl_cols->row_ptr; a.ccol_idx = bl_cols->col_idx; a.cnnz_cap = bl_cols->nnz_cap;
  a.head_active = head_active;
  a.Hh = Hh; a.S = S; a.mask_batch = mask_batch; a.causal = causal ? 1 : 0; a.scale = scale;
  const hipError_t e = dt == LX_F32 ? launch_attn_bwd_f32(D, B, a, (hipStream_t)stream)
                                    : launch_attn_bwd_bf16(dt16(dt), D, B, a, (hipStream_t)stream);
  return e == hipSuccess ? LX_OK : LX_ERR_RUNTIME;
}

static lx_status attn_bwd_dx_impl(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                                float scale, int32_t causal, const void* Q, const void* K,
                                const void* V, const void* O, const float* LSE, const void* dO,
                                const int64_t strides_bhs[3], const lx_blocklist* bl_rows,
                                const lx_blocklist* bl_cols, int32_t mask_batch,
                                const uint8_t* head_active, void* dQ, void* dK, void* dV,
                                void* workspace, size_t workspace_bytes, void* stream) {
  lx_status s = attn_bwd_check(dt, B, Hh, S, D, Q, K, V, O, LSE, dO, strides_bhs, bl_rows, bl_cols,
                               mask_batch, dQ, dK, dV);
  if (s != LX_OK) return s;
  if (!aligned16(workspace)) return LX_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < lx_sparse_attn_bwd_workspace_bytes(dt, B, Hh, S, D))
    return LX_ERR_WORKSPACE;
  float* delta = (float*)workspace;
  float* neg_lse2 = (float*)((char*)workspace + round256((size_t)B * Hh * S * sizeof(float)));
  return attn_bwd_run(dt, B, Hh, S, D, scale, causal, Q, K, V, O, LSE, dO, strides_bhs, bl_rows,
                      bl_cols, mask_batch, head_active, dQ, dK, dV, delta, neg_lse2, stream);
}

static lx_status attn_bwd_dx_noalloc_impl(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D,
                                        float scale, int32_t causal, const void* Q, const void* K,
                                        const void* V, const void* O, const float* LSE,
                                        const void* dO, const int64_t strides_bhs[3],
                                        const lx_blocklist* bl_rows, const lx_blocklist* bl_cols,
                                        int32_t mask_batch, const uint8_t* head_active, void* dQ,
                                        void* dK, void* dV, void* stream) {
  lx_status s = attn_bwd_check(dt, B, Hh, S, D, Q, K, V, O, LSE, dO, strides_bhs, bl_rows, bl_cols,
                               mask_batch, dQ, dK, dV);
  if (s != LX_OK) return s;
  const size_t rows = (size_t)B * Hh * S;
  if (rows > kScratchRows) return LX_ERR_WORKSPACE;   // beyond the library's own scratch
  float* scratch = nullptr;
  if (scratch_of_current_device(&scratch) != hipSuccess) {
    (void)hipGetLastError();
    return LX_ERR_RUNTIME;
  }
  // both halves are written in full by the query-side kernel before the key-side kernel reads
  // them: nothing of an earlier call is read, nothing has to be cleared
  return attn_bwd_run(dt, B, Hh, S, D, scale, causal, Q, K, V, O, LSE, dO, strides_bhs, bl_rows,
                      bl_cols, mask_batch, head_active, dQ, dK, dV, scratch, scratch + kScratchRows,
                      stream);
}

lx_status lx_sparse_ffn_fwd(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t, int32_t blk_n, const void* X, const void* W_up, const void* b_up, const void* W_down, const void* b_down, const lx_blocklist* bl, void* Y, void* H_act, void* workspace, size_t workspace_bytes, void* stream) {
  const lx_status s = ffn_fwd_impl(dt, T, d, F, tile_t, blk_n, X, W_up, b_up, W_down, b_down, bl, Y, H_act, workspace, workspace_bytes, stream);
  LX_LOGF("lx_sparse_ffn_fwd dt=%d T=%d d=%d F=%d tile=%dx%d list rows=%d nnz_cap=%d ws=%zu -> %s", (int)dt, T, d, F, tile_t, blk_n, bl ? bl->rows : -1, bl ? bl->nnz_cap : -1, workspace_bytes, lx_status_string(s));
  return s;
}

lx_status lx_sparse_ffn_bwd_dx(lx_dtype dt, int32_t T, int32_t d, int32_t F, int32_t tile_t, int32_t blk_n, const void* dY, const void* H_act, const void* W_up, const void* W_down, const void* W_up_t, const void* W_down_t, const lx_blocklist* bl, void* dX, void* workspace, size_t workspace_bytes, void* stream) {
  const lx_status s = ffn_bwd_dx_impl(dt, T, d, F, tile_t, blk_n, dY, H_act, W_up, W_down, W_up_t, W_down_t, bl, dX, workspace, workspace_bytes, stream);
  LX_LOGF("lx_sparse_ffn_bwd_dx dt=%d T=%d d=%d F=%d tile=%dx%d list rows=%d nnz_cap=%d packed=%d ws=%zu -> %s", (int)dt, T, d, F, tile_t, blk_n, bl ? bl->rows : -1, bl ? bl->nnz_cap : -1, (int)(W_up_t && W_down_t), workspace_bytes, lx_status_string(s));
  return s;
}

lx_status lx_sparse_attn_fwd(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D, float scale, int32_t causal, const void* Q, const void* K, const void* V, const int64_t strides_bhs[3], const lx_blocklist* bl, int32_t mask_batch, const uint8_t* head_active, void* O, float* LSE, void* stream) {
  const lx_status s = attn_fwd_impl(dt, B, Hh, S, D, scale, causal, Q, K, V, strides_bhs, bl, mask_batch, head_active, O, LSE, stream);
  LX_LOGF("lx_sparse_attn_fwd dt=%d B=%d Hh=%d S=%d D=%d causal=%d mask_batch=%d nnz_cap=%d -> %s", (int)dt, B, Hh, S, D, causal, mask_batch, bl ? bl->nnz_cap : -1, lx_status_string(s));
  return s;
}

lx_status lx_sparse_attn_bwd_dx(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D, float scale, int32_t causal, const void* Q, const void* K, const void* V, const void* O, const float* LSE, const void* dO, const int64_t strides_bhs[3], const lx_blocklist* bl_rows, const lx_blocklist* bl_cols, int32_t mask_batch, const uint8_t* head_active, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, void* stream) {
  const lx_status s = attn_bwd_dx_impl(dt, B, Hh, S, D, scale, causal, Q, K, V, O, LSE, dO, strides_bhs, bl_rows, bl_cols, mask_batch, head_active, dQ, dK, dV, workspace, workspace_bytes, stream);
  LX_LOGF("lx_sparse_attn_bwd_dx dt=%d B=%d Hh=%d S=%d D=%d causal=%d mask_batch=%d ws=%zu -> %s", (int)dt, B, Hh, S, D, causal, mask_batch, workspace_bytes, lx_status_string(s));
  return s;
}

lx_status lx_sparse_attn_bwd_dx_noalloc(lx_dtype dt, int32_t B, int32_t Hh, int32_t S, int32_t D, float scale, int32_t causal, const void* Q, const void* K, const void* V, const void* O, const float* LSE, const void* dO, const int64_t strides_bhs[3], const lx_blocklist* bl_rows, const lx_blocklist* bl_cols, int32_t mask_batch, const uint8_t* head_active, void* dQ, void* dK, void* dV, void* stream) {
  const lx_status s = attn_bwd_dx_noalloc_impl(dt, B, Hh, S, D, scale, causal, Q, K, V, O, LSE, dO, strides_bhs, bl_rows, bl_cols, mask_batch, head_active, dQ, dK, dV, stream);
  LX_LOGF("lx_sparse_attn_bwd_dx_noalloc dt=%d B=%d Hh=%d S=%d D=%d causal=%d mask_batch=%d -> %s", (int)dt, B, Hh, S, D, causal, mask_batch, lx_status_string(s));
  return s;
}

lx_status lx_mask_compact_batch(const lx_compact_job* jobs, int32_t n_jobs, void* stream) {
  const lx_status s = mask_compact_batch_impl(jobs, n_jobs, stream);
  LX_LOGF("lx_mask_compact_batch jobs=%d -> %s", n_jobs, lx_status_string(s));
  return s;
}

lx_status lx_mask_compact(const uint8_t* mask, int32_t batch, int32_t rows, int32_t cols, int64_t batch_stride, int64_t row_stride, int64_t col_stride, int32_t* row_ptr, int32_t* col_idx, int32_t col_idx_cap, void* stream) {
  const lx_status s = mask_compact_impl(mask, batch, rows, cols, batch_stride, row_stride, col_stride, row_ptr, col_idx, col_idx_cap, stream);
  LX_LOGF("lx_mask_compact batch=%d rows=%d cols=%d cap=%d -> %s", batch, rows, cols, col_idx_cap, lx_status_string(s));
  return s;
}

}  // extern "C"
