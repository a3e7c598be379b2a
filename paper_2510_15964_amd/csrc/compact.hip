// Active-block list compaction (online index-list construction of Sec. VI-A;
// neuron-block index list of Sec. VI-B).
//
// The masks of one layer are tiny (tens of thousands of bytes), so the whole
// job is latency-bound: a 1024-thread workgroup does count -> scan -> scatter
// for a list (or for a part of its rows) in a single launch with no host
// round trip.  One wavefront owns a mask row at
// a time: a 64-wide ballot gives the row's bit pattern, popcount its total and
// mbcnt the rank of every set lane, so columns come out ascending.
#include "lx_dev.h"
#include "lx_launch.h"

namespace lx {

constexpr int kCompactThreads = 1024;
constexpr int kCompactWaves = kCompactThreads / kWave;
constexpr int kChunkRows = 4096;    // rows scanned per pass (4 per thread)
constexpr int kStageBytes = 32768;  // mask bytes staged in LDS per pass

// The mask chunk is first copied into LDS with all loads in flight at once (strided or not),
// because a wavefront that walks rows straight from global memory pays one full memory
// latency per row; the ballots then run out of LDS.

constexpr int kMaxJobs = 8;
struct CompactJobs {
  CompactJob j[kMaxJobs];
};

// Workgroups (blockIdx.x = job, blockIdx.y = part of the job's rows): a launch builds one list,
// the row list and the column list of the same masks, or the lists of several independent masks
// side by side.  A mask of more than kSplitBytes is divided by rows among up to kMaxSplit
// workgroups; a workgroup that does not start at row 0 first counts the active entries of all
// rows before its own (a plain count over bytes it would otherwise wait for another workgroup to
// scan), so the parts need no communication.
constexpr int kSplitBytes = 4096, kMaxSplit = 16;
__host__ __device__ inline int compact_parts(long long total_rows, int cols) {
  long long p = (total_rows * cols + kSplitBytes - 1) / kSplitBytes;
  if (p > kMaxSplit) p = kMaxSplit;
  if (p > total_rows) p = total_rows;
  return p < 1 ? 1 : (int)p;
}

// Walks the flattened (batch, row, column) index space of a job in steps of kCompactThreads
// elements without dividing per element (a 32-bit division costs some forty vector instructions,
// three of them per byte were most of this kernel's time): the position is kept as (batch entry,
// row, column) and advanced with carries.
struct MaskCursor {
  int bi, ri, c;          // batch entry, row inside it, column
  int dbi, dri, dc;       // the step, decomposed the same way
  int rows, cols;
  __device__ __forceinline__ void init(long long first, int rows_, int cols_) {
    rows = rows_;
    cols = cols_;
    const long long gr = first / cols;
    c = (int)(first - gr * cols);
    bi = (int)(gr / rows);
    ri = (int)(gr - (long long)bi * rows);
    const int dr = kCompactThreads / cols;
    dc = kCompactThreads - dr * cols;
    dbi = dr / rows;
    dri = dr - dbi * rows;
  }
  __device__ __forceinline__ void advance() {
    c += dc;
    ri += dri;
    bi += dbi;
    if (c >= cols) {
      c -= cols;
      ++ri;
    }
    if (ri >= rows) {
      ri -= rows;
      ++bi;
    }
  }
  __device__ __forceinline__ long long offset(long long bstride, long long rstride,
                                              long long cstride) const {
    return (long long)bi * bstride + (long long)ri * rstride + (long long)c * cstride;
  }
};

// number of non-zero bytes of a 32-bit word
__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
  const uint32_t t = ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w;   // bit 7 of a byte set <=> byte != 0
  return __popc(t & 0x80808080u);
}

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(const CompactJobs jobs) {
  const CompactJob& job = jobs.j[blockIdx.x];
  const uint8_t* __restrict__ mask = job.mask;
  const int batch = job.batch, rows = job.rows, cols = job.cols, cap = job.cap;
  const long long bstride = job.bstride, rstride = job.rstride, cstride = job.cstride;
  int* __restrict__ row_ptr = job.row_ptr;
  int* __restrict__ col_idx = job.col_idx;
  __shared__ int offs[kChunkRows];
  __shared__ int wave_tot[kCompactWaves];
  __shared__ __attribute__((aligned(16))) uint8_t stage[kStageBytes + 16];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int total_rows = batch * rows;
  const int parts = compact_parts(total_rows, cols), part = blockIdx.y;
  if (part >= parts) return;
  const int per_part = (total_rows + parts - 1) / parts;
  const int row_lo = min(part * per_part, total_rows), row_hi = min(row_lo + per_part, total_rows);
  const bool staged = cols <= kStageBytes;
  const int chunk_rows = staged ? max(1, min(kChunkRows, kStageBytes / cols)) : 1;
  int cp = kWave;                       // columns handled per wave pass (power of two)
  while (cp > 1 && (cp >> 1) >= cols) cp >>= 1;
  const int rpw = kWave / cp;           // rows per wave pass
  const int sub = lane / cp, cl = lane % cp;
  const unsigned long long field = cp == 64 ? ~0ull : ((1ull << cp) - 1ull);
  // all rows of all masks are one contiguous range of bytes, row after row
  const bool rowmajor = cstride == 1 && rstride == cols && (batch == 1 || bstride == (long long)rows * cols);
  int carry = 0;
  if (row_lo > 0) {      // active entries of the rows before this part
    const long long before = (long long)row_lo * cols;
    int cnt = 0;
    // Bytes before this part that are one contiguous range are counted 16 bytes per load: all of
    // them when the rows lie one after the other, else the whole masks before the part when each
    // mask is contiguous in the other orientation; the rest (the rows of the mask the part
    // starts in, masks with other strides) byte by byte below.
    long long done = 0;
    const bool dense = bstride == (long long)rows * cols && rstride == 1 && cstride == rows;
    const long long nbytes = rowmajor ? before
                             : (dense && row_lo >= rows ? (long long)(row_lo / rows) * rows * cols : 0);
    if (nbytes > 0) {
      long long head = (16 - (long long)(reinterpret_cast<uintptr_t>(mask) & 15)) & 15;
      head = head < nbytes ? head : nbytes;
      if (tid < head) cnt += mask[tid] != 0;
      const long long nvec = (nbytes - head) / 16;
      const uint4* __restrict__ vp = reinterpret_cast<const uint4*>(mask + head);
      constexpr int kVec = 4;
      for (long long i0 = tid; i0 < nvec; i0 += (long long)kCompactThreads * kVec) {
        uint4 q[kVec];
#pragma unroll
        for (int u = 0; u < kVec; ++u) {
          const long long i = i0 + (long long)u * kCompactThreads;
          q[u] = i < nvec ? vp[i] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kVec; ++u)
          cnt += nonzero_bytes(q[u].x) + nonzero_bytes(q[u].y) + nonzero_bytes(q[u].z) +
                 nonzero_bytes(q[u].w);
      }
      const long long tail = head + nvec * 16;   // fewer than 16 bytes remain
      if (tail + tid < nbytes) cnt += mask[tail + tid] != 0;
      done = nbytes;
    }
    constexpr int kBatch = 8;
    MaskCursor cur;
    cur.init(done + tid, rows, cols);
    for (long long i0 = done + tid; i0 < before; i0 += (long long)kCompactThreads * kBatch) {
      uint8_t v[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const long long idx = i0 + (long long)u * kCompactThreads;
        v[u] = idx < before ? mask[cur.offset(bstride, rstride, cstride)] : (uint8_t)0;
        cur.advance();
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) cnt += v[u] != 0;
    }
#pragma unroll
    for (int dlt = 32; dlt > 0; dlt >>= 1) cnt += __shfl_xor(cnt, dlt);
    if (lane == 0) wave_tot[wave] = cnt;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kCompactWaves; ++w) carry += wave_tot[w];
    __syncthreads();
  }
  for (int chunk = row_lo; chunk < row_hi; chunk += chunk_rows) {
    const int n = min(chunk_rows, row_hi - chunk);
    int soff = 0;          // where the chunk's first byte sits in `stage`
    if (staged && rowmajor) {
      // a contiguous range: 16 bytes per load, placed so that source and stage are aligned alike
      const uint8_t* __restrict__ src = mask + (long long)chunk * cols;
      const int len = n * cols;
      soff = (int)(reinterpret_cast<uintptr_t>(src) & 15);
      const int head = min((16 - soff) & 15, len);
      if (tid < head) stage[soff + tid] = src[tid];
      const int nvec = (len - head) / 16;
      const uint4* __restrict__ vp = reinterpret_cast<const uint4*>(src + head);
      uint4* sp = reinterpret_cast<uint4*>(stage + soff + head);
      for (int i = tid; i < nvec; i += kCompactThreads) sp[i] = vp[i];
      const int tail = head + nvec * 16;                   // fewer than 16 bytes remain
      if (tail + tid < len) stage[soff + tail + tid] = src[tail + tid];
      __syncthreads();
    } else if (staged) {
      // any strides: byte loads, eight in flight per thread
      constexpr int kBatch = 8;
      MaskCursor cur;
      cur.init((long long)chunk * cols + tid, rows, cols);
      for (int i0 = tid; i0 < n * cols; i0 += kCompactThreads * kBatch) {
        uint8_t v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          v[u] = i0 + u * kCompactThreads < n * cols ? mask[cur.offset(bstride, rstride, cstride)] : (uint8_t)0;
          cur.advance();
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
          if (i0 + u * kCompactThreads < n * cols) stage[i0 + u * kCompactThreads] = v[u];
      }
      __syncthreads();
    }
    auto is_on = [&](int r, int c) -> bool {
      if (c >= cols) return false;
      if (staged) return stage[soff + r * cols + c] != 0;
      const int gr = chunk + r;
      return mask[(long long)(gr / rows) * bstride + (long long)(gr % rows) * rstride +
                  (long long)c * cstride] != 0;
    };
    // 1. per-row counts.  A wavefront covers `rpw` rows at once when rows are short
    //    (cols <= 32): lane l looks at column l % cp of row l / cp, cp = cols rounded up to a
    //    power of two; each row's bits are a cp-wide field of the 64-bit ballot.
    for (int r0 = wave * rpw; r0 < n; r0 += kCompactWaves * rpw) {
      const int r = r0 + sub;
      int cnt = 0;
      for (int c0 = 0; c0 < cols; c0 += cp) {
        const unsigned long long bits = __ballot(r < n && is_on(r, c0 + cl));
        cnt += __popcll((bits >> (sub * cp)) & field);
      }
      if (cl == 0 && r < n) offs[r] = cnt;
    }
    __syncthreads();
    // 2. exclusive scan of the counts (4 consecutive rows per thread)
    int v[4], s = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = tid * 4 + e;
      v[e] = idx < n ? offs[idx] : 0;
      s += v[e];
    }
    int incl = s;
#pragma unroll
    for (int dlt = 1; dlt < kWave; dlt <<= 1) {
      const int up = __shfl_up(incl, dlt);
      if (lane >= dlt) incl += up;
    }
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    int wbase = 0, chunk_total = 0;
#pragma unroll
    for (int w = 0; w < kCompactWaves; ++w) {
      const int t = wave_tot[w];
      if (w < wave) wbase += t;
      chunk_total += t;
    }
    int run = carry + wbase + incl - s;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = tid * 4 + e;
      if (idx < n) {
        offs[idx] = run;
        row_ptr[chunk + idx] = run;
      }
      run += v[e];
    }
    __syncthreads();
    // 3. scatter the ascending column indices
    for (int r0 = wave * rpw; r0 < n; r0 += kCompactWaves * rpw) {
      const int r = r0 + sub;
      int off = r < n ? offs[r] : 0;
      for (int c0 = 0; c0 < cols; c0 += cp) {
        const int c = c0 + cl;
        const bool on = r < n && is_on(r, c);
        const unsigned long long mine = (__ballot(on) >> (sub * cp)) & field;
        const int rank = __popcll(mine & ((1ull << cl) - 1ull));
        if (on && off + rank < cap) col_idx[off + rank] = c;
        off += __popcll(mine);
      }
    }
    carry += chunk_total;
    __syncthreads();
  }
  if (part == parts - 1 && tid == 0) row_ptr[total_rows] = carry;
}

hipError_t launch_compact_jobs(const CompactJob* jobs, int n, hipStream_t stream) {
  CompactJobs js = {};
  int parts = 1;
  for (int i = 0; i < n; ++i) {
    js.j[i] = jobs[i];
    const int p = compact_parts((long long)jobs[i].batch * jobs[i].rows, jobs[i].cols);
    parts = p > parts ? p : parts;
  }
  ProfScope ps(kKCompact, stream);
  hipLaunchKernelGGL(compact_kernel, dim3(n, parts), dim3(kCompactThreads), 0, stream, js);
  return hipGetLastError();
}

hipError_t launch_compact(const uint8_t* mask, int batch, int rows, int cols, long long bs,
                          long long rs, long long cs, int* row_ptr, int* col_idx, int cap,
                          hipStream_t stream) {
  const CompactJob j = {mask, batch, rows, cols, bs, rs, cs, row_ptr, col_idx, cap};
  return launch_compact_jobs(&j, 1, stream);
}

hipError_t launch_compact_pair(const uint8_t* mask, int batch, int rows, int cols, long long bs,
                               long long rs, long long cs, int* row_ptr_r, int* col_idx_r,
                               int* row_ptr_c, int* col_idx_c, int cap, hipStream_t stream) {
  const CompactJob j[2] = {{mask, batch, rows, cols, bs, rs, cs, row_ptr_r, col_idx_r, cap},
                           {mask, batch, cols, rows, bs, cs, rs, row_ptr_c, col_idx_c, cap}};
  return launch_compact_jobs(j, 2, stream);
}

// ---------------------------------------------------------------------------
// Online pattern combination (Sec. VI-A): the list of a multi-head attention
// whose head h carries pattern head_pattern[h] of a pool whose layouts
// (row-compressed lists, the "lookup tables") were computed beforehand.  The
// layout of a head is the layout of its pattern plus an offset: the number of
// blocks of the heads before it.  No mask is read.
// Workgroup (h, list): sums the lengths of the heads before h, then copies row
// pointers (+ offset) and block indices.  Pattern ids outside 0..P-1 give a head
// without blocks.  Entries beyond the capacity of the pool's or the output's
// index buffer are dropped; row_ptr stays exact.
// ---------------------------------------------------------------------------
struct CombineLists {
  CombineList l[2];
};
constexpr int kCombineThreads = 256;

__global__ __launch_bounds__(kCombineThreads) void combine_patterns_kernel(
    const CombineLists lists, const int* __restrict__ head_pattern, int P, int nblk, int n_heads) {
  __shared__ int part[kCombineThreads / kWave];
  const CombineList L = lists.l[blockIdx.y];
  const int h = blockIdx.x, tid = threadIdx.x, lane = tid % kWave;
  auto length = [&](int p) { return p >= 0 && p < P ? L.pool_row_ptr[(p + 1) * nblk] - L.pool_row_ptr[p * nblk] : 0; };
  int off = 0;
  for (int g = tid; g < h; g += kCombineThreads) off += length(head_pattern[g]);
#pragma unroll
  for (int dlt = 32; dlt > 0; dlt >>= 1) off += __shfl_xor(off, dlt);
  if (lane == 0) part[tid / kWave] = off;
  __syncthreads();
  off = 0;
#pragma unroll
  for (int w = 0; w < kCombineThreads / kWave; ++w) off += part[w];

  const int p = head_pattern[h];
  const bool valid = p >= 0 && p < P;
  const int start = valid ? L.pool_row_ptr[p * nblk] : 0;
  const int len = length(p);
  for (int r = tid; r < nblk; r += kCombineThreads)
    L.row_ptr[h * nblk + r] = off + (valid ? L.pool_row_ptr[p * nblk + r] - start : 0);
  if (h == n_heads - 1 && tid == 0) L.row_ptr[n_heads * nblk] = off + len;
  for (int k = tid; k < len; k += kCombineThreads)
    if (off + k < L.cap && start + k < L.pool_cap) L.col_idx[off + k] = L.pool_col_idx[start + k];
}

hipError_t launch_combine_patterns(const CombineList* lists, int n_lists, const int* head_pattern,
                                   int P, int nblk, int n_heads, hipStream_t stream) {
  CombineLists ls = {};
  for (int i = 0; i < n_lists; ++i) ls.l[i] = lists[i];
  ProfScope ps(kKCombine, stream);
  hipLaunchKernelGGL(combine_patterns_kernel, dim3(n_heads, n_lists), dim3(kCombineThreads), 0,
                     stream, ls, head_pattern, P, nblk, n_heads);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Gather of the listed neuron blocks of a neuron-major weight matrix (Sec. VII-B, memory
// footprint: the weights may stay in CPU memory, only the active ones are moved to the GPU).
// W [Fb][block_bytes] -> Wc [entry][block_bytes] in the order of the one-row list; the source
// may be device memory or host memory the device can address.  A unit of work is 1024 16-byte
// words of one entry; at most kGatherGroups workgroups walk the units with a grid stride: reads
// over the host link are bound by the link, a few hundred KB in flight saturate it, and a CU whose
// memory pipeline is waiting on such reads serves the other kernels on it slowly, so the gather
// keeps to a few CUs.  Also writes the list of the compact matrix (row pointers {0, n}, columns
// 0 .. n - 1) when asked to.
// ---------------------------------------------------------------------------
constexpr int kGatherThreads = 256, kGatherU = 4, kGatherGroups = 64;
constexpr int kGatherUnit = kGatherThreads * kGatherU;   // words per unit
__global__ __launch_bounds__(kGatherThreads) void gather_blocks_kernel(
    const uint4* __restrict__ W, int Fb, long long words_per_block, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int cap, uint4* __restrict__ Wc, int* __restrict__ id_row_ptr,
    int* __restrict__ id_col_idx) {
  const int rs = row_ptr[0];
  const int n = max(min(row_ptr[1], cap) - rs, 0);   // entries within the capacity of the list
  if (blockIdx.x == 0) {
    if (id_row_ptr && threadIdx.x < 2) id_row_ptr[threadIdx.x] = threadIdx.x == 0 ? 0 : n;
    if (id_col_idx)
      for (int i = threadIdx.x; i < cap; i += kGatherThreads) id_col_idx[i] = i;
  }
  const long long per_block = (words_per_block + kGatherUnit - 1) / kGatherUnit;
  const long long units = (long long)n * per_block;
  for (long long u = blockIdx.x; u < units; u += gridDim.x) {
    const int e = (int)(u / per_block);
    const long long w0 = (u - (long long)e * per_block) * kGatherUnit + threadIdx.x;
    const int j = col_idx[rs + e];
    if (j < 0 || j >= Fb) continue;                  // not a block of W: nothing is read
    const uint4* __restrict__ src = W + (long long)j * words_per_block;
    uint4* __restrict__ dst = Wc + (long long)e * words_per_block;
    uint4 v[kGatherU];
#pragma unroll
    for (int k = 0; k < kGatherU; ++k)
      if (w0 + k * kGatherThreads < words_per_block) v[k] = src[w0 + k * kGatherThreads];
#pragma unroll
    for (int k = 0; k < kGatherU; ++k)
      if (w0 + k * kGatherThreads < words_per_block) dst[w0 + k * kGatherThreads] = v[k];
  }
}

hipError_t launch_gather_blocks(const void* W, int Fb, long long block_bytes, const int* row_ptr,
                                const int* col_idx, int cap, void* Wc, int* id_row_ptr,
                                int* id_col_idx, hipStream_t stream) {
  const long long words = block_bytes / 16;
  long long groups = (long long)cap * ((words + kGatherUnit - 1) / kGatherUnit);
  groups = groups < 1 ? 1 : (groups > kGatherGroups ? kGatherGroups : groups);
  hipLaunchKernelGGL(gather_blocks_kernel, dim3((unsigned)groups), dim3(kGatherThreads), 0, stream,
                     (const uint4*)W, Fb, words, row_ptr, col_idx, cap, (uint4*)Wc, id_row_ptr,
                     id_col_idx);
  return hipGetLastError();
}

}  // namespace lx
