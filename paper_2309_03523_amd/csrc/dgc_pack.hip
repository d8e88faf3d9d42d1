// Chunk-fusion packing on the device (Section 5.1.1 of the paper: the chunks assigned to a
// GPU are loaded and executed together, and a vertex that another chunk depends on is loaded
// once).  Integer kernels only: segment bounds, the de-duplicated halo list of every segment
// (a bitmap over vertex ids per segment, ranked by a prefix sum of its popcounts), local
// column ids, the list of split rows, and the per-row degree scaling.
#include "dgc_internal.h"

namespace dgc {

namespace {

constexpr int kBlock = 256;

__device__ __forceinline__ int64_t find_segment_by_nnz(const Segment* segs, int64_t nseg, int64_t p) {
  int64_t lo = 0, hi = nseg - 1;  // largest s with segs[s].nnz_off <= p
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) >> 1;
    if (segs[mid].nnz_off <= p) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__device__ __forceinline__ int64_t find_segment_by_row(const Segment* segs, int64_t nseg, int64_t q) {
  int64_t lo = 0, hi = nseg - 1;
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) >> 1;
    if (segs[mid].row_off <= q) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__global__ void k_segment_bounds(GraphDev g, Segment* segs, int64_t nseg) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= nseg) return;
  const int64_t* rp = g.rowptr[segs[s].t];
  const int64_t e0 = rp[segs[s].v_lo];
  segs[s].e0 = e0;
  segs[s].nnz_off = rp[segs[s].v_hi] - e0;  // the host turns the counts into offsets
}

__global__ void k_deg_inv_sqrt(GraphDev g, float* dinv) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)g.T * g.N) return;
  const int64_t t = idx / g.N, i = idx - t * g.N;
  const int64_t* rp = g.rowptr[t];
  const int64_t d = rp[i + 1] - rp[i];
  dinv[idx] = d > 0 ? 1.0f / sqrtf((float)d) : 0.0f;
}

// Also the one place where every column a later kernel will follow is range-checked.
__global__ void k_mark_halo(GraphDev g, const Segment* segs, int64_t nseg, int64_t total_nnz,
                            int64_t wps, uint32_t* bitmap, int32_t* flags) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= total_nnz) return;
  const int64_t s = find_segment_by_nnz(segs, nseg, p);
  const Segment sg = segs[s];
  const int32_t j = g.colidx[sg.t][sg.e0 + (p - sg.nnz_off)];
  if (j < 0 || j >= g.N) { atomicOr(&flags[1], 1); return; }
  if (j < sg.v_lo || j >= sg.v_hi) {
    atomicOr(&bitmap[s * wps + (j >> 5)], 1u << (j & 31));
  }
}

// rowptr starts at 0 and never decreases: with that, every row's range lies inside colidx.
__global__ void k_validate_rowptr(GraphDev g, int32_t* flags) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)g.T * g.N) return;
  const int64_t t = idx / g.N, i = idx - t * g.N;
  const int64_t* rp = g.rowptr[t];
  if ((i == 0 && rp[0] != 0) || rp[i + 1] < rp[i]) atomicOr(&flags[0], 1);
}

__global__ void k_popcount_words(const uint32_t* bitmap, int64_t n_words, int64_t* counts) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) counts[i] = __popc(bitmap[i]);
}

// ---- exclusive scan of int64, 2048 items per block
constexpr int kScanItems = 8;
constexpr int kScanTile = kBlock * kScanItems;

__device__ __forceinline__ int64_t block_exclusive_scan(int64_t v, int64_t* total) {
  // exclusive scan of one value per thread over a block of kBlock threads
  __shared__ int64_t wave_sums[kBlock / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int64_t incl = v;
  for (int d = 1; d < kWave; d <<= 1) {
    const int64_t up = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += up;
  }
  if (lane == kWave - 1) wave_sums[wave] = incl;
  __syncthreads();
  int64_t base = 0, tot = 0;
  for (int w = 0; w < kBlock / kWave; ++w) {
    if (w < wave) base += wave_sums[w];
    tot += wave_sums[w];
  }
  __syncthreads();
  *total = tot;
  return base + incl - v;
}

__global__ void k_scan_block_sums(const int64_t* data, int64_t n, int64_t* block_sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int64_t s = 0;
  for (int k = 0; k < kScanItems; ++k)
    if (base + k < n) s += data[base + k];
  int64_t tot;
  block_exclusive_scan(s, &tot);
  if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

__global__ void k_scan_sums(int64_t* block_sums, int64_t n_blocks, int64_t* total_dev) {
  // one block; walks the block sums in slabs of kBlock with a running carry
  int64_t carry = 0;
  for (int64_t b0 = 0; b0 < n_blocks; b0 += kBlock) {
    const int64_t i = b0 + threadIdx.x;
    const int64_t v = i < n_blocks ? block_sums[i] : 0;
    int64_t tot;
    const int64_t ex = block_exclusive_scan(v, &tot);
    if (i < n_blocks) block_sums[i] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) *total_dev = carry;
}

__global__ void k_scan_apply(int64_t* data, int64_t n, const int64_t* block_sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int64_t v[kScanItems];
  int64_t s = 0;
  for (int k = 0; k < kScanItems; ++k) {
    v[k] = base + k < n ? data[base + k] : 0;
    s += v[k];
  }
  int64_t tot;
  int64_t run = block_sums[blockIdx.x] + block_exclusive_scan(s, &tot);
  for (int k = 0; k < kScanItems; ++k) {
    if (base + k < n) data[base + k] = run;
    run += v[k];
  }
}

__global__ void k_fill_halo(const uint32_t* bitmap, const int64_t* word_rank, int64_t n_words,
                            int64_t wps, int32_t* halo_idx) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_words) return;
  uint32_t w = bitmap[i];
  if (!w) return;
  int64_t dst = word_rank[i];
  const int32_t base = (int32_t)((i % wps) << 5);
  while (w) {
    const int b = __ffs(w) - 1;
    halo_idx[dst++] = base + b;
    w &= w - 1;
  }
}

__global__ void k_seg_halo_off(const int64_t* word_rank, int64_t nseg, int64_t wps, int64_t total_words,
                               const int64_t* total_dev, Segment* segs, int64_t* halo_ptr) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s > nseg) return;
  const int64_t v = (s == nseg || s * wps >= total_words) ? *total_dev : word_rank[s * wps];
  halo_ptr[s] = v;
  if (s < nseg) segs[s].halo_off = v;
}

__global__ void k_col_local(GraphDev g, const Segment* segs, int64_t nseg, int64_t total_nnz, int64_t wps,
                            const uint32_t* bitmap, const int64_t* word_rank, int32_t* col_local) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= total_nnz) return;
  const int64_t s = find_segment_by_nnz(segs, nseg, p);
  const Segment sg = segs[s];
  const int32_t j = g.colidx[sg.t][sg.e0 + (p - sg.nnz_off)];
  int32_t out;
  if (j < 0 || j >= g.N) {
    out = -1;  // reported by k_mark_halo; never followed
  } else if (j >= sg.v_lo && j < sg.v_hi) {
    out = (int32_t)(j - sg.v_lo);
  } else {
    const int64_t w = s * wps + (j >> 5);
    const int64_t rank = word_rank[w] - sg.halo_off + __popc(bitmap[w] & ((1u << (j & 31)) - 1u));
    out = (int32_t)(sg.v_hi - sg.v_lo + rank);
  }
  col_local[p] = out;
}

__global__ void k_long_count(GraphDev g, const Segment* segs, int64_t nseg, int64_t total_rows,
                             int32_t long_nnz, int32_t part_nnz, int64_t* counts) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= total_rows) return;
  const int64_t s = find_segment_by_row(segs, nseg, q);
  const int64_t i = segs[s].v_lo + (q - segs[s].row_off);
  const int64_t* rp = g.rowptr[segs[s].t];
  const int64_t nnz = rp[i + 1] - rp[i];
  counts[q] = nnz > long_nnz ? (nnz + part_nnz - 1) / part_nnz : 0;
}

__global__ void k_long_fill(GraphDev g, const Segment* segs, int64_t nseg, int64_t total_rows,
                            int32_t long_nnz, int32_t part_nnz, const int64_t* offs, int32_t* work_long) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= total_rows) return;
  const int64_t s = find_segment_by_row(segs, nseg, q);
  const int64_t i = segs[s].v_lo + (q - segs[s].row_off);
  const int64_t* rp = g.rowptr[segs[s].t];
  const int64_t nnz = rp[i + 1] - rp[i];
  if (nnz <= long_nnz) return;
  const int64_t parts = (nnz + part_nnz - 1) / part_nnz;
  int32_t* dst = work_long + 4 * offs[q];
  for (int64_t p = 0; p < parts; ++p) {
    dst[4 * p + 0] = (int32_t)s;
    dst[4 * p + 1] = (int32_t)(i - segs[s].v_lo);
    dst[4 * p + 2] = (int32_t)p;
    dst[4 * p + 3] = (int32_t)parts;
  }
}

// flags[0]: rowptr not starting at 0 / decreasing; [1]: column out of range or not strictly
// ascending; [2]: self-loop missing; [3]: (i,j) stored without (j,i).
__global__ void k_validate_graph(GraphDev g, int32_t* flags) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)g.T * g.N) return;
  const int64_t t = idx / g.N, i = idx - t * g.N;
  const int64_t* rp = g.rowptr[t];
  const int32_t* cj = g.colidx[t];
  if (i == 0 && rp[0] != 0) atomicOr(&flags[0], 1);
  const int64_t a = rp[i], b = rp[i + 1];
  if (b < a || a < 0) { atomicOr(&flags[0], 1); return; }
  bool self = false;
  int64_t prev = -1;
  for (int64_t e = a; e < b; ++e) {
    const int64_t j = cj[e];
    if (j < 0 || j >= g.N || j <= prev) { atomicOr(&flags[1], 1); return; }
    prev = j;
    if (j == i) { self = true; continue; }
    int64_t lo = rp[j], hi = rp[j + 1];  // binary search i in row j
    if (hi < lo || lo < 0) { atomicOr(&flags[0], 1); return; }
    bool found = false;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      const int64_t c = cj[mid];
      if (c == i) { found = true; break; }
      if (c < i) lo = mid + 1; else hi = mid;
    }
    if (!found) atomicOr(&flags[3], 1);
  }
  if (!self) atomicOr(&flags[2], 1);
}

inline unsigned grid_for(int64_t n, int per_block = kBlock) {
  return (unsigned)((n + per_block - 1) / per_block);
}

}  // namespace

void launch_segment_bounds(const GraphDev& g, Segment* segs, int64_t nseg, hipStream_t st) {
  if (nseg > 0) hipLaunchKernelGGL(k_segment_bounds, grid_for(nseg), kBlock, 0, st, g, segs, nseg);
}

void launch_deg_inv_sqrt(const GraphDev& g, float* dinv, hipStream_t st) {
  const int64_t n = (int64_t)g.T * g.N;
  if (n > 0) hipLaunchKernelGGL(k_deg_inv_sqrt, grid_for(n), kBlock, 0, st, g, dinv);
}

void launch_mark_halo(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_nnz,
                      int64_t words_per_seg, uint32_t* bitmap, int32_t* flags, hipStream_t st) {
  if (total_nnz > 0)
    hipLaunchKernelGGL(k_mark_halo, grid_for(total_nnz), kBlock, 0, st, g, segs, nseg, total_nnz,
                       words_per_seg, bitmap, flags);
}

void launch_validate_rowptr(const GraphDev& g, int32_t* flags, hipStream_t st) {
  const int64_t n = (int64_t)g.T * g.N;
  if (n > 0) hipLaunchKernelGGL(k_validate_rowptr, grid_for(n), kBlock, 0, st, g, flags);
}

void launch_popcount_words(const uint32_t* bitmap, int64_t n_words, int64_t* counts, hipStream_t st) {
  if (n_words > 0) hipLaunchKernelGGL(k_popcount_words, grid_for(n_words), kBlock, 0, st, bitmap, n_words, counts);
}

int64_t scan_tmp_elems(int64_t n) { return (n + kScanTile - 1) / kScanTile + 2; }

void launch_exclusive_scan(int64_t* data, int64_t n, int64_t* tmp, int64_t* total_dev, hipStream_t st) {
  const int64_t nb = (n + kScanTile - 1) / kScanTile;
  if (nb > 0) hipLaunchKernelGGL(k_scan_block_sums, (unsigned)nb, kBlock, 0, st, data, n, tmp);
  hipLaunchKernelGGL(k_scan_sums, 1, kBlock, 0, st, tmp, nb, total_dev);
  if (nb > 0) hipLaunchKernelGGL(k_scan_apply, (unsigned)nb, kBlock, 0, st, data, n, tmp);
}

void launch_fill_halo(const uint32_t* bitmap, const int64_t* word_rank, int64_t nseg, int64_t words_per_seg,
                      int32_t* halo_idx, hipStream_t st) {
  const int64_t n_words = nseg * words_per_seg;
  if (n_words > 0)
    hipLaunchKernelGGL(k_fill_halo, grid_for(n_words), kBlock, 0, st, bitmap, word_rank, n_words,
                       words_per_seg, halo_idx);
}

void launch_seg_halo_off(const int64_t* word_rank, int64_t nseg, int64_t words_per_seg, int64_t total_words,
                         const int64_t* total_dev, Segment* segs, int64_t* halo_ptr, hipStream_t st) {
  hipLaunchKernelGGL(k_seg_halo_off, grid_for(nseg + 1), kBlock, 0, st, word_rank, nseg, words_per_seg,
                     total_words, total_dev, segs, halo_ptr);
}

void launch_col_local(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_nnz,
                      int64_t words_per_seg, const uint32_t* bitmap, const int64_t* word_rank,
                      int32_t* col_local, hipStream_t st) {
  if (total_nnz > 0)
    hipLaunchKernelGGL(k_col_local, grid_for(total_nnz), kBlock, 0, st, g, segs, nseg, total_nnz,
                       words_per_seg, bitmap, word_rank, col_local);
}

void launch_long_count(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_rows,
                       int32_t long_nnz, int32_t part_nnz, int64_t* counts, hipStream_t st) {
  if (total_rows > 0)
    hipLaunchKernelGGL(k_long_count, grid_for(total_rows), kBlock, 0, st, g, segs, nseg, total_rows,
                       long_nnz, part_nnz, counts);
}

void launch_long_fill(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_rows,
                      int32_t long_nnz, int32_t part_nnz, const int64_t* offs, int32_t* work_long,
                      hipStream_t st) {
  if (total_rows > 0)
    hipLaunchKernelGGL(k_long_fill, grid_for(total_rows), kBlock, 0, st, g, segs, nseg, total_rows,
                       long_nnz, part_nnz, offs, work_long);
}

void launch_validate_graph(const GraphDev& g, int32_t* flags, hipStream_t st) {
  const int64_t n = (int64_t)g.T * g.N;
  if (n > 0) hipLaunchKernelGGL(k_validate_graph, grid_for(n), kBlock, 0, st, g, flags);
}

}  // namespace dgc
