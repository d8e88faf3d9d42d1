// Spatial-fusion selection (Section 5.1.1 of the paper) and chunk assignment (Section 4.2,
// Algorithm 1).
//
// Device part: the estimate of redundant loading between every pair of chunks.  A chunk has to
// load its own (snapshot, vertex) rows and, per snapshot, the de-duplicated neighbours outside its
// vertex range (the halo lists of the packing); two chunks processed one after the other load the
// rows they have in common twice, fused once.  shared(a,b) = number of common rows:
//   1. one bit per (row, chunk): bit c of mask[t*N + v] says chunk c loads row (t, v)
//      (integer atomic OR from the packed rows and halo lists);
//   2. every row with k loaders adds one to each of its k(k-1)/2 pairs: counted per workgroup in an
//      LDS matrix (integer atomics: exact and independent of order), flushed once per workgroup.
// Host part: the two greedy procedures, O(n^3) and O(n^2 m) on chunk-level tables.
#include <algorithm>
#include <vector>

#include "dgc_internal.h"

namespace dgc {
namespace {

constexpr int kFsBlock = 256;
constexpr int kFsLdsChunks = 128;  // n*n uint32 counters fit 64 KB of LDS up to this many chunks

__global__ void k_fs_zero(unsigned long long* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// blockIdx.y = segment; x strides over the segment's own rows, then over its halo list
__global__ void k_fs_mark(const Segment* segs, const int64_t* halo_ptr, const int32_t* halo_idx, int64_t N, int W,
                          unsigned long long* mask) {
  const Segment sg = segs[blockIdx.y];
  const int word = sg.chunk >> 6;
  const unsigned long long bit = 1ull << (sg.chunk & 63);
  unsigned long long* m = mask + (int64_t)sg.t * N * W + word;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x, first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int64_t v = sg.v_lo + first; v < sg.v_hi; v += stride) atomicOr(m + v * W, bit);
  for (int64_t p = halo_ptr[blockIdx.y] + first; p < halo_ptr[blockIdx.y + 1]; p += stride)
    atomicOr(m + (int64_t)halo_idx[p] * W, bit);
}

template <bool LDS>
__global__ __launch_bounds__(kFsBlock) void k_fs_pairs(const unsigned long long* mask, int64_t rows, int W, int n,
                                                       unsigned long long* out) {
  extern __shared__ unsigned int cnt[];
  if (LDS) {
    for (int i = threadIdx.x; i < n * n; i += kFsBlock) cnt[i] = 0;
    __syncthreads();
  }
  for (int64_t r = (int64_t)blockIdx.x * kFsBlock + threadIdx.x; r < rows; r += (int64_t)gridDim.x * kFsBlock) {
    const unsigned long long* m = mask + r * W;
    for (int wa = 0; wa < W; ++wa) {
      unsigned long long ma = m[wa];
      while (ma) {
        const int a = wa * 64 + __ffsll((long long)ma) - 1;
        ma &= ma - 1;
        unsigned long long mb = ma;  // partners b > a: the rest of this word, then the later words
        for (int wb = wa;;) {
          while (mb) {
            const int b = wb * 64 + __ffsll((long long)mb) - 1;
            mb &= mb - 1;
            if (LDS) atomicAdd(&cnt[a * n + b], 1u); else atomicAdd(&out[(int64_t)a * n + b], 1ull);
          }
          if (++wb >= W) break;
          mb = m[wb];
        }
      }
    }
  }
  if (LDS) {
    __syncthreads();
    for (int i = threadIdx.x; i < n * n; i += kFsBlock)
      if (cnt[i]) atomicAdd(&out[i], (unsigned long long)cnt[i]);
  }
}

}  // namespace

int64_t shared_rows_mask_words(int32_t T, int64_t N, int32_t n_chunks) { return (int64_t)T * N * ((n_chunks + 63) / 64); }

void launch_shared_rows(const Segment* segs, int64_t nseg, const int64_t* halo_ptr, const int32_t* halo_idx, int32_t T,
                        int64_t N, int32_t n_chunks, unsigned long long* mask, unsigned long long* out,
                        hipStream_t st) {
  const int W = (n_chunks + 63) / 64;
  const int64_t rows = (int64_t)T * N;
  hipLaunchKernelGGL(k_fs_zero, 2048, 256, 0, st, mask, rows * W);
  hipLaunchKernelGGL(k_fs_zero, 64, 256, 0, st, out, (int64_t)n_chunks * n_chunks);
  hipLaunchKernelGGL(k_fs_mark, dim3(32, (unsigned)nseg), 256, 0, st, segs, halo_ptr, halo_idx, N, W, mask);
  const unsigned grid = (unsigned)std::min<int64_t>((rows + kFsBlock - 1) / kFsBlock, 256 * 8);
  if (n_chunks <= kFsLdsChunks)
    hipLaunchKernelGGL(k_fs_pairs<true>, grid, kFsBlock, sizeof(unsigned) * n_chunks * n_chunks, st, mask, rows, W,
                       n_chunks, out);
  else
    hipLaunchKernelGGL(k_fs_pairs<false>, grid, kFsBlock, 0, st, mask, rows, W, n_chunks, out);
}

}  // namespace dgc

using namespace dgc;

extern "C" {

dgc_status_t dgc_fusion_select(int32_t n, const int64_t* shared, const int64_t* mem, int64_t cap, int32_t* group_out) {
  if (n < 1 || !shared || !mem || !group_out) { set_thread_error("fusion select: NULL argument or n < 1"); return DGC_ERR_INVALID_ARG; }
  for (int32_t a = 0; a < n; ++a) {
    if (mem[a] < 0) { set_thread_error("fusion select: negative memory"); return DGC_ERR_INVALID_ARG; }
    for (int32_t b = 0; b < n; ++b)
      if (shared[(int64_t)a * n + b] != shared[(int64_t)b * n + a] || shared[(int64_t)a * n + b] < 0) {
        set_thread_error("fusion select: the shared matrix must be symmetric and non-negative");
        return DGC_ERR_INVALID_ARG;
      }
  }
  // groups are named by their smallest member; S is the matrix contracted over the groups
  std::vector<int64_t> S(shared, shared + (int64_t)n * n), gm(mem, mem + n);
  std::vector<int32_t> owner(n);
  std::vector<char> alive(n, 1);
  for (int32_t a = 0; a < n; ++a) owner[a] = a;
  for (;;) {
    int32_t ba = -1, bb = -1;
    int64_t best = -1;
    for (int32_t a = 0; a < n; ++a) {
      if (!alive[a]) continue;
      for (int32_t b = a + 1; b < n; ++b)
        if (alive[b] && gm[a] + gm[b] <= cap && S[(int64_t)a * n + b] > best) { best = S[(int64_t)a * n + b]; ba = a; bb = b; }
    }
    if (ba < 0) break;
    for (int32_t c = 0; c < n; ++c) {
      S[(int64_t)ba * n + c] += S[(int64_t)bb * n + c];
      S[(int64_t)c * n + ba] = S[(int64_t)ba * n + c];
    }
    gm[ba] += gm[bb];
    alive[bb] = 0;
    for (int32_t c = 0; c < n; ++c) if (owner[c] == bb) owner[c] = ba;
  }
  std::vector<int32_t> gid(n, -1);
  int32_t next = 0;
  for (int32_t a = 0; a < n; ++a) if (alive[a]) gid[a] = next++;
  for (int32_t a = 0; a < n; ++a) group_out[a] = gid[owner[a]];
  return DGC_OK;
}

// Chunk assignment (Section 4.2, Algorithm 1) with a running traffic table: traffic[m][a] is what
// chunk a would exchange with the chunks already placed on worker m.  Placing chunk b on m adds
// h(a, b) to row m for every chunk a still waiting, so scoring a chunk costs O(workers) and the whole
// procedure O(n^2 + n * workers) instead of summing over every worker's chunk list for every chunk.
// (The additions happen in placement order, the order in which a sum over the list would run.)
// Readings the paper leaves open: a worker without chunks, or without traffic to the chunk, scores 0
// whatever its load; equal scores go to the worker with the smaller assigned load, then the smaller index.
dgc_status_t dgc_chunk_assign(int32_t n, const double* g, const double* h, int32_t n_gpus, int32_t* x_out) {
  if (n < 1 || n_gpus < 1 || !g || !h || !x_out) { set_thread_error("chunk assign: NULL argument, n < 1 or n_gpus < 1"); return DGC_ERR_INVALID_ARG; }
  std::vector<int32_t> by_work(n);
  for (int32_t a = 0; a < n; ++a) by_work[a] = a;
  std::stable_sort(by_work.begin(), by_work.end(), [&](int32_t a, int32_t b) { return g[a] > g[b]; });
  double work_sum = 0.0;
  for (int32_t a = 0; a < n; ++a) work_sum += g[a];
  const double fair_share = work_sum / n_gpus;
  std::vector<double> traffic((size_t)n_gpus * n, 0.0), assigned(n_gpus, 0.0);
  std::vector<char> waiting(n, 1);
  for (int32_t a : by_work) {
    int32_t pick = 0;
    double pick_score = (fair_share - assigned[0]) * traffic[a];
    for (int32_t m = 1; m < n_gpus; ++m) {
      const double score = (fair_share - assigned[m]) * traffic[(size_t)m * n + a];
      if (score > pick_score || (score == pick_score && assigned[m] < assigned[pick])) { pick = m; pick_score = score; }
    }
    x_out[a] = pick;
    assigned[pick] += g[a];
    waiting[a] = 0;
    double* row = traffic.data() + (size_t)pick * n;
    for (int32_t c = 0; c < n; ++c)
      if (waiting[c]) row[c] += h[(int64_t)c * n + a];
  }
  return DGC_OK;
}

}  // extern "C"
