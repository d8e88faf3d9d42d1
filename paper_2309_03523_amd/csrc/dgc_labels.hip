// Generated chunks as the layer's input (Sections 4.1 and 5.2): a chunk is the set of
// (snapshot, vertex) pairs that carry one label.  Two tables turn the labels into what the
// aggregation and the recurrent kernels already understand:
//   col_signed[e]  the stored column j of non-zero e if label[t, j] == label[t, i] (the neighbour
//                  is in the row's chunk: read the fresh row), else ~j (read the cache row);
//   seq_in / seq_out [t*N + i]  t*N + i where a vertex's run of equal labels starts / ends
//                  (the state enters from, or leaves to, the state cache there), else -1.
// Integer work, done once per labelling.
#include "dgc_internal.h"

namespace dgc {
namespace {

// one thread per stored non-zero of snapshot blockIdx.y (grid-stride over the snapshot)
__global__ __launch_bounds__(256) void k_lab_cols(GraphDev g, const Segment* segs, const int32_t* labels,
                                                  int32_t* col_signed) {
  const int t = blockIdx.y;               // segment t is snapshot t: the layer has one chunk over everything
  const int64_t* rp = g.rowptr[t];
  const int32_t* cj = g.colidx[t];
  const int32_t* lab = labels + (int64_t)t * g.N;
  int32_t* out = col_signed + segs[t].nnz_off;
  const int64_t nnz = rp[g.N];
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * blockDim.x) {
    int64_t lo = 0, hi = g.N - 1;        // the row of e: largest i with rowptr[i] <= e
    while (lo < hi) {
      const int64_t mid = (lo + hi + 1) >> 1;
      if (rp[mid] <= e) lo = mid; else hi = mid - 1;
    }
    const int32_t j = cj[e];
    out[e] = lab[j] == lab[lo] ? j : ~j;
  }
}

__global__ __launch_bounds__(256) void k_lab_seq(const int32_t* labels, int32_t T, int64_t N, int64_t* seq_in,
                                                 int64_t* seq_out) {
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= (int64_t)T * N) return;
  const int64_t t = x / N;
  const int32_t me = labels[x];
  seq_in[x] = (t == 0 || labels[x - N] != me) ? x : -1;
  seq_out[x] = (t == T - 1 || labels[x + N] != me) ? x : -1;
}

}  // namespace

void labels_build(const GraphDev& g, const Segment* segs, const int32_t* labels, int32_t* col_signed,
                  int64_t* seq_in, int64_t* seq_out, hipStream_t st) {
  if (g.N <= 0 || g.T <= 0) return;
  hipLaunchKernelGGL(k_lab_cols, dim3(1024, (unsigned)g.T), 256, 0, st, g, segs, labels, col_signed);
  const int64_t n = (int64_t)g.T * g.N;
  hipLaunchKernelGGL(k_lab_seq, (unsigned)((n + 255) / 256), 256, 0, st, labels, g.T, g.N, seq_in, seq_out);
}

}  // namespace dgc
