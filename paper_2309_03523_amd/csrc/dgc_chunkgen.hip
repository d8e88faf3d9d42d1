// Chunk generation by weighted label propagation on the super-graph (Section 4.1 of the paper).
//
// Super-vertex x = t*N + i; spatial edges of snapshot t (self-loops dropped) weigh w_s, the
// virtual temporal edges (t, i) - (t +- 1, i) weigh w_t.  Labels start all different
// (c(v_{i,t}) = t*N + i).  One iteration, all on the labels of the iteration before:
//   propose  every vertex scores the labels of its neighbours (sum of edge weights per label) and
//            takes as candidate the admissible one (carried by fewer than `cap` vertices) with
//            the largest score, ties to the label carried by fewer vertices, then to the smaller
//            label; it wants to change if the candidate scores strictly more than its own label;
//   decide   a vertex that wants to change does so unless a neighbour with a smaller index also
//            wants to (no two neighbours change together, so every change raises the weight
//            inside chunks and the iteration count is bounded); chunk sizes follow.
// Scores are integers: sums and the integer atomics on the sizes are exact in any order.
//
// Rows of at most kShort neighbours: one thread each, neighbour labels in a private LDS strip,
// scores by comparing all pairs.  Longer rows (a list built once): one workgroup each, scores in
// an LDS hash table, in several passes over disjoint label classes when the row is longer than
// the table can take.
#include <algorithm>

#include "dgc_internal.h"

namespace dgc {
namespace {

constexpr int kBlock = 256;
constexpr int kShort = 32;            // neighbours (spatial + temporal) a thread handles alone
constexpr int kSlots = 4096;          // hash table of the long-row kernel
constexpr int kPerPass = 1024;        // distinct labels a pass is sized for
constexpr uint32_t kTemporal = 0x80000000u;

struct CgArgs {
  GraphDev g;
  int32_t w_s, w_t;
  int64_t cap;
  int32_t* labels;       // [T*N]
  int32_t* want;         // [T*N] candidate, or -1
  int32_t* size;         // [T*N] vertices per label
  const int32_t* long_rows; int32_t n_long;
  int32_t* counters;     // [0] vertices changed this iteration, [1] long-row list fill, [2] hash overflow
};

struct Best {            // ordered by (score desc, size asc, label asc)
  uint32_t score; int32_t size; int32_t label;
};
__device__ __forceinline__ bool better(const Best& a, const Best& b) {
  if (a.score != b.score) return a.score > b.score;
  if (a.size != b.size) return a.size < b.size;
  return a.label < b.label;
}

__device__ __forceinline__ int32_t degree_of(const GraphDev& g, int32_t t, int64_t i) {
  const int64_t* rp = g.rowptr[t];
  return (int32_t)(rp[i + 1] - rp[i]) - 1 + (t > 0) + (t + 1 < g.T);   // the stored self-loop is not an edge
}

__global__ void k_cg_init(CgArgs a, int64_t n) {
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= n) return;
  a.labels[x] = (int32_t)x;
  a.size[x] = 1;
  a.want[x] = -1;
}

__global__ void k_cg_count_long(CgArgs a, int64_t n, int32_t* list) {
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= n) return;
  const int32_t t = (int32_t)(x / a.g.N);
  if (degree_of(a.g, t, x - (int64_t)t * a.g.N) > kShort) {
    const int32_t k = atomicAdd(&a.counters[1], 1);
    if (list) list[k] = (int32_t)x;
  }
}

// ---- short rows
__global__ __launch_bounds__(kBlock) void k_cg_propose_short(CgArgs a, int64_t n) {
  __shared__ uint32_t strip[kShort * kBlock];   // [k][thread]: neighbour label, top bit = temporal edge
  const int64_t x = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (x >= n) return;
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t* rp = a.g.rowptr[t];
  const int64_t e0 = rp[i], e1 = rp[i + 1];
  const int d = (int)(e1 - e0) - 1 + (t > 0) + (t + 1 < a.g.T);
  if (d > kShort) return;                        // the long-row kernel's
  uint32_t* s = strip + threadIdx.x;
  int k = 0;
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  for (int64_t e = e0; e < e1; ++e) {
    const int32_t j = col[e];
    if (j != i && k < kShort) { s[k * kBlock] = (uint32_t)a.labels[base + j]; ++k; }
  }
  if (t > 0 && k < kShort) { s[k * kBlock] = (uint32_t)a.labels[x - a.g.N] | kTemporal; ++k; }
  if (t + 1 < a.g.T && k < kShort) { s[k * kBlock] = (uint32_t)a.labels[x + a.g.N] | kTemporal; ++k; }
  const int32_t own_label = a.labels[x];
  uint32_t own = 0;
  Best best{0u, 0, -1};
  for (int p = 0; p < k; ++p) {
    const uint32_t lp = s[p * kBlock] & ~kTemporal;
    bool first = true;
    uint32_t score = 0;
    for (int q = 0; q < k; ++q) {
      const uint32_t v = s[q * kBlock];
      if ((v & ~kTemporal) == lp) {
        if (q < p) { first = false; break; }
        score += (v & kTemporal) ? (uint32_t)a.w_t : (uint32_t)a.w_s;
      }
    }
    if (!first || score == 0) continue;
    if ((int32_t)lp == own_label) { own = score; continue; }
    const int32_t sz = a.size[lp];
    if (sz >= a.cap) continue;
    const Best c{score, sz, (int32_t)lp};
    if (best.label < 0 || better(c, best)) best = c;
  }
  a.want[x] = (best.label >= 0 && best.score > own) ? best.label : -1;
}

__device__ __forceinline__ void apply_change(const CgArgs& a, int64_t x, int32_t to) {
  const int32_t from = a.labels[x];
  a.labels[x] = to;
  atomicAdd(&a.size[to], 1);
  atomicSub(&a.size[from], 1);
  atomicAdd(&a.counters[0], 1);
}

__global__ __launch_bounds__(kBlock) void k_cg_decide_short(CgArgs a, int64_t n) {
  const int64_t x = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (x >= n) return;
  const int32_t w = a.want[x];
  if (w < 0) return;
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t* rp = a.g.rowptr[t];
  const int64_t e0 = rp[i], e1 = rp[i + 1];
  if ((int)(e1 - e0) - 1 + (t > 0) + (t + 1 < a.g.T) > kShort) return;
  if (t > 0 && a.want[x - a.g.N] >= 0) return;   // the earlier copy has the smaller index
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  for (int64_t e = e0; e < e1; ++e) {            // columns ascend: only those below i can block
    const int32_t j = col[e];
    if (j >= i) break;
    if (a.want[base + j] >= 0) return;
  }
  apply_change(a, x, w);
}

// ---- long rows
__device__ __forceinline__ uint32_t mix(uint32_t v) {   // a bijection on 32 bits
  v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
  return v;
}

__device__ __forceinline__ Best block_best(Best b, Best* red) {
  red[threadIdx.x] = b;
  __syncthreads();
  for (int s = kBlock / 2; s > 0; s >>= 1) {
    if (threadIdx.x < s) {
      const Best o = red[threadIdx.x + s];
      Best& m = red[threadIdx.x];
      if (o.label >= 0 && (m.label < 0 || better(o, m))) m = o;
    }
    __syncthreads();
  }
  const Best r = red[0];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(kBlock) void k_cg_propose_long(CgArgs a) {
  __shared__ int32_t key[kSlots];
  __shared__ uint32_t val[kSlots];
  __shared__ Best red[kBlock];
  __shared__ uint32_t own_score;
  __shared__ int overflow;
  const int64_t x = a.long_rows[blockIdx.x];
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t e0 = a.g.rowptr[t][i], e1 = a.g.rowptr[t][i + 1];
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  const int32_t own_label = a.labels[x];
  const int64_t n_sp = e1 - e0;                  // stored entries, self-loop included
  uint32_t passes = (uint32_t)((n_sp + 2 + kPerPass - 1) / kPerPass);
  for (;;) {                                     // again with twice the passes if a table overflowed
    Best best{0u, 0, -1};
    if (threadIdx.x == 0) { own_score = 0; overflow = 0; }
    for (uint32_t p = 0; p < passes; ++p) {
      for (int sidx = threadIdx.x; sidx < kSlots; sidx += kBlock) { key[sidx] = -1; val[sidx] = 0; }
      __syncthreads();
      for (int64_t e = threadIdx.x; e < n_sp + 2; e += kBlock) {
        int32_t lab; uint32_t w;
        if (e < n_sp) {
          const int32_t j = col[e0 + e];
          if (j == i) continue;
          lab = a.labels[base + j]; w = (uint32_t)a.w_s;
        } else if (e == n_sp) {
          if (t == 0) continue;
          lab = a.labels[x - a.g.N]; w = (uint32_t)a.w_t;
        } else {
          if (t + 1 >= a.g.T) continue;
          lab = a.labels[x + a.g.N]; w = (uint32_t)a.w_t;
        }
        if (w == 0) continue;
        const uint32_t h = mix((uint32_t)lab);
        if (h % passes != p) continue;
        uint32_t slot = (h / passes) & (kSlots - 1);
        int probes = 0;
        for (;; slot = (slot + 1) & (kSlots - 1)) {
          const int32_t prev = atomicCAS(&key[slot], -1, lab);
          if (prev == -1 || prev == lab) { atomicAdd(&val[slot], w); break; }
          if (++probes >= kSlots) { overflow = 1; break; }
        }
      }
      __syncthreads();
      for (int sidx = threadIdx.x; sidx < kSlots; sidx += kBlock) {
        const int32_t lab = key[sidx];
        if (lab < 0) continue;
        if (lab == own_label) { own_score = val[sidx]; continue; }
        const int32_t sz = a.size[lab];
        if (sz >= a.cap) continue;
        const Best c{val[sidx], sz, lab};
        if (best.label < 0 || better(c, best)) best = c;
      }
      __syncthreads();
    }
    const int ovf = overflow;
    const uint32_t own = own_score;
    best = block_best(best, red);
    if (!ovf) {
      if (threadIdx.x == 0) a.want[x] = (best.label >= 0 && best.score > own) ? best.label : -1;
      return;
    }
    if (passes > (1u << 20)) {                   // cannot happen with a bijective mix; leave a trace and stop
      if (threadIdx.x == 0) { a.want[x] = -1; atomicAdd(&a.counters[2], 1); }
      return;
    }
    passes *= 2;
  }
}

__global__ __launch_bounds__(kBlock) void k_cg_decide_long(CgArgs a) {
  __shared__ int blocked;
  const int64_t x = a.long_rows[blockIdx.x];
  const int32_t w = a.want[x];
  if (w < 0) return;                             // the same for the whole workgroup
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t e0 = a.g.rowptr[t][i], e1 = a.g.rowptr[t][i + 1];
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  if (threadIdx.x == 0) blocked = (t > 0 && a.want[x - a.g.N] >= 0) ? 1 : 0;
  __syncthreads();
  for (int64_t e = e0 + threadIdx.x; e < e1; e += kBlock) {
    const int32_t j = col[e];
    if (j < i && a.want[base + j] >= 0) blocked = 1;
  }
  __syncthreads();
  if (threadIdx.x == 0 && !blocked) apply_change(a, x, w);
}

unsigned grid_of(int64_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

}  // namespace
}  // namespace dgc

using namespace dgc;

extern "C" dgc_status_t dgc_chunk_generate(const dgc_graph_t* graph, int32_t w_s, int32_t w_t, int64_t cap,
                                           int32_t max_iters, int32_t* labels, int32_t* iters_out,
                                           int32_t* converged_out, void* stream) {
  auto bad = [](dgc_status_t code, const std::string& msg) { set_thread_error(msg); return code; };
  if (!graph || !labels || !graph->rowptr || !graph->colidx) return bad(DGC_ERR_INVALID_ARG, "chunk generate: NULL argument");
  if (graph->T < 1 || graph->N < 1) return bad(DGC_ERR_INVALID_ARG, "chunk generate: T and N must be >= 1");
  const int64_t n = (int64_t)graph->T * graph->N;
  if (n >= (int64_t)1 << 31) return bad(DGC_ERR_UNSUPPORTED, "chunk generate: T*N must be below 2^31 (labels are int32)");
  if (w_s < 0 || w_t < 0 || w_s > (1 << 20) || w_t > (1 << 20))
    return bad(DGC_ERR_INVALID_ARG, "chunk generate: edge weights must be in [0, 2^20]");
  if (cap < 1 || max_iters < 1) return bad(DGC_ERR_INVALID_ARG, "chunk generate: cap and max_iters must be >= 1");
  for (int32_t t = 0; t < graph->T; ++t)
    if (!graph->rowptr[t] || !graph->colidx[t]) return bad(DGC_ERR_INVALID_ARG, "chunk generate: NULL snapshot pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);

  std::vector<void*> owned;
  auto release = [&]() { for (void* p : owned) (void)hipFree(p); };
  auto alloc = [&](void** p, size_t bytes) {
    const hipError_t e = hipMalloc(p, std::max<size_t>(bytes, 8));
    if (e == hipSuccess) owned.push_back(*p);
    return e;
  };
#define CG_TRY(expr)                                                                          \
  do {                                                                                        \
    const hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                                   \
      release();                                                                              \
      return bad(e_ == hipErrorOutOfMemory ? DGC_ERR_OOM : DGC_ERR_DEVICE,                    \
                 std::string("chunk generate: " #expr ": ") + hipGetErrorString(e_));         \
    }                                                                                         \
  } while (0)

  const int64_t** d_rp = nullptr; const int32_t** d_ci = nullptr;
  int32_t *want = nullptr, *size = nullptr, *counters = nullptr, *list = nullptr;
  CG_TRY(alloc((void**)&d_rp, sizeof(void*) * graph->T));
  CG_TRY(alloc((void**)&d_ci, sizeof(void*) * graph->T));
  CG_TRY(alloc((void**)&want, sizeof(int32_t) * n));
  CG_TRY(alloc((void**)&size, sizeof(int32_t) * n));
  CG_TRY(alloc((void**)&counters, sizeof(int32_t) * 4));
  CG_TRY(hipMemcpyAsync(d_rp, graph->rowptr, sizeof(void*) * graph->T, hipMemcpyHostToDevice, st));
  CG_TRY(hipMemcpyAsync(d_ci, graph->colidx, sizeof(void*) * graph->T, hipMemcpyHostToDevice, st));
  CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t) * 4, st));

  CgArgs a{};
  a.g = GraphDev{graph->T, graph->N, d_rp, d_ci};
  {  // the kernels index by the stored columns: check the graph contract first
    int32_t flags[4] = {0, 0, 0, 0};
    launch_validate_rowptr(a.g, counters, st);
    CG_TRY(hipMemcpyAsync(flags, counters, sizeof(flags), hipMemcpyDeviceToHost, st));
    CG_TRY(hipStreamSynchronize(st));
    if (flags[0]) { release(); return bad(DGC_ERR_BAD_GRAPH, "chunk generate: rowptr does not start at 0 or decreases"); }
    launch_validate_graph(a.g, counters, st);
    CG_TRY(hipMemcpyAsync(flags, counters, sizeof(flags), hipMemcpyDeviceToHost, st));
    CG_TRY(hipStreamSynchronize(st));
    if (flags[0] || flags[1] || flags[2] || flags[3]) {
      release();
      return bad(DGC_ERR_BAD_GRAPH, "chunk generate: the CSR arrays violate the graph contract (columns in range, "
                                     "ascending and unique, self-loop stored, symmetric)");
    }
    CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t) * 4, st));
  }
  a.w_s = w_s; a.w_t = w_t; a.cap = cap;
  a.labels = labels; a.want = want; a.size = size; a.counters = counters;
  int32_t host_c[4] = {0, 0, 0, 0};
  hipLaunchKernelGGL(k_cg_init, grid_of(n), kBlock, 0, st, a, n);
  hipLaunchKernelGGL(k_cg_count_long, grid_of(n), kBlock, 0, st, a, n, (int32_t*)nullptr);
  CG_TRY(hipMemcpyAsync(host_c, counters, sizeof(host_c), hipMemcpyDeviceToHost, st));
  CG_TRY(hipStreamSynchronize(st));
  const int32_t n_long = host_c[1];
  if (n_long > 0) {
    CG_TRY(alloc((void**)&list, sizeof(int32_t) * n_long));
    CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t) * 4, st));
    hipLaunchKernelGGL(k_cg_count_long, grid_of(n), kBlock, 0, st, a, n, list);
  }
  a.long_rows = list; a.n_long = n_long;

  int32_t it = 0, converged = 0;
  while (it < max_iters) {
    CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t), st));
    hipLaunchKernelGGL(k_cg_propose_short, grid_of(n), kBlock, 0, st, a, n);
    if (n_long > 0) hipLaunchKernelGGL(k_cg_propose_long, (unsigned)n_long, kBlock, 0, st, a);
    hipLaunchKernelGGL(k_cg_decide_short, grid_of(n), kBlock, 0, st, a, n);
    if (n_long > 0) hipLaunchKernelGGL(k_cg_decide_long, (unsigned)n_long, kBlock, 0, st, a);
    CG_TRY(hipMemcpyAsync(host_c, counters, sizeof(host_c), hipMemcpyDeviceToHost, st));
    CG_TRY(hipStreamSynchronize(st));
    ++it;
    if (host_c[2]) { release(); return bad(DGC_ERR_UNSUPPORTED, "chunk generate: a label table overflowed"); }
    if (host_c[0] == 0) { converged = 1; break; }
  }
  CG_TRY(hipGetLastError());
  release();
#undef CG_TRY
  if (iters_out) *iters_out = it;
  if (converged_out) *converged_out = converged;
  return DGC_OK;
}
