// Chunk generation by weighted label propagation on the super-graph (Section 4.1 of the paper).
//
// Super-vertex x = t*N + i; spatial edges of snapshot t (self-loops dropped) weigh w_s, the
// virtual temporal edges (t, i) - (t +- 1, i) weigh w_t.  Labels start all different
// (c(v_{i,t}) = t*N + i).  One iteration, all on the labels of the iteration before:
//   propose  every vertex scores the labels of its neighbours (sum of edge weights per label) and
//            takes as candidate the admissible one (carried by fewer than `cap` vertices) with
//            the largest score, ties to the label carried by fewer vertices, then to the smaller
//            label; it wants to change if the candidate scores strictly more than its own label;
//   decide   a vertex that wants to change does so unless a neighbour that also wants to comes
//            before it in the iteration's order (a hash of vertex and iteration, then the index):
//            no two neighbours change together, so every change raises the weight inside chunks
//            and the iteration count is bounded; the hashed order keeps chains of waiting
//            vertices short.  Chunk sizes follow.
// Scores are integers: sums and the integer atomics on the sizes are exact in any order.
//
// Rows of at most kShort neighbours: one thread each, neighbour labels in a private LDS strip,
// scores by comparing all pairs.  Longer rows (two lists built once): one wavefront (up to kMid
// neighbours) or one 256-thread workgroup each, scores in an LDS hash table sized to the row, in
// several passes over disjoint label classes when the row holds more distinct labels than the
// table takes; the pass count that worked is remembered per row (labels merge as the propagation
// goes on) and doubled when a table fills up.
//
// Most iterations change few labels.  When a vertex is looked at, the margin by which its own
// label's score exceeds every other label's score is kept (-1 if it does not: the vertex is looked
// at again next time).  A neighbour that changes label over an edge of weight w moves w from one
// label's score to another's, so it can lower that margin by at most 2w: the decide step adds 2w to
// the vertex's `drift`, and while drift <= margin no candidate can score strictly more than the own
// label, whatever the sizes and ties - the vertex still does not want to change and is skipped.
// A vertex that changes its own label is looked at again.  The result is exactly that of looking at
// every vertex every time; hub rows with a clear majority label stay skipped through many changes
// of their neighbourhood.
#include <algorithm>

#include "dgc_internal.h"

namespace dgc {
namespace {

constexpr int kBlock = 256;
constexpr int kShort = 32;            // neighbours (spatial + temporal) a thread handles alone
constexpr int kMid = 448;             // up to here a wavefront with a 1024-slot table (never more than one pass)
constexpr int kMidSlots = 1024;
constexpr int kBigSlots = 8192;       // table of the workgroup-per-row kernel
constexpr uint32_t kTemporal = 0x80000000u;

struct CgArgs {
  GraphDev g;
  int32_t w_s, w_t;
  int64_t cap;
  int32_t* labels;       // [T*N]
  int32_t* want;         // [T*N] candidate, or -1
  int32_t* size;         // [T*N] vertices per label
  const int32_t* rows;   // list of the long-row kernel at hand
  int32_t* passes_hint;  // per entry of that list: pass count that last worked (0 = none yet)
  uint32_t salt;         // changes with the iteration: order of the decide step
  long long* margin;             // [T*N] own score - best other score at the last look, -1 = look again
  unsigned long long* drift;     // [T*N] twice the weight of the neighbour edges whose far end changed label since
  int32_t* counters;     // [0] vertices changed this iteration, [1] / [2] list fills, [3] hash overflow
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
  a.margin[x] = -1;        // everybody is looked at in the first iteration
  a.drift[x] = 0;
}

__global__ void k_cg_count_long(CgArgs a, int64_t n, int32_t* mid, int32_t* big) {
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= n) return;
  const int32_t t = (int32_t)(x / a.g.N);
  const int32_t d = degree_of(a.g, t, x - (int64_t)t * a.g.N);
  if (d <= kShort) return;
  if (!mid && !big) atomicMax(&a.counters[3], d);   // counting pass: also the largest degree
  const int which = d <= kMid ? 1 : 2;
  const int32_t k = atomicAdd(&a.counters[which], 1);
  int32_t* list = which == 1 ? mid : big;
  if (list) list[k] = (int32_t)x;
}

__device__ __forceinline__ uint32_t mix(uint32_t v) {   // a bijection on 32 bits
  v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
  return v;
}

// true if wanting neighbour u comes before x in this iteration's order
__device__ __forceinline__ bool before(uint32_t salt, int64_t u, int64_t x) {
  const uint32_t pu = mix((uint32_t)u ^ salt), px = mix((uint32_t)x ^ salt);
  return pu != px ? pu < px : u < x;
}

// ---- short rows
__global__ __launch_bounds__(kBlock) void k_cg_propose_short(CgArgs a, int64_t n) {
  __shared__ uint32_t strip[kShort * kBlock];   // [k][thread]: neighbour label, top bit = temporal edge
  const int64_t x = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (x >= n) return;
  if (a.margin[x] >= 0 && a.drift[x] <= (unsigned long long)a.margin[x]) return;   // want[x] stays -1
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t* rp = a.g.rowptr[t];
  const int64_t e0 = rp[i], e1 = rp[i + 1];
  const int d = (int)(e1 - e0) - 1 + (t > 0) + (t + 1 < a.g.T);
  if (d > kShort) return;                        // the long-row kernels'
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
  uint32_t own = 0, max_other = 0;
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
    max_other = max(max_other, score);
    const int32_t sz = a.size[lp];
    if (sz >= a.cap) continue;
    const Best c{score, sz, (int32_t)lp};
    if (best.label < 0 || better(c, best)) best = c;
  }
  a.want[x] = (best.label >= 0 && best.score > own) ? best.label : -1;
  a.margin[x] = own >= max_other ? (long long)(own - max_other) : -1;
  a.drift[x] = 0;
}

__device__ __forceinline__ void apply_change(const CgArgs& a, int64_t x, int32_t to) {
  const int32_t from = a.labels[x];
  a.labels[x] = to;
  atomicAdd(&a.size[to], 1);
  atomicSub(&a.size[from], 1);
  atomicAdd(&a.counters[0], 1);
  a.margin[x] = -1;          // (its neighbours' drift is raised by the caller)
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
  if (t > 0 && a.want[x - a.g.N] >= 0 && before(a.salt, x - a.g.N, x)) return;
  if (t + 1 < a.g.T && a.want[x + a.g.N] >= 0 && before(a.salt, x + a.g.N, x)) return;
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  for (int64_t e = e0; e < e1; ++e) {
    const int32_t j = col[e];
    if (j != i && a.want[base + j] >= 0 && before(a.salt, base + j, x)) return;
  }
  apply_change(a, x, w);
  const unsigned long long ds = 2ull * (unsigned long long)a.w_s, dt = 2ull * (unsigned long long)a.w_t;
  for (int64_t e = e0; e < e1; ++e)
    if (col[e] != i) atomicAdd(&a.drift[base + col[e]], ds);
  if (t > 0) atomicAdd(&a.drift[x - a.g.N], dt);
  if (t + 1 < a.g.T) atomicAdd(&a.drift[x + a.g.N], dt);
}

// ---- long rows: one workgroup of THREADS per row, hash table of at most SLOTS entries
template <int THREADS>
__device__ __forceinline__ Best group_best(Best b, Best* red) {
  red[threadIdx.x] = b;
  __syncthreads();
  for (int s = THREADS / 2; s > 0; s >>= 1) {
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

template <int THREADS, int SLOTS>
__global__ __launch_bounds__(THREADS) void k_cg_propose_long(CgArgs a) {
  __shared__ int32_t key[SLOTS];
  __shared__ uint32_t val[SLOTS];
  __shared__ Best red[THREADS];
  __shared__ uint32_t own_score;
  __shared__ int n_keys;
  __shared__ int overflow;
  __shared__ uint32_t max_other;
  const int64_t x = a.rows[blockIdx.x];
  if (a.margin[x] >= 0 && a.drift[x] <= (unsigned long long)a.margin[x]) return;   // the same for the whole workgroup
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t e0 = a.g.rowptr[t][i], e1 = a.g.rowptr[t][i + 1];
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  const int32_t own_label = a.labels[x];
  const int64_t n_sp = e1 - e0;                  // stored entries, self-loop included
  // table sized to the row: at least twice its entries when that fits
  int slots = 64;
  while (slots < SLOTS && slots < 2 * (n_sp + 2)) slots *= 2;
  const int limit = slots / 4 * 3;               // distinct labels a pass may hold
  const int32_t hint = a.passes_hint[blockIdx.x];
  uint32_t passes = hint > 0 ? (uint32_t)max(1, hint / 2) : (uint32_t)((n_sp + 2 + limit - 1) / limit);
  for (;;) {                                     // again with twice the passes if a table filled up
    Best best{0u, 0, -1};
    if (threadIdx.x == 0) { own_score = 0; overflow = 0; max_other = 0; }
    for (uint32_t p = 0; p < passes; ++p) {
      for (int sidx = threadIdx.x; sidx < slots; sidx += THREADS) { key[sidx] = -1; val[sidx] = 0; }
      if (threadIdx.x == 0) n_keys = 0;
      __syncthreads();
      for (int64_t e = threadIdx.x; e < n_sp + 2; e += THREADS) {
        if (*(volatile int*)&overflow) break;
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
        uint32_t slot = (h / passes) & (slots - 1);
        for (int probes = 0; probes < slots; ++probes, slot = (slot + 1) & (slots - 1)) {
          const int32_t prev = atomicCAS(&key[slot], -1, lab);
          if (prev == -1 && atomicAdd(&n_keys, 1) >= limit) overflow = 1;
          if (prev == -1 || prev == lab) { atomicAdd(&val[slot], w); break; }
        }
      }
      __syncthreads();
      if (overflow) break;                       // the same for the whole workgroup
      for (int sidx = threadIdx.x; sidx < slots; sidx += THREADS) {
        const int32_t lab = key[sidx];
        if (lab < 0) continue;
        if (lab == own_label) { own_score = val[sidx]; continue; }
        atomicMax(&max_other, val[sidx]);
        const int32_t sz = a.size[lab];
        if (sz >= a.cap) continue;
        const Best c{val[sidx], sz, lab};
        if (best.label < 0 || better(c, best)) best = c;
      }
      __syncthreads();
    }
    const int ovf = overflow;
    const uint32_t own = own_score;
    best = group_best<THREADS>(best, red);
    if (!ovf) {
      if (threadIdx.x == 0) {
        a.want[x] = (best.label >= 0 && best.score > own) ? best.label : -1;
        a.margin[x] = own >= max_other ? (long long)(own - max_other) : -1;
        a.drift[x] = 0;
        a.passes_hint[blockIdx.x] = (int32_t)passes;
      }
      return;
    }
    if (passes > (1u << 20)) {                   // cannot happen with a bijective mix; leave a trace and stop
      if (threadIdx.x == 0) { a.want[x] = -1; atomicAdd(&a.counters[3], 1); }
      return;
    }
    passes *= 2;
  }
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_cg_decide_long(CgArgs a) {
  __shared__ int blocked;
  const int64_t x = a.rows[blockIdx.x];
  const int32_t w = a.want[x];
  if (w < 0) return;                             // the same for the whole workgroup
  const int32_t t = (int32_t)(x / a.g.N);
  const int64_t i = x - (int64_t)t * a.g.N;
  const int64_t e0 = a.g.rowptr[t][i], e1 = a.g.rowptr[t][i + 1];
  const int32_t* col = a.g.colidx[t];
  const int64_t base = (int64_t)t * a.g.N;
  if (threadIdx.x == 0)
    blocked = ((t > 0 && a.want[x - a.g.N] >= 0 && before(a.salt, x - a.g.N, x)) ||
               (t + 1 < a.g.T && a.want[x + a.g.N] >= 0 && before(a.salt, x + a.g.N, x))) ? 1 : 0;
  __syncthreads();
  for (int64_t e = e0 + threadIdx.x; e < e1; e += THREADS) {
    const int32_t j = col[e];
    if (j != i && a.want[base + j] >= 0 && before(a.salt, base + j, x)) blocked = 1;
  }
  __syncthreads();
  if (blocked) return;                           // the same for the whole workgroup
  const unsigned long long ds = 2ull * (unsigned long long)a.w_s, dt = 2ull * (unsigned long long)a.w_t;
  if (threadIdx.x == 0) {
    apply_change(a, x, w);
    if (t > 0) atomicAdd(&a.drift[x - a.g.N], dt);
    if (t + 1 < a.g.T) atomicAdd(&a.drift[x + a.g.N], dt);
  }
  for (int64_t e = e0 + threadIdx.x; e < e1; e += THREADS)
    if (col[e] != i) atomicAdd(&a.drift[base + col[e]], ds);
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
  int32_t *want = nullptr, *size = nullptr, *counters = nullptr, *mid = nullptr, *big = nullptr, *hints = nullptr;
  long long* margin = nullptr;
  unsigned long long* drift = nullptr;
  CG_TRY(alloc((void**)&d_rp, sizeof(void*) * graph->T));
  CG_TRY(alloc((void**)&d_ci, sizeof(void*) * graph->T));
  CG_TRY(alloc((void**)&want, sizeof(int32_t) * n));
  CG_TRY(alloc((void**)&size, sizeof(int32_t) * n));
  CG_TRY(alloc((void**)&counters, sizeof(int32_t) * 4));
  CG_TRY(alloc((void**)&margin, sizeof(long long) * n));
  CG_TRY(alloc((void**)&drift, sizeof(unsigned long long) * n));
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
  a.margin = margin; a.drift = drift;
  int32_t host_c[4] = {0, 0, 0, 0};
  hipLaunchKernelGGL(k_cg_init, grid_of(n), kBlock, 0, st, a, n);
  hipLaunchKernelGGL(k_cg_count_long, grid_of(n), kBlock, 0, st, a, n, (int32_t*)nullptr, (int32_t*)nullptr);
  CG_TRY(hipMemcpyAsync(host_c, counters, sizeof(host_c), hipMemcpyDeviceToHost, st));
  CG_TRY(hipStreamSynchronize(st));
  const int32_t n_mid = host_c[1], n_big = host_c[2];
  {  // scores are 32-bit sums of edge weights over a row
    const int64_t max_deg = std::max<int64_t>(host_c[3], kShort) + 2;
    if (max_deg * std::max(w_s, w_t) >= ((int64_t)1 << 32)) {
      release();
      return bad(DGC_ERR_UNSUPPORTED, "chunk generate: largest degree x edge weight must stay below 2^32");
    }
  }
  CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t) * 4, st));
  if (n_mid + n_big > 0) {
    CG_TRY(alloc((void**)&mid, sizeof(int32_t) * n_mid));
    CG_TRY(alloc((void**)&big, sizeof(int32_t) * n_big));
    CG_TRY(alloc((void**)&hints, sizeof(int32_t) * (n_mid + n_big)));
    CG_TRY(hipMemsetAsync(hints, 0, sizeof(int32_t) * (n_mid + n_big), st));
    CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t) * 4, st));
    hipLaunchKernelGGL(k_cg_count_long, grid_of(n), kBlock, 0, st, a, n, mid, big);
  }
  CgArgs am = a, ab = a;
  am.rows = mid; am.passes_hint = hints;
  ab.rows = big; ab.passes_hint = hints + n_mid;

  int32_t it = 0, converged = 0;
  while (it < max_iters) {
    CG_TRY(hipMemsetAsync(counters, 0, sizeof(int32_t), st));
    a.salt = am.salt = ab.salt = (uint32_t)it * 0x9E3779B9u;
    hipLaunchKernelGGL(k_cg_propose_short, grid_of(n), kBlock, 0, st, a, n);
    if (n_mid > 0) hipLaunchKernelGGL((k_cg_propose_long<64, kMidSlots>), (unsigned)n_mid, 64, 0, st, am);
    if (n_big > 0) hipLaunchKernelGGL((k_cg_propose_long<kBlock, kBigSlots>), (unsigned)n_big, kBlock, 0, st, ab);
    hipLaunchKernelGGL(k_cg_decide_short, grid_of(n), kBlock, 0, st, a, n);
    if (n_mid > 0) hipLaunchKernelGGL(k_cg_decide_long<64>, (unsigned)n_mid, 64, 0, st, am);
    if (n_big > 0) hipLaunchKernelGGL(k_cg_decide_long<kBlock>, (unsigned)n_big, kBlock, 0, st, ab);
    CG_TRY(hipMemcpyAsync(host_c, counters, sizeof(host_c), hipMemcpyDeviceToHost, st));
    CG_TRY(hipStreamSynchronize(st));
    ++it;
    if (host_c[3]) { release(); return bad(DGC_ERR_UNSUPPORTED, "chunk generate: a label table overflowed"); }
    if (host_c[0] == 0) { converged = 1; break; }
  }
  CG_TRY(hipGetLastError());
  release();
#undef CG_TRY
  if (iters_out) *iters_out = it;
  if (converged_out) *converged_out = converged;
  return DGC_OK;
}
