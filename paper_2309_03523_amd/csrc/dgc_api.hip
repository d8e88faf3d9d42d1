// C ABI of libdgc: argument checks, packing at create time, and the launch sequence of the
// forward pass.  See include/dgc.h for the contract of every entry point.
#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <set>

#include "dgc_internal.h"

using namespace dgc;

namespace {

thread_local std::string g_create_error = "";

struct Param {
  float* raw = nullptr;       // device, [n_out][n_in] or [n]
  float4* packed = nullptr;   // device, fragment order (weights only)
  int32_t n_out = 0, n_in = 0;  // n_in = 0: a bias vector of n_out elements
  int64_t numel() const { return n_in ? (int64_t)n_out * n_in : n_out; }
};

}  // namespace

namespace dgc {
void set_thread_error(const std::string& msg) { g_create_error = msg; }
}  // namespace dgc

// Largest y / z extent of a launch grid: kernels that take one grid row per segment, chunk or snapshot
// are refused beyond it instead of failing at launch.
constexpr int64_t kMaxGridYZ = 65535;

struct dgc_layer {
  dgc_layer_desc_t desc{};
  int32_t T = 0;
  int64_t N = 0;
  int32_t n_chunks = 0;
  int64_t nseg = 0, total_rows = 0, total_nnz = 0, total_halo = 0, total_state_rows = 0;
  int64_t n_short = 0, n_long = 0, n_tiles = 0;
  int32_t rows_per_group = 16, long_nnz = 1024, part_nnz = 512;
  std::vector<dgc_chunk_t> chunks;
  std::vector<Segment> segs_host;
  std::vector<void*> allocs;          // everything hipMalloc'ed, freed in destroy
  // device
  const int64_t** d_rowptr = nullptr;
  const int32_t** d_colidx = nullptr;
  Segment* d_segs = nullptr;
  ChunkInfo* d_chunks = nullptr;
  DenseTile* d_tiles = nullptr;
  DenseTile* d_tiles32 = nullptr;
  int64_t n_tiles32 = 0;
  float* d_dinv = nullptr;
  int64_t* d_halo_ptr = nullptr;
  int32_t* d_halo_idx = nullptr;
  int32_t* d_col_local = nullptr;
  int32_t* d_work_short = nullptr;
  int32_t* d_work_long = nullptr;
  int2* d_etab = nullptr;                        // edge table of the aggregation kernels (see SpmmArgs)
  float* d_M = nullptr; int64_t ldm = 0;         // aggregated rows of the current GCN layer
  float* d_partial = nullptr;                    // split-row partial sums
  float* d_halo = nullptr; int64_t ld_halo = 0;  // STAGED: gathered cache rows
  float* d_Z1 = nullptr;                         // 2 layers: first layer's output [T,N,S]
  float* d_zero_bias = nullptr;                  // [S] zeros (EvolveGCN-O has no bias)
  EvolveWs evo{};                                // EvolveGCN-O workspace
  DysatWs dy{};                                  // graph attention + temporal attention workspace
  hipEvent_t evd[8] = {};                        // its stage boundaries: forward 0..3, backward 4..7
  bool evd_fwd = false, evd_bwd = false;
  TFusion tf{};                                  // temporal-fusion packing (dgc_layer_set_presence)
  Labelled lab{};                                // generated chunks (dgc_layer_set_labels)
  // input-gradient pass of EvolveGCN-O, allocated by the first backward that asks for dX
  float* d_dM = nullptr;                         // [T*N][F] gradient of the aggregated rows
  int64_t* d_rowidx = nullptr;                   // [total rows] packed row -> t*N + v
  float4* d_Wt_plain = nullptr;                  // every W_t as (out = F, in = S) fragments
  bool m_saved = false;                          // d_M holds the aggregated rows of the last forward
  unsigned long long* fs_mask = nullptr;         // loader bitmap and pair counters of dgc_layer_shared_rows,
  unsigned long long* fs_out = nullptr;          // allocated by its first call
  std::vector<ChunkInfo> cinfo_host;
  bool has_grads = false;
  std::map<std::string, Param> params;
  bool forward_done = false;
  bool profiling = false;
  hipEvent_t ev[DGC_N_STAGES + 1] = {};   // forward: boundaries of stages 0..3
  hipEvent_t evx[6] = {};                 // pairs around stage 4 (weight evolution), 5 and 6 (backward)
  bool ev_valid = false, evx_fwd = false, evx_bwd = false;
  std::string error;

  GraphDev graph_dev() const { return GraphDev{T, N, d_rowptr, d_colidx}; }
};

namespace {

dgc_status_t fail_create(dgc_status_t code, const std::string& msg) {
  g_create_error = msg;
  return code;
}

struct Failer {
  dgc_layer* L;
  dgc_status_t operator()(dgc_status_t code, const std::string& msg) const {
    if (L) L->error = msg; else g_create_error = msg;
    return code;
  }
};

template <class T>
hipError_t dev_alloc(dgc_layer* L, T** p, int64_t count) {
  *p = nullptr;
  if (count <= 0) count = 1;
  void* v = nullptr;
  hipError_t e = hipMalloc(&v, (size_t)count * sizeof(T));
  if (e == hipSuccess) {
    L->allocs.push_back(v);
    *p = static_cast<T*>(v);
  }
  return e;
}

template <class T>
void dev_free(dgc_layer* L, T* p) {
  if (!p) return;
  auto it = std::find(L->allocs.begin(), L->allocs.end(), static_cast<void*>(p));
  if (it != L->allocs.end()) L->allocs.erase(it);
  (void)hipFree(p);
}

void free_all(dgc_layer* L) {
  for (void* p : L->allocs) (void)hipFree(p);
  L->allocs.clear();
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

dgc_status_t check_desc(const dgc_layer_desc_t& d, std::string* msg) {
  if (d.struct_kind != DGC_STRUCT_GCN && d.struct_kind != DGC_STRUCT_EVOLVE_GCN_O && d.struct_kind != DGC_STRUCT_GAT) {
    *msg = "unknown struct_kind"; return DGC_ERR_INVALID_ARG;
  }
  const bool gat = d.struct_kind == DGC_STRUCT_GAT;
  if (gat != (d.time_kind == DGC_TIME_SELF_ATTN) || gat != (d.dtype == DGC_DTYPE_BF16)) {
    *msg = "DGC_STRUCT_GAT, DGC_TIME_SELF_ATTN and DGC_DTYPE_BF16 are built only together";
    return DGC_ERR_UNSUPPORTED;
  }
  if (gat) {
    if (d.F != 128 || d.S != 128 || d.heads != 8 || d.n_struct_layers != 1) {
      *msg = "the graph attention layer is built for F = S = 128, heads = 8, one layer"; return DGC_ERR_UNSUPPORTED;
    }
    if (d.validate_level < 0 || d.validate_level > 1) { *msg = "validate_level must be 0 or 1"; return DGC_ERR_INVALID_ARG; }
    if (d.rows_per_group < 0 || d.rows_per_group > 32) { *msg = "rows_per_group must be in [0,32]"; return DGC_ERR_INVALID_ARG; }
    if (d.long_nnz < 0 || d.part_nnz < 0) { *msg = "long_nnz / part_nnz must be >= 0"; return DGC_ERR_INVALID_ARG; }
    if (d.lstm_input_concat) { *msg = "lstm_input_concat needs a GCN + LSTM layer"; return DGC_ERR_INVALID_ARG; }
    return DGC_OK;
  }
  if (d.struct_kind == DGC_STRUCT_EVOLVE_GCN_O &&
      (d.time_kind != DGC_TIME_NONE || d.n_struct_layers != 1 || d.F != d.S || d.act_out != DGC_ACT_RELU)) {
    *msg = "EvolveGCN-O needs time_kind NONE, one layer, F = S and act_out RELU"; return DGC_ERR_INVALID_ARG;
  }
  if (d.dtype != DGC_DTYPE_F32) { *msg = "unknown dtype"; return DGC_ERR_INVALID_ARG; }
  if (d.n_struct_layers < 1 || d.n_struct_layers > 2) { *msg = "n_struct_layers must be 1 or 2"; return DGC_ERR_INVALID_ARG; }
  if (d.time_kind < DGC_TIME_NONE || d.time_kind > DGC_TIME_LSTM) { *msg = "unknown time_kind"; return DGC_ERR_INVALID_ARG; }
  if (d.F < 1 || d.F > 512) { *msg = "F must be in [1,512]"; return DGC_ERR_INVALID_ARG; }
  if (d.S < 32 || d.S > 256 || d.S % 32) { *msg = "S must be a multiple of 32 in [32,256]"; return DGC_ERR_INVALID_ARG; }
  if (d.time_kind != DGC_TIME_NONE && (d.H < 32 || d.H > 256 || d.H % 32)) {
    *msg = "H must be a multiple of 32 in [32,256]"; return DGC_ERR_INVALID_ARG;
  }
  for (int32_t act : {d.act_hidden, d.act_out})
    if (act != DGC_ACT_NONE && act != DGC_ACT_RELU) { *msg = "unknown activation"; return DGC_ERR_INVALID_ARG; }
  if (d.gather_mode != DGC_GATHER_IN_PLACE && d.gather_mode != DGC_GATHER_STAGED) { *msg = "unknown gather_mode"; return DGC_ERR_INVALID_ARG; }
  if (d.validate_level < 0 || d.validate_level > 1) { *msg = "validate_level must be 0 or 1"; return DGC_ERR_INVALID_ARG; }
  if (d.rows_per_group < 0 || d.rows_per_group > 32) { *msg = "rows_per_group must be in [0,32]"; return DGC_ERR_INVALID_ARG; }
  if (d.dense_kernel < DGC_DENSE_AUTO || d.dense_kernel > DGC_DENSE_WAVE) { *msg = "unknown dense_kernel"; return DGC_ERR_INVALID_ARG; }
  if (d.long_nnz < 0 || d.part_nnz < 0) { *msg = "long_nnz / part_nnz must be >= 0"; return DGC_ERR_INVALID_ARG; }
  // Where the workgroup-tile kernel runs a dense stage, its operand tile must fit the 160 KB of LDS.
  auto tile_kernel_runs = [&](int32_t S, int32_t H, int32_t kind) {
    const bool s_ok = S == 32 || S == 64 || S == 128 || (S == 256 && kind == DGC_TIME_NONE);
    return d.dense_kernel == DGC_DENSE_TILE || !(s_ok && (kind == DGC_TIME_NONE || H == S));
  };
  auto fits = [&](int32_t K0, int32_t S, int32_t H, int32_t kind) {
    return !tile_kernel_runs(S, H, kind) || dense_lds_bytes(K0, S, kind == DGC_TIME_NONE ? 0 : H) <= 160 * 1024;
  };
  if (d.agg_kernel < DGC_AGG_TABLE || d.agg_kernel > DGC_AGG_WALK) { *msg = "unknown agg_kernel"; return DGC_ERR_INVALID_ARG; }
  if (d.lstm_input_concat < 0 || d.lstm_input_concat > 1) { *msg = "lstm_input_concat must be 0 or 1"; return DGC_ERR_INVALID_ARG; }
  if (d.lstm_input_concat) {
    if (d.struct_kind != DGC_STRUCT_GCN || d.n_struct_layers != 2 || d.time_kind != DGC_TIME_LSTM) {
      *msg = "lstm_input_concat needs two GCN layers and the LSTM"; return DGC_ERR_INVALID_ARG;
    }
    if (tile_kernel_runs(d.S, d.H, d.time_kind)) {
      *msg = "lstm_input_concat is built in the wave-private dense kernel: S = H in {32, 64, 128}, dense_kernel not DGC_DENSE_TILE";
      return DGC_ERR_UNSUPPORTED;
    }
  }
  if (d.n_time_layers < 0 || d.n_time_layers > 2) { *msg = "n_time_layers must be 0, 1 or 2"; return DGC_ERR_INVALID_ARG; }
  if (d.n_time_layers == 2) {
    if (d.struct_kind != DGC_STRUCT_GCN || (d.time_kind != DGC_TIME_GRU && d.time_kind != DGC_TIME_LSTM)) {
      *msg = "a stacked time encoder needs a GCN layer with a GRU or LSTM"; return DGC_ERR_INVALID_ARG;
    }
    if (tile_kernel_runs(d.S, d.H, d.time_kind)) {
      *msg = "the stacked time encoder is built in the wave-private dense kernel: S = H in {32, 64, 128}, dense_kernel not DGC_DENSE_TILE";
      return DGC_ERR_UNSUPPORTED;
    }
  }
  const bool two = d.n_struct_layers == 2;
  if (!fits(two ? d.S : d.F, d.S, d.H, d.time_kind) || (two && !fits(d.F, d.S, 0, DGC_TIME_NONE))) {
    *msg = "these dimensions need the workgroup-tile kernel, whose tile holds max(F rounded up to 8, S, H) <= 304 columns";
    return DGC_ERR_UNSUPPORTED;
  }
  return DGC_OK;
}

// Chunks: non-empty, inside the graph, pairwise disjoint in (vertex, snapshot) space.
dgc_status_t check_chunks(const dgc_chunk_t* c, int32_t n, int32_t T, int64_t N, std::string* msg) {
  for (int32_t k = 0; k < n; ++k) {
    if (c[k].v_lo < 0 || c[k].v_hi > N || c[k].v_lo >= c[k].v_hi || c[k].t_lo < 0 || c[k].t_hi > T ||
        c[k].t_lo >= c[k].t_hi) {
      *msg = "chunk " + std::to_string(k) + " is empty or outside the graph";
      return DGC_ERR_BAD_CHUNK;
    }
    if (c[k].v_hi - c[k].v_lo > INT32_MAX) { *msg = "chunk too wide"; return DGC_ERR_BAD_CHUNK; }
  }
  // sweep over vertex starts; compare each chunk with the ones whose vertex range is still open
  std::vector<int32_t> order(n);
  for (int32_t k = 0; k < n; ++k) order[k] = k;
  std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return c[a].v_lo < c[b].v_lo; });
  std::vector<int32_t> open;
  for (int32_t k : order) {
    open.erase(std::remove_if(open.begin(), open.end(), [&](int32_t o) { return c[o].v_hi <= c[k].v_lo; }),
               open.end());
    for (int32_t o : open)
      if (c[o].t_lo < c[k].t_hi && c[k].t_lo < c[o].t_hi) {
        *msg = "chunks " + std::to_string(o) + " and " + std::to_string(k) + " overlap";
        return DGC_ERR_BAD_CHUNK;
      }
    open.push_back(k);
  }
  return DGC_OK;
}

dgc_status_t add_param(dgc_layer* L, const std::string& name, int32_t n_out, int32_t n_in, hipStream_t st) {
  Failer fail{L};
  Param p;
  p.n_out = n_out; p.n_in = n_in;
  DGC_HIP_TRY(dev_alloc(L, &p.raw, p.numel()));
  DGC_HIP_TRY(hipMemsetAsync(p.raw, 0, sizeof(float) * p.numel(), st));
  if (n_in) {
    const int64_t pe = packed_weight_elems(n_out, n_in);
    float* pk = nullptr;
    DGC_HIP_TRY(dev_alloc(L, &pk, pe));
    DGC_HIP_TRY(hipMemsetAsync(pk, 0, sizeof(float) * pe, st));
    p.packed = reinterpret_cast<float4*>(pk);
  }
  L->params[name] = p;
  return DGC_OK;
}

const char* const kEvolveNames[EV_NPAR] = {"evolve.W_init", "evolve.U_z", "evolve.V_z", "evolve.B_z", "evolve.U_r",
                                           "evolve.V_r",    "evolve.B_r", "evolve.U_h", "evolve.V_h", "evolve.B_h"};

// EvolveGCN-O: parameters, their gradients, the evolved weights and the per-snapshot tile lists
dgc_status_t build_evolve(dgc_layer* L, const std::vector<ChunkInfo>& cinfo, hipStream_t st) {
  Failer fail{L};
  const int32_t T = L->T, F = L->desc.F, S = L->desc.S;
  const int64_t n = (int64_t)F * S;
  EvolveWs& ev = L->evo;
  ev.T = T; ev.F = F; ev.S = S;
  for (int k = 0; k < EV_NPAR; ++k) {
    const bool fs = (k == EV_W || k == EV_BZ || k == EV_BR || k == EV_BH);
    Param p;                      // stored as [rows][cols] with n_out = rows, n_in = cols; never packed
    p.n_out = F; p.n_in = fs ? S : F;
    DGC_HIP_TRY(dev_alloc(L, &p.raw, p.numel()));
    DGC_HIP_TRY(hipMemsetAsync(p.raw, 0, sizeof(float) * p.numel(), st));
    L->params[kEvolveNames[k]] = p;
    ev.P[k] = p.raw;
    Param g = p;
    DGC_HIP_TRY(dev_alloc(L, &g.raw, g.numel()));
    DGC_HIP_TRY(hipMemsetAsync(g.raw, 0, sizeof(float) * g.numel(), st));
    L->params[std::string(kEvolveNames[k]) + ".grad"] = g;
    ev.G[k] = g.raw;
    DGC_HIP_TRY(dev_alloc(L, &ev.Pd[k], n));
    DGC_HIP_TRY(dev_alloc(L, &ev.Gd[k], n));
  }
  DGC_HIP_TRY(dev_alloc(L, &ev.Wt_f32, T * n));
  DGC_HIP_TRY(dev_alloc(L, &ev.Wt, T * n));
  DGC_HIP_TRY(dev_alloc(L, &ev.Zg, T * n));
  DGC_HIP_TRY(dev_alloc(L, &ev.Rg, T * n));
  DGC_HIP_TRY(dev_alloc(L, &ev.Wc, T * n));
  float* pk = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &pk, (int64_t)T * packed_weight_elems(S, F)));
  ev.Wt_packed = reinterpret_cast<float4*>(pk);
  for (double*& t : ev.tmp) DGC_HIP_TRY(dev_alloc(L, &t, n));
  DGC_HIP_TRY(dev_alloc(L, &ev.dWd, T * n));
  DGC_HIP_TRY(dev_alloc(L, &ev.partial, evolve_partial_elems(T, F, S)));
  DGC_HIP_TRY(dev_alloc(L, &ev.loss_partial, evolve_loss_partial_elems(T)));
  DGC_HIP_TRY(dev_alloc(L, &L->d_zero_bias, S));
  DGC_HIP_TRY(hipMemsetAsync(L->d_zero_bias, 0, sizeof(float) * S, st));
  // 32-row tiles of every snapshot, snapshot by snapshot, chunks in order
  std::vector<DenseTile> items;
  std::vector<int64_t> ptr(T + 1, 0);
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t k = 0; k < L->n_chunks; ++k) {
      if (t < cinfo[k].t_lo || t >= cinfo[k].t_lo + cinfo[k].w) continue;
      for (int64_t v0 = 0; v0 < cinfo[k].nv; v0 += kWaveTileRows)
        items.push_back(DenseTile{k, (int32_t)v0, (int32_t)std::min<int64_t>(kWaveTileRows, cinfo[k].nv - v0), 0});
    }
    ptr[t + 1] = (int64_t)items.size();
  }
  DenseTile* d_items = nullptr;
  int64_t* d_ptr = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_items, (int64_t)items.size()));
  DGC_HIP_TRY(dev_alloc(L, &d_ptr, T + 1));
  DGC_HIP_TRY(hipMemcpyAsync(d_items, items.data(), sizeof(DenseTile) * items.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(d_ptr, ptr.data(), sizeof(int64_t) * (T + 1), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  ev.items = d_items; ev.item_ptr = d_ptr;
  return DGC_OK;
}

const char* const kDysatNames[DY_NPAR] = {"gat.weight", "gat.att_src", "gat.att_dst", "attn.pos",
                                          "attn.weight_q", "attn.weight_k", "attn.weight_v"};

// graph attention + temporal self-attention: parameters, operand fragments, workspace
dgc_status_t build_dysat(dgc_layer* L, const std::vector<ChunkInfo>& cinfo, hipStream_t st) {
  Failer fail{L};
  const int32_t T = L->T, S = L->desc.S, heads = L->desc.heads;
  const int64_t N = L->N, TN = (int64_t)T * N;
  DysatWs& w = L->dy;
  w.T = T; w.N = N; w.n_chunks = L->n_chunks;
  w.g = L->graph_dev(); w.segs = L->d_segs; w.nseg = L->nseg; w.chunks = L->d_chunks;
  w.work_short = L->d_work_short; w.n_short = L->n_short; w.total_rows = L->total_rows;
  w.wide = false;
  for (const ChunkInfo& c : cinfo) {
    if (c.w > 32) return fail(DGC_ERR_UNSUPPORTED, "the temporal self-attention is built for windows of at most 32 snapshots");
    if (c.w > 16) w.wide = true;     // one vertex per 32-row tile instead of two
  }
  if (L->T > 4096) return fail(DGC_ERR_UNSUPPORTED, "the attention layer is built for at most 4096 snapshots");
  const int32_t rows_of[DY_NPAR] = {S, heads, heads, T, S, S, S};
  const int32_t cols_of[DY_NPAR] = {S, S / heads, S / heads, S, S, S, S};
  for (int k = 0; k < DY_NPAR; ++k) {
    Param p;
    p.n_out = rows_of[k]; p.n_in = cols_of[k];
    DGC_HIP_TRY(dev_alloc(L, &p.raw, p.numel()));
    DGC_HIP_TRY(hipMemsetAsync(p.raw, 0, sizeof(float) * p.numel(), st));
    L->params[kDysatNames[k]] = p;
    w.P[k] = p.raw;
    Param g = p;
    DGC_HIP_TRY(dev_alloc(L, &g.raw, g.numel()));
    DGC_HIP_TRY(hipMemsetAsync(g.raw, 0, sizeof(float) * g.numel(), st));
    L->params[std::string(kDysatNames[k]) + ".grad"] = g;
    w.G[k] = g.raw;
  }
  uint4** frags[9] = {&w.Wp, &w.Wqp, &w.Wkp, &w.Wvp, &w.WqT, &w.WkT, &w.WvT, &w.WT, &w.WTlo};
  for (uint4** f : frags) DGC_HIP_TRY(dev_alloc(L, f, 4 * 8 * 64));
  // snapshots in use, tiles of the temporal kernels per chunk, owner map
  std::vector<int32_t> used;
  {
    std::vector<char> seen(T, 0);
    for (const ChunkInfo& c : cinfo)
      for (int32_t t = c.t_lo; t < c.t_lo + c.w; ++t) seen[t] = 1;
    for (int32_t t = 0; t < T; ++t)
      if (seen[t]) used.push_back(t);
  }
  std::vector<int64_t> tptr(L->n_chunks + 1, 0);
  for (int32_t k = 0; k < L->n_chunks; ++k) tptr[k + 1] = tptr[k] + (w.wide ? cinfo[k].nv : (cinfo[k].nv + 1) / 2);
  w.n_used = (int32_t)used.size(); w.n_tiles = tptr.back();
  int32_t *d_used = nullptr, *d_owner = nullptr;
  int64_t* d_tptr = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_used, (int64_t)used.size()));
  DGC_HIP_TRY(dev_alloc(L, &d_tptr, (int64_t)tptr.size()));
  DGC_HIP_TRY(dev_alloc(L, &d_owner, TN));
  DGC_HIP_TRY(hipMemcpyAsync(d_used, used.data(), sizeof(int32_t) * used.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(d_tptr, tptr.data(), sizeof(int64_t) * tptr.size(), hipMemcpyHostToDevice, st));
  dysat_build_owner(L->d_segs, L->nseg, T, N, d_owner, st);
  DGC_HIP_TRY(hipStreamSynchronize(st));
  w.used_t = d_used; w.tile_ptr = d_tptr; w.owner = d_owner;
  uint16_t** rowbufs[8] = {&w.zX, &w.zC, &w.dU, &w.dQ, &w.dK, &w.dV, &w.dzX, &w.dzC};
  for (uint16_t** b : rowbufs) DGC_HIP_TRY(dev_alloc(L, b, TN * S));
  DGC_HIP_TRY(dev_alloc(L, &w.U, TN * S));
  DGC_HIP_TRY(dev_alloc(L, &w.sX, TN * 16));
  DGC_HIP_TRY(dev_alloc(L, &w.sC, TN * 8));
  DGC_HIP_TRY(dev_alloc(L, &w.lse, TN * 8));
  DGC_HIP_TRY(dev_alloc(L, &w.st2, TN * 32));
  DGC_HIP_TRY(dev_alloc(L, &w.dss, TN * 16));
  // split rows: those of the covered rows come from the packing; the reverse-edge pass walks every
  // vertex of the snapshots in use and gets its own list
  w.long_nnz = L->long_nnz; w.part_nnz = L->part_nnz;
  w.work_long = L->d_work_long; w.n_long = L->n_long;
  {
    int32_t* d_cnt = nullptr;
    int32_t n_parts = 0;
    DGC_HIP_TRY(dev_alloc(L, &d_cnt, 1));
    DGC_HIP_TRY(hipMemsetAsync(d_cnt, 0, sizeof(int32_t), st));
    dysat_cols_long(w.g, w.used_t, w.n_used, w.long_nnz, w.part_nnz, d_cnt, nullptr, st);
    DGC_HIP_TRY(hipMemcpyAsync(&n_parts, d_cnt, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    DGC_HIP_TRY(hipStreamSynchronize(st));
    int32_t* d_list = nullptr;
    DGC_HIP_TRY(dev_alloc(L, &d_list, 4 * (int64_t)n_parts));
    DGC_HIP_TRY(hipMemsetAsync(d_cnt, 0, sizeof(int32_t), st));
    if (n_parts > 0) dysat_cols_long(w.g, w.used_t, w.n_used, w.long_nnz, w.part_nnz, d_cnt, d_list, st);
    DGC_HIP_TRY(hipStreamSynchronize(st));
    w.cols_long = d_list; w.n_cols_long = n_parts;
  }
  DGC_HIP_TRY(dev_alloc(L, &w.long_partial, dysat_long_partial_elems(w)));
  {
    // edge codes of the reverse-edge pass: one byte per stored non-zero of the snapshots in use
    std::vector<int64_t> off(T, 0);
    std::vector<const int64_t*> rp(T);
    DGC_HIP_TRY(hipMemcpy(rp.data(), L->d_rowptr, sizeof(void*) * T, hipMemcpyDeviceToHost));
    int64_t total = 0;
    for (int32_t t : used) {
      int64_t nnz = 0;
      DGC_HIP_TRY(hipMemcpy(&nnz, rp[t] + N, sizeof(int64_t), hipMemcpyDeviceToHost));
      off[t] = total;
      total += nnz;
    }
    int64_t* d_off = nullptr;
    uint8_t* d_code = nullptr;
    DGC_HIP_TRY(dev_alloc(L, &d_off, T));
    DGC_HIP_TRY(dev_alloc(L, &d_code, total));
    DGC_HIP_TRY(hipMemcpy(d_off, off.data(), sizeof(int64_t) * T, hipMemcpyHostToDevice));
    dysat_edge_code(w.g, w.used_t, w.n_used, w.owner, d_off, d_code, st);
    DGC_HIP_TRY(hipStreamSynchronize(st));
    w.ecode = d_code; w.ecode_off = d_off;
  }
  w.partial_elems = dysat_partial_elems(w);
  DGC_HIP_TRY(dev_alloc(L, &w.partial, w.partial_elems));
  DGC_HIP_TRY(dev_alloc(L, &w.loss_partial, dysat_loss_partial_elems(w)));
  dysat_pack_params(w, st);
  return DGC_OK;
}

dgc_status_t build_layer(dgc_layer* L, const dgc_graph_t* graph, hipStream_t st) {
  Failer fail{L};
  const dgc_layer_desc_t& d = L->desc;
  const int32_t T = L->T;
  const int64_t N = L->N;

  // graph pointer tables
  DGC_HIP_TRY(dev_alloc(L, &L->d_rowptr, T));
  DGC_HIP_TRY(dev_alloc(L, &L->d_colidx, T));
  DGC_HIP_TRY(hipMemcpyAsync(L->d_rowptr, graph->rowptr, sizeof(void*) * T, hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(L->d_colidx, graph->colidx, sizeof(void*) * T, hipMemcpyHostToDevice, st));
  const GraphDev g = L->graph_dev();

  int32_t* d_flags = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_flags, 4));
  DGC_HIP_TRY(hipMemsetAsync(d_flags, 0, sizeof(int32_t) * 4, st));
  launch_validate_rowptr(g, d_flags, st);
  int32_t flags[4] = {0, 0, 0, 0};
  DGC_HIP_TRY(hipMemcpyAsync(flags, d_flags, sizeof(flags), hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  if (flags[0]) return fail(DGC_ERR_BAD_GRAPH, "rowptr does not start at 0 or decreases");
  if (d.validate_level >= 1) {
    launch_validate_graph(g, d_flags, st);
    DGC_HIP_TRY(hipMemcpyAsync(flags, d_flags, sizeof(flags), hipMemcpyDeviceToHost, st));
    DGC_HIP_TRY(hipStreamSynchronize(st));
    if (flags[0]) return fail(DGC_ERR_BAD_GRAPH, "rowptr does not start at 0 or decreases");
    if (flags[1]) return fail(DGC_ERR_BAD_GRAPH, "a column index is out of range, unsorted or duplicated");
    if (flags[2]) return fail(DGC_ERR_BAD_GRAPH, "a vertex has no stored self-loop");
    if (flags[3]) return fail(DGC_ERR_BAD_GRAPH, "the adjacency is not symmetric");
  }

  // segments: (chunk as given, snapshot ascending)
  std::vector<Segment>& segs = L->segs_host;
  std::vector<ChunkInfo> cinfo(L->n_chunks);
  int64_t row_off = 0, state_off = 0;
  for (int32_t k = 0; k < L->n_chunks; ++k) {
    const dgc_chunk_t& c = L->chunks[k];
    cinfo[k] = ChunkInfo{c.v_lo, c.v_hi - c.v_lo, row_off, state_off, c.t_lo, c.t_hi - c.t_lo};
    for (int32_t t = c.t_lo; t < c.t_hi; ++t) {
      Segment s{};
      s.row_off = row_off; s.v_lo = c.v_lo; s.v_hi = c.v_hi; s.t = t; s.chunk = k;
      segs.push_back(s);
      row_off += c.v_hi - c.v_lo;
    }
    state_off += c.v_hi - c.v_lo;
  }
  L->cinfo_host = cinfo;
  L->nseg = (int64_t)segs.size();
  L->total_rows = row_off;
  L->total_state_rows = state_off;
  if (L->nseg > INT32_MAX) return fail(DGC_ERR_UNSUPPORTED, "too many segments");
  DGC_HIP_TRY(dev_alloc(L, &L->d_segs, L->nseg));
  DGC_HIP_TRY(hipMemcpyAsync(L->d_segs, segs.data(), sizeof(Segment) * L->nseg, hipMemcpyHostToDevice, st));
  launch_segment_bounds(g, L->d_segs, L->nseg, st);
  DGC_HIP_TRY(hipMemcpyAsync(segs.data(), L->d_segs, sizeof(Segment) * L->nseg, hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  int64_t nnz_off = 0;
  for (Segment& s : segs) {
    const int64_t nnz = s.nnz_off;  // the kernel left the count here
    if (nnz < 0) return fail(DGC_ERR_BAD_GRAPH, "negative segment size");
    s.nnz_off = nnz_off;
    nnz_off += nnz;
  }
  L->total_nnz = nnz_off;
  DGC_HIP_TRY(hipMemcpyAsync(L->d_segs, segs.data(), sizeof(Segment) * L->nseg, hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(dev_alloc(L, &L->d_chunks, L->n_chunks));
  DGC_HIP_TRY(hipMemcpyAsync(L->d_chunks, cinfo.data(), sizeof(ChunkInfo) * L->n_chunks, hipMemcpyHostToDevice, st));

  // degree scaling
  DGC_HIP_TRY(dev_alloc(L, &L->d_dinv, (int64_t)T * N));
  launch_deg_inv_sqrt(g, L->d_dinv, st);

  // halo lists: bitmap per segment -> ranks -> ids -> local columns
  const int64_t wps = (N + 31) / 32;
  const int64_t n_words = L->nseg * wps;
  uint32_t* d_bitmap = nullptr;
  int64_t *d_rank = nullptr, *d_tmp = nullptr, *d_total = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_bitmap, n_words));
  DGC_HIP_TRY(dev_alloc(L, &d_rank, n_words));
  DGC_HIP_TRY(dev_alloc(L, &d_tmp, std::max(scan_tmp_elems(n_words), scan_tmp_elems(L->total_rows))));
  DGC_HIP_TRY(dev_alloc(L, &d_total, 1));
  DGC_HIP_TRY(hipMemsetAsync(d_bitmap, 0, sizeof(uint32_t) * std::max<int64_t>(n_words, 1), st));
  launch_mark_halo(g, L->d_segs, L->nseg, L->total_nnz, wps, d_bitmap, d_flags, st);
  launch_popcount_words(d_bitmap, n_words, d_rank, st);
  launch_exclusive_scan(d_rank, n_words, d_tmp, d_total, st);
  DGC_HIP_TRY(hipMemcpyAsync(&L->total_halo, d_total, sizeof(int64_t), hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipMemcpyAsync(flags, d_flags, sizeof(flags), hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  if (flags[1]) return fail(DGC_ERR_BAD_GRAPH, "a column index is out of range");
  DGC_HIP_TRY(dev_alloc(L, &L->d_halo_ptr, L->nseg + 1));
  DGC_HIP_TRY(dev_alloc(L, &L->d_halo_idx, L->total_halo));
  DGC_HIP_TRY(dev_alloc(L, &L->d_col_local, L->total_nnz));
  launch_seg_halo_off(d_rank, L->nseg, wps, n_words, d_total, L->d_segs, L->d_halo_ptr, st);
  launch_fill_halo(d_bitmap, d_rank, L->nseg, wps, L->d_halo_idx, st);
  launch_col_local(g, L->d_segs, L->nseg, L->total_nnz, wps, d_bitmap, d_rank, L->d_col_local, st);
  DGC_HIP_TRY(hipMemcpyAsync(segs.data(), L->d_segs, sizeof(Segment) * L->nseg, hipMemcpyDeviceToHost, st));

  // work list: row groups (host arithmetic on the chunk table) and split rows (device)
  {
    // short list: snapshot by snapshot, so that concurrently resident waves gather from the
    // same snapshot's feature rows (cache locality); within a snapshot in chunk order
    std::vector<int32_t> ws;
    const int32_t R = L->rows_per_group;
    std::vector<int64_t> order(L->nseg);
    for (int64_t s = 0; s < L->nseg; ++s) order[s] = s;
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return segs[a].t < segs[b].t; });
    for (int64_t s : order) {
      const int64_t rows = segs[s].v_hi - segs[s].v_lo;
      for (int64_t r = 0; r < rows; r += R) {
        ws.push_back((int32_t)s);
        ws.push_back((int32_t)r);
        ws.push_back((int32_t)std::min<int64_t>(R, rows - r));
      }
    }
    L->n_short = (int64_t)ws.size() / 3;
    DGC_HIP_TRY(dev_alloc(L, &L->d_work_short, (int64_t)ws.size()));
    DGC_HIP_TRY(hipMemcpyAsync(L->d_work_short, ws.data(), sizeof(int32_t) * ws.size(), hipMemcpyHostToDevice, st));
    DGC_HIP_TRY(hipStreamSynchronize(st));  // ws goes out of scope
  }
  int64_t* d_cnt = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_cnt, L->total_rows));
  launch_long_count(g, L->d_segs, L->nseg, L->total_rows, L->long_nnz, L->part_nnz, d_cnt, st);
  launch_exclusive_scan(d_cnt, L->total_rows, d_tmp, d_total, st);
  DGC_HIP_TRY(hipMemcpyAsync(&L->n_long, d_total, sizeof(int64_t), hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  DGC_HIP_TRY(dev_alloc(L, &L->d_work_long, 4 * L->n_long));
  launch_long_fill(g, L->d_segs, L->nseg, L->total_rows, L->long_nnz, L->part_nnz, d_cnt, L->d_work_long, st);

  // aggregation kernels' edge table and launch order
  const bool gat_layer = d.struct_kind == DGC_STRUCT_GAT;
  if (!gat_layer && d.gather_mode == DGC_GATHER_IN_PLACE && d.agg_kernel != DGC_AGG_WALK) {
    if (dev_alloc(L, &L->d_etab, L->total_nnz + kEtabPad) != hipSuccess)
      return fail(DGC_ERR_OOM, "no device memory for the aggregation's edge table (8 bytes per stored non-zero); "
                               "agg_kernel = DGC_AGG_WALK runs without it");
    launch_edge_table(g, L->d_segs, L->nseg, L->total_nnz, L->d_dinv, nullptr, L->d_etab, st);
  }

  // dense tiles: 64 consecutive vertices of a chunk
  {
    std::vector<DenseTile> tiles;
    for (int32_t k = 0; k < L->n_chunks; ++k)
      for (int64_t v0 = 0; v0 < cinfo[k].nv; v0 += kTileRows)
        tiles.push_back(DenseTile{k, (int32_t)v0, (int32_t)std::min<int64_t>(kTileRows, cinfo[k].nv - v0), 0});
    L->n_tiles = (int64_t)tiles.size();
    DGC_HIP_TRY(dev_alloc(L, &L->d_tiles, L->n_tiles));
    DGC_HIP_TRY(hipMemcpyAsync(L->d_tiles, tiles.data(), sizeof(DenseTile) * tiles.size(), hipMemcpyHostToDevice, st));
    std::vector<DenseTile> tiles32;
    for (int32_t k = 0; k < L->n_chunks; ++k)
      for (int64_t v0 = 0; v0 < cinfo[k].nv; v0 += kWaveTileRows)
        tiles32.push_back(DenseTile{k, (int32_t)v0, (int32_t)std::min<int64_t>(kWaveTileRows, cinfo[k].nv - v0), 0});
    L->n_tiles32 = (int64_t)tiles32.size();
    DGC_HIP_TRY(dev_alloc(L, &L->d_tiles32, L->n_tiles32));
    DGC_HIP_TRY(hipMemcpyAsync(L->d_tiles32, tiles32.data(), sizeof(DenseTile) * tiles32.size(), hipMemcpyHostToDevice, st));
    DGC_HIP_TRY(hipStreamSynchronize(st));
  }

  // workspace
  const int32_t Fmax = std::max(d.F, d.n_struct_layers == 2 ? d.S : 0);
  L->ldm = (Fmax + 7) / 8 * 8;  // whole k-blocks of 8; the aggregation zero-fills the pad columns
  const bool gat = d.struct_kind == DGC_STRUCT_GAT;
  if (!gat) {
    DGC_HIP_TRY(dev_alloc(L, &L->d_M, L->total_rows * L->ldm));
    DGC_HIP_TRY(dev_alloc(L, &L->d_partial, L->n_long * L->ldm));
  }
  if (!gat && d.gather_mode == DGC_GATHER_STAGED) {
    L->ld_halo = L->ldm;
    DGC_HIP_TRY(dev_alloc(L, &L->d_halo, L->total_halo * L->ld_halo));
  }
  if (d.n_struct_layers == 2) DGC_HIP_TRY(dev_alloc(L, &L->d_Z1, (int64_t)T * N * d.S));

  // parameters
  dgc_status_t rc;
  if (gat) {
    if ((rc = build_dysat(L, cinfo, st)) != DGC_OK) return rc;
  } else if (d.struct_kind == DGC_STRUCT_EVOLVE_GCN_O) {
    if ((rc = build_evolve(L, cinfo, st)) != DGC_OK) return rc;
  } else {
  if ((rc = add_param(L, "gcn0.weight", d.S, d.F, st)) != DGC_OK) return rc;
  if ((rc = add_param(L, "gcn0.bias", d.S, 0, st)) != DGC_OK) return rc;
  if (d.n_struct_layers == 2) {
    if ((rc = add_param(L, "gcn1.weight", d.S, d.S, st)) != DGC_OK) return rc;
    if ((rc = add_param(L, "gcn1.bias", d.S, 0, st)) != DGC_OK) return rc;
  }
  if (d.time_kind != DGC_TIME_NONE) {
    const int32_t gH = (d.time_kind == DGC_TIME_LSTM ? 4 : 3) * d.H;
    if ((rc = add_param(L, "rnn.weight_ih", gH, d.lstm_input_concat ? 2 * d.S : d.S, st)) != DGC_OK) return rc;
    if ((rc = add_param(L, "rnn.weight_hh", gH, d.H, st)) != DGC_OK) return rc;
    if ((rc = add_param(L, "rnn.bias_ih", gH, 0, st)) != DGC_OK) return rc;
    if ((rc = add_param(L, "rnn.bias_hh", gH, 0, st)) != DGC_OK) return rc;
    if (d.n_time_layers == 2) {
      if ((rc = add_param(L, "rnn1.weight_ih", gH, d.H, st)) != DGC_OK) return rc;
      if ((rc = add_param(L, "rnn1.weight_hh", gH, d.H, st)) != DGC_OK) return rc;
      if ((rc = add_param(L, "rnn1.bias_ih", gH, 0, st)) != DGC_OK) return rc;
      if ((rc = add_param(L, "rnn1.bias_hh", gH, 0, st)) != DGC_OK) return rc;
    }
  }
  }
  DGC_HIP_TRY(hipStreamSynchronize(st));
  DGC_HIP_TRY(hipGetLastError());
  // packing temporaries
  dev_free(L, d_bitmap); dev_free(L, d_rank); dev_free(L, d_tmp); dev_free(L, d_total);
  dev_free(L, d_cnt); dev_free(L, d_flags);
  return DGC_OK;
}

dgc_status_t check_tensor(const Failer& fail, const char* name, const void* p, int64_t ld, int64_t min_ld,
                          bool required, int64_t ld_multiple = 4) {
  if (!p) return required ? fail(DGC_ERR_INVALID_ARG, std::string(name) + " is NULL") : DGC_OK;
  if (!aligned16(p)) return fail(DGC_ERR_INVALID_ARG, std::string(name) + " is not 16-byte aligned");
  if (ld < min_ld || ld % ld_multiple)
    return fail(DGC_ERR_INVALID_ARG, std::string(name) + ": pitch too small or not a multiple of " + std::to_string(ld_multiple));
  return DGC_OK;
}

SpmmArgs spmm_args(dgc_layer* L, const float* fresh, int64_t ld_fresh, const float* stale, int64_t ld_stale,
                   int32_t F, float* M, int64_t ldm) {
  SpmmArgs a{};
  a.g = L->graph_dev();
  a.segs = L->d_segs;
  a.work_short = L->d_work_short; a.n_short = L->n_short;
  a.work_long = L->d_work_long; a.n_long = L->n_long;
  a.dinv = L->d_dinv;
  a.fresh = fresh; a.ld_fresh = ld_fresh;
  a.stale = stale; a.ld_stale = ld_stale;
  a.halo = nullptr; a.ld_halo = 0; a.col_local = nullptr;
  a.col_signed = L->lab.built ? L->lab.col_signed : nullptr;
  a.F = F;
  a.long_nnz = L->long_nnz; a.part_nnz = L->part_nnz;
  a.partial = L->d_partial;
  a.M = M; a.ldm = ldm;
  a.row_map = nullptr;
  a.ld_out = 0;
  a.skip_stale = false;
  a.etab = L->d_etab;
  return a;
}

// aggregation of one GCN layer, with or without the staged gather
void run_aggregate(dgc_layer* L, const float* fresh, int64_t ld_fresh, const float* stale, int64_t ld_stale,
                   int32_t F, float* M, int64_t ldm, hipStream_t st, const int64_t* row_map = nullptr) {
  SpmmArgs a = spmm_args(L, fresh, ld_fresh, stale, ld_stale, F, M, ldm);
  a.row_map = row_map;
  if (L->desc.gather_mode == DGC_GATHER_STAGED) {
    launch_gather(L->d_segs, L->nseg, L->d_halo_idx, L->d_halo_ptr, L->total_halo, L->N, stale, ld_stale, F,
                  L->d_halo, L->ld_halo, st);
    a.halo = L->d_halo; a.ld_halo = L->ld_halo; a.col_local = L->d_col_local;
  }
  launch_spmm(a, st);
}

// First-fit over lanes of `cap` slots: sequences come in packing order with their lengths; returns the
// number of lanes and fills lane / first slot of each.  by_free[f] = lanes with f free slots.
int32_t first_fit_lanes(const std::vector<int32_t>& lens, int32_t cap, std::vector<int32_t>* lane, std::vector<int32_t>* off) {
  std::vector<std::set<int32_t>> by_free(cap + 1);
  int32_t n_l = 0;
  lane->resize(lens.size()); off->resize(lens.size());
  for (size_t q = 0; q < lens.size(); ++q) {
    const int32_t n = lens[q];
    int32_t best = -1, bf = 0;
    for (int32_t f = n; f <= cap; ++f)
      if (!by_free[f].empty() && (best < 0 || *by_free[f].begin() < best)) { best = *by_free[f].begin(); bf = f; }
    if (best < 0) { best = n_l++; bf = cap; } else by_free[bf].erase(by_free[bf].begin());
    (*lane)[q] = best;
    (*off)[q] = cap - bf;
    by_free[bf - n].insert(best);
  }
  return n_l;
}

// Temporal fusion over generated chunks (the layer has labels): sequences are a vertex's runs of
// present instances with one label; all of them, ordered by (length descending, vertex ascending,
// first snapshot ascending), go first-fit into lanes of T slots.  The states keep the layout of the
// labelled layer: one row per (t, i), entering at a sequence's first instance, leaving at its last.
dgc_status_t set_presence_labelled(dgc_layer* L, const uint8_t* present, hipStream_t st) {
  Failer fail{L};
  TFusion& tf = L->tf;
  const int32_t T = L->T;
  const int64_t N = L->N, TN = (int64_t)T * N;
  int32_t *d_len = nullptr, *d_first = nullptr, *d_pos = nullptr;
  uint8_t* d_last = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_len, TN));
  DGC_HIP_TRY(dev_alloc(L, &d_first, TN));
  DGC_HIP_TRY(dev_alloc(L, &d_pos, TN));
  DGC_HIP_TRY(dev_alloc(L, &d_last, TN));
  lp_sequences(present, L->lab.labels, T, N, d_len, d_first, d_pos, d_last, st);
  std::vector<int32_t> len(TN);
  DGC_HIP_TRY(hipMemcpyAsync(len.data(), d_len, sizeof(int32_t) * len.size(), hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  // packing order by a counting sort on the length; within a length by vertex, then first snapshot
  std::vector<int64_t> count(T + 2, 0);
  for (int64_t x = 0; x < TN; ++x) count[len[x]]++;
  int64_t n_seq = TN - count[0];
  std::vector<int64_t> begin(T + 2, 0);     // sequences of length l start at begin[l]; longest first
  for (int32_t l = T - 1; l >= 1; --l) begin[l] = begin[l + 1] + count[l + 1];
  std::vector<int64_t> start_of(n_seq);
  std::vector<int32_t> lens(n_seq);
  for (int64_t i = 0; i < N; ++i)
    for (int32_t t = 0; t < T; ++t) {
      const int64_t x = (int64_t)t * N + i;
      if (len[x] > 0) { const int64_t q = begin[len[x]]++; start_of[q] = x; lens[q] = len[x]; }
    }
  std::vector<int32_t> lane_q, off_q;
  const int32_t n_l = first_fit_lanes(lens, T, &lane_q, &off_q);
  std::vector<int32_t> lane_of(TN, -1), off_of(TN, 0);
  for (int64_t q = 0; q < n_seq; ++q) { lane_of[start_of[q]] = lane_q[q]; off_of[start_of[q]] = off_q[q]; }
  tf.n_lanes = n_l; tf.Lmax = T; tf.rows_v = (int64_t)n_l * T;
  const int64_t n_slots = (int64_t)T * n_l;
  const std::vector<int64_t> lane_ptr = {0, n_l};
  const ChunkInfo cv{0, n_l, 0, 0, 0, T};
  int32_t *d_lane = nullptr, *d_off = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_lane, TN));
  DGC_HIP_TRY(dev_alloc(L, &d_off, TN));
  DGC_HIP_TRY(dev_alloc(L, &tf.lane_ptr, 2));
  DGC_HIP_TRY(dev_alloc(L, &tf.slot_row, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.slot_reset, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.seq_in, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.seq_out, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.row_map, TN));
  DGC_HIP_TRY(dev_alloc(L, &tf.chunks_v, 1));
  DGC_HIP_TRY(hipMemcpyAsync(d_lane, lane_of.data(), sizeof(int32_t) * lane_of.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(d_off, off_of.data(), sizeof(int32_t) * off_of.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(tf.lane_ptr, lane_ptr.data(), sizeof(int64_t) * 2, hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(tf.chunks_v, &cv, sizeof(ChunkInfo), hipMemcpyHostToDevice, st));
  lp_fill(present, d_first, d_pos, d_last, d_lane, d_off, T, N, n_l, tf.slot_row, tf.row_map, tf.slot_reset, tf.seq_in,
          tf.seq_out, st);
  std::vector<DenseTile> t64, t32;
  for (int64_t v0 = 0; v0 < n_l; v0 += kTileRows)
    t64.push_back(DenseTile{0, (int32_t)v0, (int32_t)std::min<int64_t>(kTileRows, n_l - v0), 0});
  for (int64_t v0 = 0; v0 < n_l; v0 += kWaveTileRows)
    t32.push_back(DenseTile{0, (int32_t)v0, (int32_t)std::min<int64_t>(kWaveTileRows, n_l - v0), 0});
  tf.n_tiles_v = (int64_t)t64.size(); tf.n_tiles32_v = (int64_t)t32.size();
  DGC_HIP_TRY(dev_alloc(L, &tf.tiles_v, tf.n_tiles_v));
  DGC_HIP_TRY(dev_alloc(L, &tf.tiles32_v, tf.n_tiles32_v));
  DGC_HIP_TRY(hipMemcpyAsync(tf.tiles_v, t64.data(), sizeof(DenseTile) * t64.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(tf.tiles32_v, t32.data(), sizeof(DenseTile) * t32.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(dev_alloc(L, &tf.Mv, tf.rows_v * L->ldm));
  DGC_HIP_TRY(hipMemsetAsync(tf.Mv, 0, sizeof(float) * (size_t)std::max<int64_t>(tf.rows_v * L->ldm, 1), st));  // empty slots stay zero
  DGC_HIP_TRY(hipStreamSynchronize(st));
  DGC_HIP_TRY(hipGetLastError());
  dev_free(L, d_len); dev_free(L, d_first); dev_free(L, d_pos); dev_free(L, d_last); dev_free(L, d_lane); dev_free(L, d_off);
  tf.built = true;
  L->forward_done = false;
  return DGC_OK;
}

}  // namespace

extern "C" {

const char* dgc_version(void) { return "dgc 0.1 gfx950"; }

const char* dgc_last_error(const dgc_layer_t* layer) {
  return layer ? layer->error.c_str() : g_create_error.c_str();
}

dgc_status_t dgc_layer_create(const dgc_layer_desc_t* desc, const dgc_graph_t* graph, const dgc_chunk_t* chunks,
                              int32_t n_chunks, void* stream, dgc_layer_t** out) {
  if (out) *out = nullptr;
  if (!desc || !graph || !chunks || !out) return fail_create(DGC_ERR_INVALID_ARG, "NULL argument");
  if (n_chunks < 1) return fail_create(DGC_ERR_INVALID_ARG, "n_chunks must be >= 1");
  if (graph->T < 1 || graph->N < 1 || !graph->rowptr || !graph->colidx)
    return fail_create(DGC_ERR_INVALID_ARG, "graph: T, N must be >= 1 and the pointer tables non-NULL");
  if (graph->N > INT32_MAX) return fail_create(DGC_ERR_UNSUPPORTED, "N must fit in int32 (column ids are int32)");
  for (int32_t t = 0; t < graph->T; ++t)
    if (!graph->rowptr[t] || !graph->colidx[t]) return fail_create(DGC_ERR_INVALID_ARG, "graph: NULL snapshot pointer");
  std::string msg;
  dgc_status_t rc = check_desc(*desc, &msg);
  if (rc != DGC_OK) return fail_create(rc, msg);
  rc = check_chunks(chunks, n_chunks, graph->T, graph->N, &msg);
  if (rc != DGC_OK) return fail_create(rc, msg);

  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) {
    (void)hipGetLastError();
    return fail_create(DGC_ERR_DEVICE, "no HIP device");
  }
  dgc_layer* L = new (std::nothrow) dgc_layer();
  if (!L) return fail_create(DGC_ERR_OOM, "host allocation failed");
  L->desc = *desc;
  L->T = graph->T; L->N = graph->N; L->n_chunks = n_chunks;
  L->chunks.assign(chunks, chunks + n_chunks);
  if (desc->rows_per_group) {
    L->rows_per_group = desc->rows_per_group;
  } else {
    // default 16 rows per wave; a small batch gets shorter groups (8, 4, 2, 1) until it makes at
    // least 8192 work items, so that its rows spread over the chip instead of queueing in few waves
    int64_t rows = 0;
    for (int32_t k = 0; k < n_chunks; ++k) rows += (chunks[k].v_hi - chunks[k].v_lo) * (int64_t)(chunks[k].t_hi - chunks[k].t_lo);
    while (L->rows_per_group > 1 && rows / L->rows_per_group < 8192) L->rows_per_group >>= 1;
  }
  if (desc->long_nnz) L->long_nnz = desc->long_nnz;
  if (desc->part_nnz) L->part_nnz = desc->part_nnz;
  rc = build_layer(L, graph, static_cast<hipStream_t>(stream));
  if (rc != DGC_OK) {
    g_create_error = L->error;
    if (rc == DGC_ERR_DEVICE && L->error.find("out of memory") != std::string::npos) rc = DGC_ERR_OOM;
    (void)hipGetLastError();
    free_all(L);
    delete L;
    return rc;
  }
  *out = L;
  return DGC_OK;
}

dgc_status_t dgc_layer_destroy(dgc_layer_t* L) {
  if (!L) return DGC_OK;
  (void)hipDeviceSynchronize();
  for (hipEvent_t e : L->ev)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : L->evx)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : L->evd)
    if (e) (void)hipEventDestroy(e);
  free_all(L);
  delete L;
  return DGC_OK;
}

dgc_status_t dgc_layer_set_param(dgc_layer_t* L, const char* name, const float* host_src, int64_t numel) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  if (!name || !host_src) return fail(DGC_ERR_INVALID_ARG, "NULL argument");
  auto it = L->params.find(name);
  if (it == L->params.end()) return fail(DGC_ERR_INVALID_ARG, std::string("unknown parameter ") + name);
  Param& p = it->second;
  const std::string nm(name);
  if (nm.size() > 5 && nm.compare(nm.size() - 5, 5, ".grad") == 0)
    return fail(DGC_ERR_INVALID_ARG, "gradients are read-only");
  if (numel != p.numel()) return fail(DGC_ERR_INVALID_ARG, std::string(name) + ": wrong element count");
  DGC_HIP_TRY(hipMemcpy(p.raw, host_src, sizeof(float) * numel, hipMemcpyHostToDevice));
  if (L->desc.struct_kind == DGC_STRUCT_GAT) {
    dysat_pack_params(L->dy, nullptr);
    DGC_HIP_TRY(hipDeviceSynchronize());
  } else if (p.packed) {
    launch_pack_weight(p.raw, p.n_out, p.n_in, p.packed, nullptr);
    DGC_HIP_TRY(hipDeviceSynchronize());
  }
  return DGC_OK;
}

dgc_status_t dgc_layer_get_param(dgc_layer_t* L, const char* name, float* host_dst, int64_t numel) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  if (!name || !host_dst) return fail(DGC_ERR_INVALID_ARG, "NULL argument");
  auto it = L->params.find(name);
  if (it == L->params.end()) return fail(DGC_ERR_INVALID_ARG, std::string("unknown parameter ") + name);
  if (numel != it->second.numel()) return fail(DGC_ERR_INVALID_ARG, std::string(name) + ": wrong element count");
  DGC_HIP_TRY(hipMemcpy(host_dst, it->second.raw, sizeof(float) * numel, hipMemcpyDeviceToHost));
  return DGC_OK;
}

dgc_status_t dgc_layer_aggregate(dgc_layer_t* L, const float* X, int64_t ldx, const float* C, int64_t ldc,
                                 float* M, int64_t ldm, void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  dgc_status_t rc;
  if (L->desc.struct_kind == DGC_STRUCT_GAT) return fail(DGC_ERR_UNSUPPORTED, "not a GCN layer");
  if ((rc = check_tensor(fail, "X", X, ldx, L->desc.F, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "C", C, ldc, L->desc.F, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "M", M, ldm, L->desc.F, true)) != DGC_OK) return rc;
  // the split-row scratch and the staged halo buffer are sized for pitch round_up(F,8)
  if (ldm > L->ldm) return fail(DGC_ERR_INVALID_ARG, "M: pitch must not exceed round_up(F,8)");
  run_aggregate(L, X, ldx, C, ldc, L->desc.F, M, ldm, static_cast<hipStream_t>(stream));
  DGC_HIP_TRY(hipGetLastError());
  return DGC_OK;
}

dgc_status_t dgc_layer_gather(dgc_layer_t* L, const float* C, int64_t ldc, float* halo, int64_t ldh, void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  dgc_status_t rc;
  if (L->desc.struct_kind == DGC_STRUCT_GAT) return fail(DGC_ERR_UNSUPPORTED, "not a GCN layer");
  if ((rc = check_tensor(fail, "C", C, ldc, L->desc.F, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "halo", halo, ldh, L->desc.F, true)) != DGC_OK) return rc;
  launch_gather(L->d_segs, L->nseg, L->d_halo_idx, L->d_halo_ptr, L->total_halo, L->N, C, ldc, L->desc.F, halo, ldh,
                static_cast<hipStream_t>(stream));
  DGC_HIP_TRY(hipGetLastError());
  return DGC_OK;
}

dgc_status_t dgc_layer_forward(dgc_layer_t* L, const void* Xv, int64_t ldx, const void* Cv, int64_t ldc,
                               const void* C1v, int64_t ldc1, const float* H0, const uint8_t* reset_mask, void* Yv,
                               int64_t ldy, float* HN, void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  const dgc_layer_desc_t& d = L->desc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  dgc_status_t rc;
  if (d.struct_kind == DGC_STRUCT_GAT) {
    if ((rc = check_tensor(fail, "X", Xv, ldx, d.F, true, 8)) != DGC_OK) return rc;
    if ((rc = check_tensor(fail, "C", Cv, ldc, d.F, true, 8)) != DGC_OK) return rc;
    if ((rc = check_tensor(fail, "Y", Yv, ldy, d.S, true, 8)) != DGC_OK) return rc;
    if (C1v || H0 || HN || reset_mask)
      return fail(DGC_ERR_INVALID_ARG, "C1 / H0 / HN / reset_mask do not apply to the attention layer");
    L->evd_fwd = false;
    L->dy.X = Xv; L->dy.ldx = ldx; L->dy.C = Cv; L->dy.ldc = ldc;
    dysat_forward(L->dy, Xv, ldx, Cv, ldc, Yv, ldy, L->profiling ? L->evd : nullptr, st);
    if (L->profiling) L->evd_fwd = true;
    DGC_HIP_TRY(hipGetLastError());
    L->forward_done = true;
    return DGC_OK;
  }
  const float* X = static_cast<const float*>(Xv);
  const float* C = static_cast<const float*>(Cv);
  const float* C1 = static_cast<const float*>(C1v);
  float* Y = static_cast<float*>(Yv);
  const int32_t out_dim = d.time_kind == DGC_TIME_NONE ? d.S : d.H;
  if ((rc = check_tensor(fail, "X", X, ldx, d.F, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "C", C, ldc, d.F, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "Y", Y, ldy, out_dim, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "C1", C1, ldc1, d.S, d.n_struct_layers == 2)) != DGC_OK) return rc;
  if (H0 && !aligned16(H0)) return fail(DGC_ERR_INVALID_ARG, "H0 is not 16-byte aligned");
  if (HN && !aligned16(HN)) return fail(DGC_ERR_INVALID_ARG, "HN is not 16-byte aligned");
  if (d.time_kind == DGC_TIME_NONE && (H0 || HN || reset_mask))
    return fail(DGC_ERR_INVALID_ARG, "H0 / HN / reset_mask need a time encoder");

  DenseArgs da{};
  da.tiles = L->d_tiles; da.n_tiles = L->n_tiles; da.chunks = L->d_chunks;
  da.tiles32 = L->d_tiles32; da.n_tiles32 = L->n_tiles32; da.variant = d.dense_kernel;
  da.N = L->N; da.total_state_rows = L->total_state_rows;
  da.M = L->d_M; da.ldm = L->ldm;
  da.S = d.S; da.H = d.H;
  std::string why;

  const bool prof = L->profiling;
  L->ev_valid = false;
  const bool evolve = d.struct_kind == DGC_STRUCT_EVOLVE_GCN_O;
  L->evx_fwd = false;
  if (evolve) {
    if (prof) DGC_HIP_TRY(hipEventRecord(L->evx[0], st));
    evolve_forward_weights(L->evo, st);
    if (prof) { DGC_HIP_TRY(hipEventRecord(L->evx[1], st)); L->evx_fwd = true; }
  }
  if (prof) DGC_HIP_TRY(hipEventRecord(L->ev[0], st));
  // with temporal fusion the aggregation that feeds the time encoder writes its rows in lane
  // order and skips the rows of absent vertices
  const bool tfl1 = L->tf.built && d.n_struct_layers == 1, tfl2 = L->tf.built && d.n_struct_layers == 2;
  run_aggregate(L, X, ldx, C, ldc, d.F, tfl1 ? L->tf.Mv : L->d_M, L->ldm, st, tfl1 ? L->tf.row_map : nullptr);
  if (prof) DGC_HIP_TRY(hipEventRecord(L->ev[1], st));
  const char* last = "gcn0";
  if (d.n_struct_layers == 2) {
    // first layer for every row of the batch -> Z1 [T,N,S]; then aggregate Z1 | C1
    da.K0 = d.F; da.act = d.act_hidden; da.time_kind = DGC_TIME_NONE;
    da.Wg = L->params["gcn0.weight"].packed; da.bg = L->params["gcn0.bias"].raw;
    da.wg_bytes = sizeof(float) * packed_weight_elems(d.S, d.F); da.wg_step_bytes = 0;
    da.Y = L->d_Z1; da.ldy = d.S;
    if (!launch_dense(da, st, &why)) return fail(DGC_ERR_UNSUPPORTED, why);
    if (prof) DGC_HIP_TRY(hipEventRecord(L->ev[2], st));
    run_aggregate(L, L->d_Z1, d.S, C1, ldc1, d.S, tfl2 ? L->tf.Mv : L->d_M, L->ldm, st, tfl2 ? L->tf.row_map : nullptr);
    if (prof) DGC_HIP_TRY(hipEventRecord(L->ev[3], st));
    last = "gcn1";
  } else if (prof) {
    DGC_HIP_TRY(hipEventRecord(L->ev[2], st));
    DGC_HIP_TRY(hipEventRecord(L->ev[3], st));
  }
  da.K0 = d.n_struct_layers == 2 ? d.S : d.F;
  da.act = d.act_out;
  da.time_kind = d.time_kind;
  if (evolve) {
    da.Wg = L->evo.Wt_packed;
    da.bg = L->d_zero_bias;
    da.wg_step_bytes = (int32_t)(sizeof(float) * packed_weight_elems(d.S, d.F));
    da.wg_bytes = (int64_t)L->T * da.wg_step_bytes;
  } else {
    da.Wg = L->params[std::string(last) + ".weight"].packed;
    da.bg = L->params[std::string(last) + ".bias"].raw;
    da.wg_bytes = sizeof(float) * packed_weight_elems(d.S, da.K0); da.wg_step_bytes = 0;
  }
  if (d.time_kind != DGC_TIME_NONE) {
    da.Wih = L->params["rnn.weight_ih"].packed; da.Whh = L->params["rnn.weight_hh"].packed;
    da.bih = L->params["rnn.bias_ih"].raw; da.bhh = L->params["rnn.bias_hh"].raw;
  }
  da.H0 = H0; da.reset_mask = reset_mask; da.Y = Y; da.ldy = ldy; da.HN = HN;
  if (d.lstm_input_concat) { da.X2 = L->d_Z1; da.ldx2 = d.S; }   // the LSTM reads [first layer's output, second layer's output]
  if (L->lab.built) {
    // generated chunks: a vertex's run of equal labels is a sequence; its state enters from H0's row
    // of (t, i) and leaves to HN's row of (t, i)
    if (reset_mask) return fail(DGC_ERR_INVALID_ARG, "with generated chunks reset_mask must be NULL");
    if (d.time_kind != DGC_TIME_NONE) { da.seq_in = L->lab.seq_in; da.seq_out = L->lab.seq_out; }
    da.total_state_rows = (int64_t)L->T * L->N;      // one state row per (t, i)
  }
  if (L->tf.built) {
    // temporal fusion: the dense + recurrent kernels over the lanes of every chunk with the
    // packing's reset flags, outputs back to their (snapshot, vertex) rows
    const TFusion& tf = L->tf;
    if (reset_mask) return fail(DGC_ERR_INVALID_ARG, "with temporal fusion reset_mask must be NULL");
    da.tiles = tf.tiles_v; da.n_tiles = tf.n_tiles_v; da.tiles32 = tf.tiles32_v; da.n_tiles32 = tf.n_tiles32_v;
    da.chunks = tf.chunks_v; da.N = tf.n_lanes;
    da.M = tf.Mv;
    da.y_map = tf.slot_row;       // a slot's output goes straight to its (snapshot, vertex) row of Y
    // every sequence starts from its own row of H0 (zero without H0) and leaves its final state in its
    // row of HN: the states travel through the slot tables; H0 / HN keep the layout they have without fusion
    da.reset_mask = nullptr; da.seq_in = tf.seq_in; da.seq_out = tf.seq_out;
    // (over generated chunks the states are the labelled layer's: one row per (t, i), only the rows
    // where a sequence starts are read and only those where one ends are written)
    da.total_state_rows = L->lab.built ? (int64_t)L->T * L->N : L->total_state_rows;
    da.x2_map = tf.slot_row;      // a slot's row of the first layer's output
    if (HN && !L->lab.built) tf_carry(tf.seq_len, L->total_state_rows, d.time_kind == DGC_TIME_LSTM ? 2 : 1, d.H, H0, HN, st);
    if (tf.n_lanes > 0 && !launch_dense(da, st, &why)) return fail(DGC_ERR_UNSUPPORTED, why);
  } else if (!launch_dense(da, st, &why)) return fail(DGC_ERR_UNSUPPORTED, why);
  if (d.n_time_layers == 2) {
    // The second recurrent layer: the same kernel without a transform, its input rows the first
    // layer's output, read from Y row by row one step before the row is overwritten with the second
    // layer's output; its states are the blocks of H0 / HN behind the first layer's.
    // (over lanes or generated chunks the sequence tables stay as they are: the second layer's
    //  sequences are the first one's)
    const int32_t n_st = d.time_kind == DGC_TIME_LSTM ? 2 : 1;
    const int64_t block = (int64_t)n_st * da.total_state_rows * d.H;
    da.M = Y; da.ldm = ldy; da.m_by_vertex = true; da.input_is_z = true; da.K0 = 0;
    da.Wih = L->params["rnn1.weight_ih"].packed; da.Whh = L->params["rnn1.weight_hh"].packed;
    da.bih = L->params["rnn1.bias_ih"].raw; da.bhh = L->params["rnn1.bias_hh"].raw;
    da.Wg = da.Wih; da.wg_bytes = sizeof(float) * packed_weight_elems((d.time_kind == DGC_TIME_LSTM ? 4 : 3) * d.H, d.H);
    da.wg_step_bytes = 0; da.act = DGC_ACT_NONE;
    da.X2 = nullptr; da.x2_map = nullptr;
    da.H0 = H0 ? H0 + block : nullptr; da.HN = HN ? HN + block : nullptr;
    if (L->tf.built && HN && !L->lab.built)
      tf_carry(L->tf.seq_len, L->total_state_rows, n_st, d.H, da.H0, da.HN, st);
    if ((!L->tf.built || L->tf.n_lanes > 0) && !launch_dense(da, st, &why)) return fail(DGC_ERR_UNSUPPORTED, why);
  }
  if (prof) {
    DGC_HIP_TRY(hipEventRecord(L->ev[4], st));
    L->ev_valid = true;
  }
  DGC_HIP_TRY(hipGetLastError());
  L->forward_done = true;
  L->m_saved = true;
  return DGC_OK;
}

dgc_status_t dgc_layer_set_profiling(dgc_layer_t* L, int32_t enable) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  if (enable && !L->ev[0]) {
    for (hipEvent_t& e : L->ev) DGC_HIP_TRY(hipEventCreate(&e));
    for (hipEvent_t& e : L->evx) DGC_HIP_TRY(hipEventCreate(&e));
    for (hipEvent_t& e : L->evd) DGC_HIP_TRY(hipEventCreate(&e));
  }
  L->profiling = enable != 0;
  L->ev_valid = L->evx_fwd = L->evx_bwd = L->evd_fwd = L->evd_bwd = false;
  return DGC_OK;
}

dgc_status_t dgc_layer_stage_times(dgc_layer_t* L, float* host_ms) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  if (!host_ms) return fail(DGC_ERR_INVALID_ARG, "NULL argument");
  for (int i = 0; i < DGC_N_STAGES; ++i) host_ms[i] = 0.f;
  if (L->desc.struct_kind == DGC_STRUCT_GAT) {
    if (!L->evd_fwd) return fail(DGC_ERR_STATE, "no profiled forward has been enqueued");
    DGC_HIP_TRY(hipEventSynchronize(L->evd[3]));
    for (int i = 0; i < 3; ++i) DGC_HIP_TRY(hipEventElapsedTime(&host_ms[7 + i], L->evd[i], L->evd[i + 1]));
    if (L->evd_bwd) {
      DGC_HIP_TRY(hipEventSynchronize(L->evd[7]));
      for (int i = 0; i < 3; ++i) DGC_HIP_TRY(hipEventElapsedTime(&host_ms[10 + i], L->evd[4 + i], L->evd[5 + i]));
    }
    return DGC_OK;
  }
  if (!L->ev_valid) return fail(DGC_ERR_STATE, "no profiled forward has been enqueued");
  DGC_HIP_TRY(hipEventSynchronize(L->ev[4]));
  for (int i = 0; i < 4; ++i) DGC_HIP_TRY(hipEventElapsedTime(&host_ms[i], L->ev[i], L->ev[i + 1]));
  if (L->evx_fwd) DGC_HIP_TRY(hipEventElapsedTime(&host_ms[4], L->evx[0], L->evx[1]));
  if (L->evx_bwd) {
    DGC_HIP_TRY(hipEventSynchronize(L->evx[5]));
    DGC_HIP_TRY(hipEventElapsedTime(&host_ms[5], L->evx[2], L->evx[3]));
    DGC_HIP_TRY(hipEventElapsedTime(&host_ms[6], L->evx[4], L->evx[5]));
  }
  return DGC_OK;
}

dgc_status_t dgc_layer_backward(dgc_layer_t* L, const void* Yv, int64_t ldy, const void* dYv, int64_t lddy,
                                const void* targetv, int64_t ldt, float* loss_out, void* dX, int64_t lddx,
                                void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  const dgc_layer_desc_t& d = L->desc;
  if (!L->forward_done) return fail(DGC_ERR_STATE, "backward before forward");
  if (d.struct_kind != DGC_STRUCT_EVOLVE_GCN_O && d.struct_kind != DGC_STRUCT_GAT)
    return fail(DGC_ERR_UNSUPPORTED, "backward is built for DGC_STRUCT_EVOLVE_GCN_O and DGC_STRUCT_GAT only");
  if ((dYv != nullptr) == (targetv != nullptr))
    return fail(DGC_ERR_INVALID_ARG, "give exactly one of dY and target");
  dgc_status_t rc;
  if (d.struct_kind == DGC_STRUCT_GAT) {
    if ((rc = check_tensor(fail, "Y", Yv, ldy, d.S, true, 8)) != DGC_OK) return rc;
    if ((rc = check_tensor(fail, "dY", dYv, lddy, d.S, false, 8)) != DGC_OK) return rc;
    if ((rc = check_tensor(fail, "target", targetv, ldt, d.S, false, 8)) != DGC_OK) return rc;
    if ((rc = check_tensor(fail, "dX", dX, lddx, d.F, false, 8)) != DGC_OK) return rc;
    if (dX && !L->dy.dzXlo) DGC_HIP_TRY(dev_alloc(L, &L->dy.dzXlo, (int64_t)L->T * L->N * d.S));
    L->evd_bwd = false;
    dysat_backward(L->dy, Yv, ldy, dYv, lddy, targetv, ldt, loss_out, dX, lddx, L->profiling ? L->evd + 4 : nullptr,
                   static_cast<hipStream_t>(stream));
    if (L->profiling) L->evd_bwd = true;
    DGC_HIP_TRY(hipGetLastError());
    L->has_grads = true;
    return DGC_OK;
  }
  const float* Y = static_cast<const float*>(Yv);
  const float* dY = static_cast<const float*>(dYv);
  const float* target = static_cast<const float*>(targetv);
  if ((rc = check_tensor(fail, "Y", Y, ldy, d.S, true)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "dY", dY, lddy, d.S, false)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "target", target, ldt, d.S, false)) != DGC_OK) return rc;
  if ((rc = check_tensor(fail, "dX", static_cast<const float*>(dX), lddx, d.F, false)) != DGC_OK) return rc;
  if (!L->m_saved) return fail(DGC_ERR_STATE, "the rows saved by forward were used up by a backward that computed dX: run forward again");
  hipStream_t st = static_cast<hipStream_t>(stream);
  EvolveBwdIn in{};
  in.chunks = L->d_chunks; in.N = L->N; in.M = L->d_M; in.ldm = L->ldm;
  in.Y = Y; in.ldy = ldy; in.dY = dY; in.lddy = lddy; in.target = target; in.ldt = ldt;
  in.count = L->total_rows * d.S;
  in.loss_out = loss_out;
  std::string why;
  const bool prof = L->profiling;
  L->evx_bwd = false;
  if (prof) DGC_HIP_TRY(hipEventRecord(L->evx[2], st));
  if (!evolve_backward_dw(L->evo, in, st, &why)) return fail(DGC_ERR_UNSUPPORTED, why);
  if (prof) { DGC_HIP_TRY(hipEventRecord(L->evx[3], st)); DGC_HIP_TRY(hipEventRecord(L->evx[4], st)); }
  evolve_backward_bptt(L->evo, st);
  if (prof) { DGC_HIP_TRY(hipEventRecord(L->evx[5], st)); L->evx_bwd = true; }
  if (dX) {
    // dX[t, j] = sum over the rows i of j's chunk that store j of (d_i d_j)^-1/2 dM[t, i],  dM = dP W_t^T:
    // dP into the buffer of the aggregated rows (the weight gradient above was their last reader), the
    // dense kernel with W_t as an (out = F, in = S) weight, then the aggregation kernels on dM with
    // the neighbours outside the chunk range left out (the cache is a constant) and the adjacency's symmetry.
    int64_t max_nv = 1;
    int32_t max_w = 1;
    for (const ChunkInfo& c : L->cinfo_host) { max_nv = std::max(max_nv, c.nv); max_w = std::max(max_w, c.w); }
    if (L->n_chunks > kMaxGridYZ || max_w > kMaxGridYZ)   // its kernels take one grid plane per chunk, one row per snapshot
      return fail(DGC_ERR_UNSUPPORTED, "input gradient: more than 65535 chunks or snapshots per window");
    if (!L->d_dM) {
      DGC_HIP_TRY(dev_alloc(L, &L->d_dM, (int64_t)L->T * L->N * d.F));
      DGC_HIP_TRY(dev_alloc(L, &L->d_rowidx, L->total_rows));
      DGC_HIP_TRY(dev_alloc(L, &L->d_Wt_plain, (int64_t)L->T * packed_weight_elems(d.F, d.S) / 4));
      evolve_row_index(L->d_chunks, L->n_chunks, max_nv, max_w, L->N, L->d_rowidx, st);
    }
    L->m_saved = false;
    evolve_backward_dp(in, L->n_chunks, max_nv, max_w, d.S, L->d_M, L->ldm, st);
    evolve_pack_weights_plain(L->evo, L->d_Wt_plain, st);
    DenseArgs da{};
    da.tiles = L->d_tiles; da.n_tiles = L->n_tiles; da.chunks = L->d_chunks;
    da.tiles32 = L->d_tiles32; da.n_tiles32 = L->n_tiles32; da.variant = d.dense_kernel;
    da.N = L->N; da.total_state_rows = L->total_state_rows;
    da.M = L->d_M; da.ldm = L->ldm;
    da.K0 = d.S; da.S = d.F; da.H = 0; da.act = DGC_ACT_NONE; da.time_kind = DGC_TIME_NONE;
    da.Wg = L->d_Wt_plain; da.bg = L->d_zero_bias;
    da.wg_step_bytes = (int32_t)(sizeof(float) * packed_weight_elems(d.F, d.S));
    da.wg_bytes = (int64_t)L->T * da.wg_step_bytes;
    da.Y = L->d_dM; da.ldy = d.F;
    if (!launch_dense(da, st, &why)) return fail(DGC_ERR_UNSUPPORTED, why);
    SpmmArgs sa = spmm_args(L, L->d_dM, d.F, L->d_dM, d.F, d.F, static_cast<float*>(dX), d.F);
    sa.ld_out = lddx;
    sa.row_map = L->d_rowidx;
    sa.skip_stale = true;
    launch_spmm(sa, st);
  }
  DGC_HIP_TRY(hipGetLastError());
  L->has_grads = true;
  return DGC_OK;
}

dgc_status_t dgc_layer_shared_rows(dgc_layer_t* L, int64_t* host_out, void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  if (!host_out) return fail(DGC_ERR_INVALID_ARG, "host_out is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int32_t n = L->n_chunks;
  if (L->nseg > kMaxGridYZ)      // the marking kernel takes one grid row per (chunk, snapshot) segment
    return fail(DGC_ERR_UNSUPPORTED, "shared rows: more than 65535 (chunk, snapshot) segments");
  if (!L->fs_mask) {
    if (dev_alloc(L, &L->fs_mask, shared_rows_mask_words(L->T, L->N, n)) != hipSuccess) {
      L->fs_mask = nullptr;
      return fail(DGC_ERR_OOM, "shared rows: the loader bitmap does not fit the device");
    }
    if (dev_alloc(L, &L->fs_out, (int64_t)n * n) != hipSuccess) {
      L->fs_mask = nullptr;    // the bitmap stays in the layer's allocation list and is freed with it
      return fail(DGC_ERR_OOM, "shared rows: out of device memory");
    }
  }
  launch_shared_rows(L->d_segs, L->nseg, L->d_halo_ptr, L->d_halo_idx, L->T, L->N, n, L->fs_mask, L->fs_out, st);
  hipError_t e = hipGetLastError();      // a rejected launch would leave the counters at zero
  if (e != hipSuccess) return fail(DGC_ERR_DEVICE, std::string("shared rows: ") + hipGetErrorString(e));
  e = hipMemcpyAsync(host_out, L->fs_out, sizeof(int64_t) * (size_t)n * n, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail(DGC_ERR_DEVICE, std::string("shared rows: ") + hipGetErrorString(e));
  for (int32_t a = 0; a < n; ++a) {      // the kernel fills the upper triangle
    host_out[(int64_t)a * n + a] = 0;
    for (int32_t b = a + 1; b < n; ++b) host_out[(int64_t)b * n + a] = host_out[(int64_t)a * n + b];
  }
  return DGC_OK;
}

dgc_status_t dgc_layer_set_presence(dgc_layer_t* L, const uint8_t* present, void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  const dgc_layer_desc_t& d = L->desc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!present) return fail(DGC_ERR_INVALID_ARG, "present is NULL");
  if (d.struct_kind != DGC_STRUCT_GCN || d.time_kind == DGC_TIME_NONE)
    return fail(DGC_ERR_UNSUPPORTED, "temporal fusion needs a GCN layer with a recurrent time encoder");
  if (L->tf.built) return fail(DGC_ERR_STATE, "the presence mask of a layer can be set once");
  if ((int64_t)L->T * L->N >= INT32_MAX) return fail(DGC_ERR_UNSUPPORTED, "temporal fusion needs T*N < 2^31");
  if (L->lab.built) return set_presence_labelled(L, present, st);
  if (L->n_chunks > kMaxGridYZ)  // its kernels take one grid row per chunk
    return fail(DGC_ERR_UNSUPPORTED, "temporal fusion: more than 65535 chunks");
  TFusion& tf = L->tf;
  const int32_t nc = L->n_chunks;
  const std::vector<ChunkInfo>& ci = L->cinfo_host;
  int64_t max_nv = 1;
  for (const ChunkInfo& c : ci) { max_nv = std::max(max_nv, c.nv); tf.Lmax = std::max(tf.Lmax, c.w); }
  // sequence lengths (device) -> lanes by first-fit decreasing (host arithmetic on the lengths)
  int32_t* d_len = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_len, L->total_state_rows));
  tf_lengths(present, L->d_chunks, nc, max_nv, L->N, d_len, st);
  std::vector<int32_t> len(L->total_state_rows), lane_of(L->total_state_rows, -1), off_of(L->total_state_rows, 0);
  DGC_HIP_TRY(hipMemcpyAsync(len.data(), d_len, sizeof(int32_t) * len.size(), hipMemcpyDeviceToHost, st));
  DGC_HIP_TRY(hipStreamSynchronize(st));
  std::vector<int64_t> lane_ptr(nc + 1, 0);
  std::vector<ChunkInfo> cv(nc);
  int64_t rows_v = 0;
  for (int32_t k = 0; k < nc; ++k) {
    const ChunkInfo& c = ci[k];
    // order: length descending, vertex ascending; each sequence into the first lane (in order of
    // creation) with room for all of it.  by_free[f] = lanes of this chunk with f free slots.
    std::vector<int32_t> order;
    for (int64_t v = 0; v < c.nv; ++v)
      if (len[c.state_off + v] > 0) order.push_back((int32_t)v);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return len[c.state_off + a] > len[c.state_off + b]; });
    std::vector<std::set<int32_t>> by_free(c.w + 1);
    int32_t n_l = 0;
    for (int32_t v : order) {
      const int32_t n = len[c.state_off + v];
      int32_t best = -1, bf = 0;
      for (int32_t f = n; f <= c.w; ++f)
        if (!by_free[f].empty() && (best < 0 || *by_free[f].begin() < best)) { best = *by_free[f].begin(); bf = f; }
      if (best < 0) { best = n_l++; bf = c.w; } else by_free[bf].erase(by_free[bf].begin());
      lane_of[c.state_off + v] = (int32_t)(lane_ptr[k] + best);
      off_of[c.state_off + v] = c.w - bf;
      by_free[bf - n].insert(best);
    }
    lane_ptr[k + 1] = lane_ptr[k] + n_l;
    cv[k] = ChunkInfo{lane_ptr[k], n_l, rows_v, lane_ptr[k], 0, c.w};
    rows_v += (int64_t)n_l * c.w;
  }
  tf.n_lanes = lane_ptr[nc];
  tf.rows_v = rows_v;
  if (tf.n_lanes > INT32_MAX) return fail(DGC_ERR_UNSUPPORTED, "too many lanes");
  const int64_t n_slots = (int64_t)tf.Lmax * tf.n_lanes;
  int32_t *d_lane = nullptr, *d_off = nullptr;
  DGC_HIP_TRY(dev_alloc(L, &d_lane, L->total_state_rows));
  DGC_HIP_TRY(dev_alloc(L, &d_off, L->total_state_rows));
  DGC_HIP_TRY(dev_alloc(L, &tf.lane_ptr, nc + 1));
  DGC_HIP_TRY(dev_alloc(L, &tf.slot_row, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.slot_reset, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.seq_in, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.seq_out, n_slots));
  DGC_HIP_TRY(dev_alloc(L, &tf.row_map, L->total_rows));
  DGC_HIP_TRY(dev_alloc(L, &tf.chunks_v, nc));
  DGC_HIP_TRY(hipMemcpyAsync(d_lane, lane_of.data(), sizeof(int32_t) * lane_of.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(d_off, off_of.data(), sizeof(int32_t) * off_of.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(tf.lane_ptr, lane_ptr.data(), sizeof(int64_t) * (nc + 1), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(tf.chunks_v, cv.data(), sizeof(ChunkInfo) * nc, hipMemcpyHostToDevice, st));
  tf_fill(present, L->d_chunks, nc, max_nv, L->N, d_lane, d_off, tf.n_lanes, tf.Lmax, tf.chunks_v, L->total_rows,
          tf.slot_row, tf.row_map, tf.slot_reset, tf.seq_in, tf.seq_out, st);
  // tiles of the virtual chunks
  std::vector<DenseTile> t64, t32;
  for (int32_t k = 0; k < nc; ++k) {
    for (int64_t v0 = 0; v0 < cv[k].nv; v0 += kTileRows)
      t64.push_back(DenseTile{k, (int32_t)v0, (int32_t)std::min<int64_t>(kTileRows, cv[k].nv - v0), 0});
    for (int64_t v0 = 0; v0 < cv[k].nv; v0 += kWaveTileRows)
      t32.push_back(DenseTile{k, (int32_t)v0, (int32_t)std::min<int64_t>(kWaveTileRows, cv[k].nv - v0), 0});
  }
  tf.n_tiles_v = (int64_t)t64.size(); tf.n_tiles32_v = (int64_t)t32.size();
  DGC_HIP_TRY(dev_alloc(L, &tf.tiles_v, tf.n_tiles_v));
  DGC_HIP_TRY(dev_alloc(L, &tf.tiles32_v, tf.n_tiles32_v));
  DGC_HIP_TRY(hipMemcpyAsync(tf.tiles_v, t64.data(), sizeof(DenseTile) * t64.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(hipMemcpyAsync(tf.tiles32_v, t32.data(), sizeof(DenseTile) * t32.size(), hipMemcpyHostToDevice, st));
  DGC_HIP_TRY(dev_alloc(L, &tf.Mv, rows_v * L->ldm));
  DGC_HIP_TRY(hipMemsetAsync(tf.Mv, 0, sizeof(float) * (size_t)std::max<int64_t>(rows_v * L->ldm, 1), st));  // empty slots stay zero
  DGC_HIP_TRY(hipStreamSynchronize(st));
  DGC_HIP_TRY(hipGetLastError());
  tf.seq_len = d_len;
  dev_free(L, d_lane); dev_free(L, d_off);
  tf.built = true;
  return DGC_OK;
}

dgc_status_t dgc_layer_set_labels(dgc_layer_t* L, const int32_t* labels, void* stream) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  const dgc_layer_desc_t& d = L->desc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!labels) return fail(DGC_ERR_INVALID_ARG, "labels is NULL");
  if (d.struct_kind != DGC_STRUCT_GCN && d.struct_kind != DGC_STRUCT_EVOLVE_GCN_O)
    return fail(DGC_ERR_UNSUPPORTED, "generated chunks are built for GCN and EvolveGCN-O layers");
  if (d.gather_mode != DGC_GATHER_IN_PLACE)
    return fail(DGC_ERR_UNSUPPORTED, "generated chunks need gather_mode DGC_GATHER_IN_PLACE");
  if (L->tf.built) return fail(DGC_ERR_STATE, "the labels of a layer are set before its presence mask, and not again after it");
  const dgc_chunk_t& c = L->chunks[0];
  if (L->n_chunks != 1 || c.v_lo != 0 || c.v_hi != L->N || c.t_lo != 0 || c.t_hi != L->T)
    return fail(DGC_ERR_STATE, "labels need a layer created with the single chunk [0,N) x [0,T)");
  if ((int64_t)L->T * L->N >= INT32_MAX) return fail(DGC_ERR_UNSUPPORTED, "generated chunks need T*N < 2^31");
  if (L->T > kMaxGridYZ) return fail(DGC_ERR_UNSUPPORTED, "generated chunks: more than 65535 snapshots");
  Labelled& lab = L->lab;
  if (!lab.col_signed) {
    DGC_HIP_TRY(dev_alloc(L, &lab.col_signed, L->total_nnz));
    DGC_HIP_TRY(dev_alloc(L, &lab.seq_in, (int64_t)L->T * L->N));
    DGC_HIP_TRY(dev_alloc(L, &lab.seq_out, (int64_t)L->T * L->N));
    DGC_HIP_TRY(dev_alloc(L, &lab.labels, (int64_t)L->T * L->N));
  }
  DGC_HIP_TRY(hipMemcpyAsync(lab.labels, labels, sizeof(int32_t) * (size_t)L->T * L->N, hipMemcpyDeviceToDevice, st));
  labels_build(L->graph_dev(), L->d_segs, labels, lab.col_signed, lab.seq_in, lab.seq_out, st);
  if (L->d_etab)      // the aggregation's table follows the labels: marked columns instead of the range test
    launch_edge_table(L->graph_dev(), L->d_segs, L->nseg, L->total_nnz, L->d_dinv, lab.col_signed, L->d_etab, st);
  DGC_HIP_TRY(hipStreamSynchronize(st));
  DGC_HIP_TRY(hipGetLastError());
  lab.built = true;
  L->forward_done = false;
  return DGC_OK;
}

dgc_status_t dgc_layer_packing(dgc_layer_t* L, const char* what, void* host_dst, int64_t capacity_bytes,
                               int64_t* needed_bytes) {
  if (!L) return DGC_ERR_INVALID_ARG;
  Failer fail{L};
  if (!what) return fail(DGC_ERR_INVALID_ARG, "NULL argument");
  const std::string w(what);
  const void* src = nullptr;
  int64_t bytes = 0;
  std::vector<int64_t> host_i64;
  if (w == "seg_row_off" || w == "seg_nnz_off") {
    host_i64.resize(L->nseg + 1);
    for (int64_t s = 0; s < L->nseg; ++s)
      host_i64[s] = w == "seg_row_off" ? L->segs_host[s].row_off : L->segs_host[s].nnz_off;
    host_i64[L->nseg] = w == "seg_row_off" ? L->total_rows : L->total_nnz;
    bytes = sizeof(int64_t) * (L->nseg + 1);
  } else if (w == "halo_ptr") { src = L->d_halo_ptr; bytes = sizeof(int64_t) * (L->nseg + 1);
  } else if (w == "halo_idx") { src = L->d_halo_idx; bytes = sizeof(int32_t) * L->total_halo;
  } else if (w == "col_local") { src = L->d_col_local; bytes = sizeof(int32_t) * L->total_nnz;
  } else if (w == "work_short") { src = L->d_work_short; bytes = sizeof(int32_t) * 3 * L->n_short;
  } else if (w == "work_long") { src = L->d_work_long; bytes = sizeof(int32_t) * 4 * L->n_long;
  } else if (w == "deg_inv_sqrt") { src = L->d_dinv; bytes = sizeof(float) * (int64_t)L->T * L->N;
  } else if (w == "lane_ptr" || w == "slot_row" || w == "slot_reset") {
    if (!L->tf.built) return fail(DGC_ERR_STATE, "no temporal-fusion packing: call dgc_layer_set_presence first");
    const int64_t n = (int64_t)L->tf.Lmax * L->tf.n_lanes;
    if (w == "lane_ptr") { src = L->tf.lane_ptr; bytes = sizeof(int64_t) * (L->n_chunks + 1); }
    else if (w == "slot_row") { src = L->tf.slot_row; bytes = sizeof(int64_t) * n; }
    else { src = L->tf.slot_reset; bytes = n; }
  } else {
    return fail(DGC_ERR_INVALID_ARG, "unknown packing array " + w);
  }
  if (needed_bytes) *needed_bytes = bytes;
  if (!host_dst || capacity_bytes < bytes)
    return fail(DGC_ERR_INVALID_ARG, "destination too small for " + w);
  if (bytes == 0) return DGC_OK;
  if (!host_i64.empty()) {
    std::memcpy(host_dst, host_i64.data(), (size_t)bytes);
  } else {
    DGC_HIP_TRY(hipMemcpy(host_dst, src, (size_t)bytes, hipMemcpyDeviceToHost));
  }
  return DGC_OK;
}

}  // extern "C"
