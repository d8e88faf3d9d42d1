// Normalised neighbour aggregation of the GCN convolution (the structure encoder Section 6
// names) over the fused batch, and the stale-cache gather (Section 5.2).
//
//   M[row of (t,i)] = d_i^-1/2 * sum_j d_j^-1/2 * src(t,j)
//   src(t,j) = fresh[t,j] if j lies in the row's chunk vertex range, else the cache row.
// (With generated chunks the stored columns come pre-marked instead: j = fresh, ~j = cache row.)
//
// HBM/L2-bound work: one wavefront owns one work item (a group of consecutive rows, or one
// part of a split row).  The 64 lanes span the feature dimension (1, 2 or 4 floats each), so
// every neighbour row is one fully coalesced load; column indices and their degree scalings
// are fetched 64 at a time, one per lane, and handed out with v_readlane so that the row
// address is wave-uniform.  Eight neighbour rows are in flight per wave.  Rows of 65 to 128
// floats take the two-rows-per-load variant instead (each half of the wave one neighbour, 16
// bytes per lane, sixteen rows in flight).
#include "dgc_internal.h"

namespace dgc {
namespace {

constexpr int kInflight = 8;
constexpr int kInflightPair = 8;   // pairs of rows in flight in the two-rows-per-load variant (4 and 12 measured slower)

template <int VEC> struct Vec;
template <> struct Vec<1> { using T = float; };
template <> struct Vec<2> { using T = float2; };
template <> struct Vec<4> { using T = float4; };

template <int VEC>
__device__ __forceinline__ void vload(float (&v)[VEC], const float* p) {
  if constexpr (VEC == 1) { v[0] = *p; }
  if constexpr (VEC == 2) { const float2 t = *reinterpret_cast<const float2*>(p); v[0] = t.x; v[1] = t.y; }
  if constexpr (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
}

// Output rows are written once and read later by another kernel: streaming stores, so that
// they do not push the neighbour rows being re-read out of L2.
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
template <int VEC>
__device__ __forceinline__ void vstore(float* p, const float (&v)[VEC]) {
  if constexpr (VEC == 1) { __builtin_nontemporal_store(v[0], p); }
  if constexpr (VEC == 2) { floatx2 t = {v[0], v[1]}; __builtin_nontemporal_store(t, reinterpret_cast<floatx2*>(p)); }
  if constexpr (VEC == 4) {
    floatx4 t = {v[0], v[1], v[2], v[3]};
    __builtin_nontemporal_store(t, reinterpret_cast<floatx4*>(p));
  }
}

__device__ __forceinline__ int64_t readlane64(int64_t v, int lane) {
  const int lo = __builtin_amdgcn_readlane((int)(v & 0xffffffff), lane);
  const int hi = __builtin_amdgcn_readlane((int)(v >> 32), lane);
  return ((int64_t)hi << 32) | (uint32_t)lo;
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Per-work-item constants, all wave-uniform.
struct RowCtx {
  const int32_t* cj;        // colidx of the snapshot
  const int32_t* cl;        // col_local of the segment, indexed by (e - e0)   (STAGED)
  const float* dinv_t;
  const float* fresh_t; int64_t ld_fresh;
  const float* stale_t; int64_t ld_stale;   // IN_PLACE: cache snapshot; STAGED: segment's halo rows
  int64_t v_lo, v_hi, e0;
  bool skip_stale;          // neighbours outside the range contribute nothing (input-gradient pass)
};

// MODE of the neighbour lookup
constexpr int kInPlace = 0;   // by the segment's vertex range, rows read where they are
constexpr int kStaged = 1;    // local slots: fresh rows, then the segment's gathered halo rows
constexpr int kSigned = 2;    // pre-marked columns (j fresh, ~j cache), rows read where they are

// acc += sum over stored non-zeros e in [ea, eb) of dinv[col] * src row, features fi..fi+VEC-1.
template <int VEC, int MODE>
__device__ __forceinline__ void accumulate_edges(const RowCtx& c, int64_t ea, int64_t eb, int lane, int fi,
                                                 bool active, float (&acc)[VEC]) {
  for (int64_t eb0 = ea; eb0 < eb; eb0 += kWave) {
    const int m = (int)((eb - eb0) < kWave ? (eb - eb0) : kWave);
    int j = 0, loc = 0;
    float wj = 0.f;
    if (lane < m) {
      j = __builtin_nontemporal_load(c.cj + eb0 + lane);  // streamed once
      wj = c.dinv_t[(MODE == kSigned && j < 0) ? ~j : j];
      if constexpr (MODE == kStaged) loc = __builtin_nontemporal_load(c.cl + (eb0 - c.e0) + lane);
    }
    for (int k = 0; k < m; k += kInflight) {
      float v[kInflight][VEC];
      float w[kInflight];
#pragma unroll
      for (int u = 0; u < kInflight; ++u) {
        w[u] = 0.f;
#pragma unroll
        for (int q = 0; q < VEC; ++q) v[u][q] = 0.f;
        if (k + u < m) {  // wave-uniform
          const int jj = __builtin_amdgcn_readlane(j, k + u);
          w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wj), k + u));
          const float* src;
          if constexpr (MODE == kStaged) {
            const int ll = __builtin_amdgcn_readlane(loc, k + u);
            const int64_t nv = c.v_hi - c.v_lo;
            src = ll < nv ? c.fresh_t + (c.v_lo + ll) * c.ld_fresh : c.stale_t + (ll - nv) * c.ld_stale;
          } else {
            const bool in = MODE == kSigned ? jj >= 0 : (jj >= c.v_lo && jj < c.v_hi);   // wave-uniform
            const int64_t col = (MODE == kSigned && !in) ? ~jj : jj;
            src = in ? c.fresh_t + col * c.ld_fresh : c.stale_t + col * c.ld_stale;
            if (!in && c.skip_stale) { w[u] = 0.f; continue; }
          }
          if (active) vload<VEC>(v[u], src + fi);
        }
      }
#pragma unroll
      for (int u = 0; u < kInflight; ++u)
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = fmaf(w[u], v[u][q], acc[q]);
    }
  }
}

template <int VEC>
__device__ __forceinline__ void store_row(float* out, int fi, int F, int64_t ldm, const float (&acc)[VEC], float scale);

// The same sum for rows of at most 128 floats, two neighbours per load instruction: lanes 0-31 take
// the even non-zeros of the batch and lanes 32-63 the odd ones, four floats per lane, so that one
// 16-byte load per lane fetches two whole rows (twice the bytes per instruction of a 64-lane
// 8-byte load; the aggregation is bound by the rate of load instructions, not by bytes).  Each
// half ends with the sum over its own neighbours; the caller adds the two halves.
template <int MODE>
__device__ __forceinline__ void accumulate_edges_pair(const RowCtx& c, int64_t ea, int64_t eb, int lane, int fi,
                                                      bool active, float (&acc)[4]) {
  const bool odd = lane >= 32;
  for (int64_t eb0 = ea; eb0 < eb; eb0 += kWave) {
    const int m = (int)((eb - eb0) < kWave ? (eb - eb0) : kWave);
    int j = 0, loc = 0;
    float wj = 0.f;
    if (lane < m) {
      j = __builtin_nontemporal_load(c.cj + eb0 + lane);  // streamed once
      wj = c.dinv_t[(MODE == kSigned && j < 0) ? ~j : j];
      if constexpr (MODE == kStaged) loc = __builtin_nontemporal_load(c.cl + (eb0 - c.e0) + lane);
    }
    for (int k = 0; k < m; k += 2 * kInflightPair) {
      float v[kInflightPair][4];
      float w[kInflightPair];
#pragma unroll
      for (int u = 0; u < kInflightPair; ++u) {
        w[u] = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[u][q] = 0.f;
        const int e = k + 2 * u;                      // e + 1 <= 63
        if (e < m) {                                  // wave-uniform
          const int j0 = __builtin_amdgcn_readlane(j, e), j1 = __builtin_amdgcn_readlane(j, e + 1);
          const int w0 = __builtin_amdgcn_readlane(__float_as_int(wj), e);
          const int w1 = __builtin_amdgcn_readlane(__float_as_int(wj), e + 1);
          const int jj = odd ? j1 : j0;
          bool take = !odd || e + 1 < m;              // the last non-zero of an odd batch has no partner
          w[u] = take ? __int_as_float(odd ? w1 : w0) : 0.f;
          const float* src;
          if constexpr (MODE == kStaged) {
            const int l0 = __builtin_amdgcn_readlane(loc, e), l1 = __builtin_amdgcn_readlane(loc, e + 1);
            const int ll = odd ? l1 : l0;
            const int64_t nv = c.v_hi - c.v_lo;
            src = ll < nv ? c.fresh_t + (c.v_lo + ll) * c.ld_fresh : c.stale_t + (ll - nv) * c.ld_stale;
          } else {
            const bool in = MODE == kSigned ? jj >= 0 : (jj >= c.v_lo && jj < c.v_hi);
            const int64_t col = (MODE == kSigned && !in) ? ~jj : jj;
            src = in ? c.fresh_t + col * c.ld_fresh : c.stale_t + col * c.ld_stale;
            if (!in && c.skip_stale) { w[u] = 0.f; take = false; }
          }
          if (active && take) vload<4>(v[u], src + fi);
        }
      }
#pragma unroll
      for (int u = 0; u < kInflightPair; ++u)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = fmaf(w[u], v[u][q], acc[q]);
    }
  }
}

// One output row from the paired sum: halves added, lanes 0-31 store columns 0-127, lanes 32-63
// zero-fill the pad columns from 128 to the pitch.
template <int MODE>
__device__ __forceinline__ void pair_row(const RowCtx& c, int64_t ea, int64_t eb, int lane, int F, int64_t ldm,
                                         float* out, float scale) {
  const int fi = (lane & 31) * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  accumulate_edges_pair<MODE>(c, ea, eb, lane, fi, fi < F, acc);
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] += __shfl_xor(acc[q], 32);
  if (lane < 32) {
    store_row<4>(out, fi, F, ldm, acc, scale);
  } else if (128 + fi < ldm) {
    const float z[4] = {0.f, 0.f, 0.f, 0.f};
    vstore<4>(out + 128 + fi, z);
  }
}

template <int MODE>
__device__ __forceinline__ RowCtx make_ctx(const SpmmArgs& a, const Segment& sg) {
  constexpr bool STAGED = MODE == kStaged;
  RowCtx c;
  // (the marked columns are stored segment after segment; e counts from the snapshot's start)
  c.cj = MODE == kSigned ? a.col_signed + (sg.nnz_off - sg.e0) : a.g.colidx[sg.t];
  c.cl = STAGED ? a.col_local + sg.nnz_off : nullptr;
  c.dinv_t = a.dinv + (int64_t)sg.t * a.g.N;
  c.fresh_t = a.fresh + (int64_t)sg.t * a.g.N * a.ld_fresh;
  c.ld_fresh = a.ld_fresh;
  if (STAGED) {
    c.stale_t = a.halo + sg.halo_off * a.ld_halo;
    c.ld_stale = a.ld_halo;
  } else {
    c.stale_t = a.stale + (int64_t)sg.t * a.g.N * a.ld_stale;
    c.ld_stale = a.ld_stale;
  }
  c.v_lo = sg.v_lo; c.v_hi = sg.v_hi; c.e0 = sg.e0;
  c.skip_stale = a.skip_stale;
  return c;
}

template <int VEC>
__device__ __forceinline__ void store_row(float* out, int fi, int F, int64_t ldm, const float (&acc)[VEC], float scale) {
  if (fi >= ldm) return;
  float o[VEC];
#pragma unroll
  for (int q = 0; q < VEC; ++q) o[q] = (fi + q < F) ? acc[q] * scale : 0.f;
  vstore<VEC>(out + fi, o);
}

// One wave per group of consecutive rows of a segment.  Rows longer than long_nnz are left to
// the split-row kernels.
template <int VEC, int MODE, bool PAIR>
__global__ __launch_bounds__(256) void k_spmm_short(SpmmArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t item = (int64_t)blockIdx.x * (256 / kWave) + (threadIdx.x / kWave);
  if (item >= a.n_short) return;
  const int seg = uniform(a.work_short[3 * item + 0]);
  const int r0 = uniform(a.work_short[3 * item + 1]);
  const int n = uniform(a.work_short[3 * item + 2]);
  const Segment sg = a.segs[seg];
  const RowCtx c = make_ctx<MODE>(a, sg);
  const int64_t* rp = a.g.rowptr[sg.t] + sg.v_lo + r0;
  const int64_t my_rp = lane <= n ? rp[lane] : 0;
  // optional output permutation: row_map[packed row] = row of M to write, < 0 = row not wanted
  const int64_t my_map = a.row_map ? (lane < n ? a.row_map[sg.row_off + r0 + lane] : -1) : sg.row_off + r0 + lane;
  for (int r = 0; r < n; ++r) {
    const int64_t ea = readlane64(my_rp, r), eb = readlane64(my_rp, r + 1);
    if (eb - ea > a.long_nnz) continue;
    const int64_t orow = readlane64(my_map, r);
    if (orow < 0) continue;
    const float di = c.dinv_t[sg.v_lo + r0 + r];
    float* out = a.M + orow * (a.ld_out ? a.ld_out : a.ldm);
    if constexpr (PAIR) {
      pair_row<MODE>(c, ea, eb, lane, a.F, a.ldm, out, di);
    } else {
      for (int f0 = 0; f0 < a.ldm; f0 += kWave * VEC) {
        const int fi = f0 + lane * VEC;
        float acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = 0.f;
        accumulate_edges<VEC, MODE>(c, ea, eb, lane, fi, fi < a.F, acc);
        store_row<VEC>(out, fi, a.F, a.ldm, acc, di);
      }
    }
  }
}

// One wave per part of a split row: unscaled partial sums.
template <int VEC, int MODE, bool PAIR>
__global__ __launch_bounds__(256) void k_spmm_long(SpmmArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t item = (int64_t)blockIdx.x * (256 / kWave) + (threadIdx.x / kWave);
  if (item >= a.n_long) return;
  const int seg = uniform(a.work_long[4 * item + 0]);
  const int row = uniform(a.work_long[4 * item + 1]);
  const int part = uniform(a.work_long[4 * item + 2]);
  const Segment sg = a.segs[seg];
  const RowCtx c = make_ctx<MODE>(a, sg);
  const int64_t* rp = a.g.rowptr[sg.t] + sg.v_lo + row;
  const int64_t ra = rp[0], rb = rp[1];
  const int64_t ea = ra + (int64_t)part * a.part_nnz;
  const int64_t eb = (ea + a.part_nnz < rb) ? ea + a.part_nnz : rb;
  float* out = a.partial + item * a.ldm;
  if constexpr (PAIR) {
    pair_row<MODE>(c, ea, eb, lane, a.F, a.ldm, out, 1.0f);
  } else {
    for (int f0 = 0; f0 < a.ldm; f0 += kWave * VEC) {
      const int fi = f0 + lane * VEC;
      float acc[VEC];
#pragma unroll
      for (int q = 0; q < VEC; ++q) acc[q] = 0.f;
      accumulate_edges<VEC, MODE>(c, ea, eb, lane, fi, fi < a.F, acc);
      store_row<VEC>(out, fi, a.F, a.ldm, acc, 1.0f);
    }
  }
}

// Sum the parts of each split row in part order (fixed order: results are reproducible), in
// double: a hub row's sum runs over tens of thousands of terms, and the merge of its parts is the
// one place where a wider accumulator costs nothing (a few thousand rows per launch).
template <int VEC>
__global__ __launch_bounds__(256) void k_spmm_long_reduce(SpmmArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t item = (int64_t)blockIdx.x * (256 / kWave) + (threadIdx.x / kWave);
  if (item >= a.n_long) return;
  if (uniform(a.work_long[4 * item + 2]) != 0) return;
  const int seg = uniform(a.work_long[4 * item + 0]);
  const int row = uniform(a.work_long[4 * item + 1]);
  const int parts = uniform(a.work_long[4 * item + 3]);
  const Segment sg = a.segs[seg];
  const float di = a.dinv[(int64_t)sg.t * a.g.N + sg.v_lo + row];
  const int64_t orow = a.row_map ? a.row_map[sg.row_off + row] : sg.row_off + row;
  if (orow < 0) return;
  float* out = a.M + orow * (a.ld_out ? a.ld_out : a.ldm);
  for (int f0 = 0; f0 < a.ldm; f0 += kWave * VEC) {
    const int fi = f0 + lane * VEC;
    if (fi >= a.ldm) continue;
    double sum[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) sum[q] = 0.0;
    for (int p = 0; p < parts; ++p) {
      float v[VEC];
      vload<VEC>(v, a.partial + (item + p) * a.ldm + fi);
#pragma unroll
      for (int q = 0; q < VEC; ++q) sum[q] += (double)v[q];
    }
    float acc[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) acc[q] = (float)(sum[q] * (double)di);
    store_row<VEC>(out, fi, a.F, a.ldm, acc, 1.0f);
  }
}


// ---------------------------------------------------------------------------------------------
// Second generation of the aggregation kernels (IN_PLACE and generated chunks, equal pitches of the
// fresh and the cache tensor, rows of at most 256 floats).  The first generation above spends some
// thirty vector instructions per gathered row on broadcasting column ids, range tests and 64-bit
// address arithmetic, and is bound by instruction issue, not by memory.  Here the per-non-zero
// work is prepared once, at packing time, in an edge table (SpmmArgs::etab): a lane reads the
// marked column and the neighbour's scaling with one 8-byte load at a constant offset from a
// running pointer, forms the row address with one 64-bit multiply-add, and no value has to be
// made wave-uniform.  LPR lanes (16, 32 or 64, four floats each) cover a row, so a wave's load
// instruction fetches G = 64 / LPR neighbour rows, U = 8 such loads in flight per lane group.
//   One long row:   the G groups split its non-zeros (batches of U * G), partial sums added across
//                   the groups at the end of the row.
//   Short rows:     group g takes row r + g of its own (no cross-group sum, no idle half).
// Slots past the end of a row (and, in the input-gradient pass, neighbours outside the chunk range)
// load the row's own vertex instead, with weight zero: its stored self-loop makes that a row the
// sum reads anyway, so nothing the sum does not depend on can leak a NaN into it.  The table has
// kEtabPad spare entries so that whole batches can always be read.
constexpr int kU = 8;            // table entries (neighbour rows) in flight per lane group
constexpr int kSmallRow = 16;    // rows up to this many non-zeros share a wave with their neighbours
static_assert(kEtabPad >= 4 * kU && kSmallRow <= 2 * kU, "batches of the last rows must stay inside the table's spare entries");

template <int UU, bool TAIL, bool SKIP>
__device__ __forceinline__ void agg_batch(const int2* p, int n_valid, int self_j, const char* fresh_l, const char* stale_l,
                                          uint32_t ld_bytes, float (&acc)[4]) {
  typedef int intx2 __attribute__((ext_vector_type(2)));
  intx2 ent[UU];       // streamed once
#pragma unroll
  for (int u = 0; u < UU; ++u) ent[u] = __builtin_nontemporal_load(reinterpret_cast<const intx2*>(p) + u);
  float4 v[UU];
  float w[UU];
#pragma unroll
  for (int u = 0; u < UU; ++u) {
    const bool ok = (!TAIL || u < n_valid) && (!SKIP || ent[u].x >= 0);
    const int c = ok ? ent[u].x : self_j;
    const bool in = c >= 0;
    const uint32_t j = (uint32_t)(in ? c : ~c);
    const char* base = in ? fresh_l : stale_l;
    v[u] = *reinterpret_cast<const float4*>(base + (uint64_t)j * ld_bytes);
    w[u] = ok ? __int_as_float(ent[u].y) : 0.f;
  }
#pragma unroll
  for (int u = 0; u < UU; ++u) {
    acc[0] = fmaf(w[u], v[u].x, acc[0]);
    acc[1] = fmaf(w[u], v[u].y, acc[1]);
    acc[2] = fmaf(w[u], v[u].z, acc[2]);
    acc[3] = fmaf(w[u], v[u].w, acc[3]);
  }
}

// Sum over the table entries [pos, end) of this lane's group, `stride` entries from batch to batch.
template <int LPR, bool SKIP>
__device__ __forceinline__ void agg_range(const int2* tab, int pos, int end, int stride, int self_j, const char* fresh_l,
                                          const char* stale_l, uint32_t ld_bytes, float (&acc)[4]) {
  constexpr int G = 64 / LPR;
  for (;;) {
    const int rem = end - pos;                       // uniform within a lane group
    int rem_max = __builtin_amdgcn_readlane(rem, 0);
#pragma unroll
    for (int g = 1; g < G; ++g) {
      const int r = __builtin_amdgcn_readlane(rem, g * LPR);
      rem_max = r > rem_max ? r : rem_max;
    }
    if (rem_max <= 0) break;
    int rem_min = __builtin_amdgcn_readlane(rem, 0);
#pragma unroll
    for (int g = 1; g < G; ++g) {
      const int r = __builtin_amdgcn_readlane(rem, g * LPR);
      rem_min = r < rem_min ? r : rem_min;
    }
    const int2* p = tab + pos;
    if (rem_min >= kU) agg_batch<kU, false, SKIP>(p, kU, self_j, fresh_l, stale_l, ld_bytes, acc);
    else if (rem_max > 4) agg_batch<8, true, SKIP>(p, rem, self_j, fresh_l, stale_l, ld_bytes, acc);
    else if (rem_max > 2) agg_batch<4, true, SKIP>(p, rem, self_j, fresh_l, stale_l, ld_bytes, acc);
    else if (rem_max > 1) agg_batch<2, true, SKIP>(p, rem, self_j, fresh_l, stale_l, ld_bytes, acc);
    else agg_batch<1, true, SKIP>(p, rem, self_j, fresh_l, stale_l, ld_bytes, acc);
    pos += stride;
  }
}

// Write one output row: columns < F scaled, columns F .. ldm-1 zero.  Lane l of the writing group
// owns columns 4l .. 4l+3 and, if the pitch is wider than the group, the same columns of every
// further stretch of 4 * LPR.
template <int LPR>
__device__ __forceinline__ void agg_store(float* out, int l, int F, int64_t ldm, const float (&acc)[4], float scale) {
  const int fi = 4 * l;
  if (fi < ldm) {
    float o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = (fi + q < F) ? acc[q] * scale : 0.f;
    vstore<4>(out + fi, o);
  }
  const float z[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c = fi + 4 * LPR; c < ldm; c += 4 * LPR) vstore<4>(out + c, z);
}

template <int LPR>
__device__ __forceinline__ void agg_reduce_groups(float (&acc)[4]) {
  constexpr int G = 64 / LPR;
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] += __shfl_xor(acc[q], m);
  (void)G;
}

struct AggCtx {
  const int2* tab;       // table entry of the work item's first non-zero
  const char* fresh_l;   // snapshot's fresh rows + this lane's column offset
  const char* stale_l;
  uint32_t ld_bytes;
};

template <int LPR>
__device__ __forceinline__ AggCtx agg_ctx(const SpmmArgs& a, const Segment& sg, int64_t first_e, int l) {
  AggCtx c;
  c.tab = a.etab + sg.nnz_off + (first_e - sg.e0);
  const int fi = (4 * l < a.F) ? 4 * l : 0;     // lanes past the row's end re-read its first columns (never stored)
  const int64_t snap = (int64_t)sg.t * a.g.N * a.ld_fresh;
  c.fresh_l = reinterpret_cast<const char*>(a.fresh + snap + fi);
  c.stale_l = reinterpret_cast<const char*>(a.stale + snap + fi);
  c.ld_bytes = (uint32_t)(a.ld_fresh * sizeof(float));
  return c;
}

template <int LPR, bool SKIP>
__global__ __launch_bounds__(256) void k_agg_short(SpmmArgs a) {
  constexpr int G = 64 / LPR;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (256 / kWave) + (threadIdx.x / kWave);
  const int64_t item = wave;
  if (item >= a.n_short) return;
  const int seg = uniform(a.work_short[3 * item + 0]);
  const int r0 = uniform(a.work_short[3 * item + 1]);
  const int n = uniform(a.work_short[3 * item + 2]);
  const Segment sg = a.segs[seg];
  const int g = lane / LPR, l = lane % LPR;
  const int64_t* rp = a.g.rowptr[sg.t] + sg.v_lo + r0;
  const int64_t rp0 = rp[0];
  const int my_rel = lane <= n ? (int)(rp[lane] - rp0) : 0;     // lanes 0..n: row offsets relative to the group's start
  const AggCtx c = agg_ctx<LPR>(a, sg, rp0, l);
  const float* dinv_rows = a.dinv + (int64_t)sg.t * a.g.N + sg.v_lo + r0;
  const int64_t prow0 = sg.row_off + r0;
  const int64_t ldo = a.ld_out ? a.ld_out : a.ldm;
  // rows whose output nobody wants (row_map < 0: absent under temporal fusion) are not computed
  uint64_t todo = __ballot(lane < n && (!a.row_map || a.row_map[prow0 + lane] >= 0));
  while (todo) {
    const int r = __builtin_ctzll(todo);
    const int e_r = __builtin_amdgcn_readlane(my_rel, r), e_r1 = __builtin_amdgcn_readlane(my_rel, r + 1);
    const int nnz_r = e_r1 - e_r;
    if (nnz_r > a.long_nnz) { todo &= todo - 1; continue; }
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (G == 1 || nnz_r > kSmallRow) {
      // one row for the whole wave
      agg_range<LPR, SKIP>(c.tab, e_r + g * kU, e_r1, kU * G, (int)(sg.v_lo + r0 + r), c.fresh_l, c.stale_l, c.ld_bytes, acc);
      agg_reduce_groups<LPR>(acc);
      const int64_t orow = a.row_map ? a.row_map[prow0 + r] : prow0 + r;
      if (g == 0) agg_store<LPR>(a.M + orow * ldo, l, a.F, a.ldm, acc, dinv_rows[r]);
      todo &= todo - 1;
    } else {
      // up to G of the next wanted small rows, one per lane group
      int take = 0, mine = r;
      uint64_t m = todo;
      while (take < G && m) {
        const int r2 = __builtin_ctzll(m);
        const int nn = __builtin_amdgcn_readlane(my_rel, r2 + 1) - __builtin_amdgcn_readlane(my_rel, r2);
        if (nn > kSmallRow) break;
        if (g == take) mine = r2;
        ++take;
        m &= m - 1;
      }
      todo = m;
      const int b = __shfl(my_rel, mine), e = __shfl(my_rel, mine + 1);
      agg_range<LPR, SKIP>(c.tab, b, g < take ? e : b, kU, (int)(sg.v_lo + r0 + mine), c.fresh_l, c.stale_l, c.ld_bytes, acc);
      const int64_t orow = a.row_map ? a.row_map[prow0 + mine] : prow0 + mine;
      if (g < take) agg_store<LPR>(a.M + orow * ldo, l, a.F, a.ldm, acc, dinv_rows[mine]);
    }
  }
}

// One wave per part of a split row: unscaled partial sums.
template <int LPR, bool SKIP>
__global__ __launch_bounds__(256) void k_agg_long(SpmmArgs a) {
  constexpr int G = 64 / LPR;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (256 / kWave) + (threadIdx.x / kWave);
  const int64_t item = wave;
  if (item >= a.n_long) return;
  const int seg = uniform(a.work_long[4 * item + 0]);
  const int row = uniform(a.work_long[4 * item + 1]);
  const int part = uniform(a.work_long[4 * item + 2]);
  const Segment sg = a.segs[seg];
  const int g = lane / LPR, l = lane % LPR;
  if (a.row_map && a.row_map[sg.row_off + row] < 0) return;     // nobody wants this row (the merge skips it too)
  const int64_t* rp = a.g.rowptr[sg.t] + sg.v_lo + row;
  const int64_t ra = rp[0], rb = rp[1];
  const int64_t ea = ra + (int64_t)part * a.part_nnz;
  const int len = (int)((ea + a.part_nnz < rb ? ea + a.part_nnz : rb) - ea);
  const AggCtx c = agg_ctx<LPR>(a, sg, ea, l);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  agg_range<LPR, SKIP>(c.tab, g * kU, len, kU * G, (int)(sg.v_lo + row), c.fresh_l, c.stale_l, c.ld_bytes, acc);
  agg_reduce_groups<LPR>(acc);
  if (g == 0) agg_store<LPR>(a.partial + item * a.ldm, l, a.F, a.ldm, acc, 1.0f);
}

template <int LPR>
void launch_agg(const SpmmArgs& a, hipStream_t st) {
  const unsigned gs = (unsigned)((a.n_short + 3) / 4), gl = (unsigned)((a.n_long + 3) / 4);
  if (gs) {
    if (a.skip_stale) hipLaunchKernelGGL((k_agg_short<LPR, true>), gs, 256, 0, st, a);
    else hipLaunchKernelGGL((k_agg_short<LPR, false>), gs, 256, 0, st, a);
  }
  if (gl) {
    if (a.skip_stale) hipLaunchKernelGGL((k_agg_long<LPR, true>), gl, 256, 0, st, a);
    else hipLaunchKernelGGL((k_agg_long<LPR, false>), gl, 256, 0, st, a);
    if (a.ldm <= 64) hipLaunchKernelGGL((k_spmm_long_reduce<1>), gl, 256, 0, st, a);
    else if (a.ldm <= 128) hipLaunchKernelGGL((k_spmm_long_reduce<2>), gl, 256, 0, st, a);
    else hipLaunchKernelGGL((k_spmm_long_reduce<4>), gl, 256, 0, st, a);
  }
}

// etab[p] = (marked column, scaling of the neighbour) for packed non-zero p
__global__ __launch_bounds__(256) void k_edge_table(GraphDev g, const Segment* segs, int64_t nseg, int64_t total_nnz,
                                                    const float* dinv, const int32_t* col_signed, int2* etab) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= total_nnz + kEtabPad) return;
  if (p >= total_nnz) { etab[p] = make_int2(0, 0); return; }
  int64_t lo = 0, hi = nseg - 1;     // the segment of p: largest s with nnz_off[s] <= p
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) >> 1;
    if (segs[mid].nnz_off <= p) lo = mid; else hi = mid - 1;
  }
  const Segment sg = segs[lo];
  const int32_t j = g.colidx[sg.t][sg.e0 + (p - sg.nnz_off)];
  const int32_t marked = col_signed ? col_signed[p] : ((j >= sg.v_lo && j < sg.v_hi) ? j : ~j);
  const bool valid = j >= 0 && j < g.N;
  const float w = valid ? dinv[(int64_t)sg.t * g.N + j] : 0.f;
  etab[p] = make_int2(valid ? marked : 0, __float_as_int(w));
}

template <int VEC, bool PAIR = false>
void launch_spmm_v(const SpmmArgs& a, hipStream_t st) {
  constexpr int RV = PAIR ? 2 : VEC;   // the merge of split rows walks the pitch 64 x RV floats at a time
  const int mode = a.halo != nullptr ? kStaged : a.col_signed != nullptr ? kSigned : kInPlace;
  const unsigned gs = (unsigned)((a.n_short + 3) / 4), gl = (unsigned)((a.n_long + 3) / 4);
  if (gs) {
    if (mode == kStaged) hipLaunchKernelGGL((k_spmm_short<VEC, kStaged, PAIR>), gs, 256, 0, st, a);
    else if (mode == kSigned) hipLaunchKernelGGL((k_spmm_short<VEC, kSigned, PAIR>), gs, 256, 0, st, a);
    else hipLaunchKernelGGL((k_spmm_short<VEC, kInPlace, PAIR>), gs, 256, 0, st, a);
  }
  if (gl) {
    if (mode == kStaged) hipLaunchKernelGGL((k_spmm_long<VEC, kStaged, PAIR>), gl, 256, 0, st, a);
    else if (mode == kSigned) hipLaunchKernelGGL((k_spmm_long<VEC, kSigned, PAIR>), gl, 256, 0, st, a);
    else hipLaunchKernelGGL((k_spmm_long<VEC, kInPlace, PAIR>), gl, 256, 0, st, a);
    hipLaunchKernelGGL((k_spmm_long_reduce<RV>), gl, 256, 0, st, a);
  }
}

// halo[p] = C[t(p), halo_idx[p], :] for every packed halo slot p.  One thread per float4.
__global__ __launch_bounds__(256) void k_gather(const Segment* segs, int64_t nseg, const int32_t* halo_idx,
                                                const int64_t* halo_ptr, int64_t total_halo, int64_t N,
                                                const float* C, int64_t ldc, int32_t f4, float* halo,
                                                int64_t ldh) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t p = idx / f4;
  if (p >= total_halo) return;
  const int c = (int)(idx - p * f4);
  int64_t lo = 0, hi = nseg - 1;  // largest s with halo_ptr[s] <= p
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) >> 1;
    if (halo_ptr[mid] <= p) lo = mid; else hi = mid - 1;
  }
  const int64_t t = segs[lo].t;
  const float4 v = *reinterpret_cast<const float4*>(C + (t * N + halo_idx[p]) * ldc + 4 * c);
  *reinterpret_cast<float4*>(halo + p * ldh + 4 * c) = v;
}

}  // namespace

void launch_edge_table(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_nnz, const float* dinv,
                       const int32_t* col_signed, int2* etab, hipStream_t st) {
  const int64_t n = total_nnz + kEtabPad;
  hipLaunchKernelGGL(k_edge_table, (unsigned)((n + 255) / 256), 256, 0, st, g, segs, nseg, total_nnz, dinv, col_signed, etab);
}


void launch_spmm(const SpmmArgs& a, hipStream_t st) {
  // the edge-table kernels: rows read in place, one pitch for both sources, at most 256 columns
  if (a.etab && !a.halo && a.ld_fresh == a.ld_stale && a.F <= 256 && a.ld_fresh * 4 < (int64_t(1) << 31)) {
    if (a.F <= 64) launch_agg<16>(a, st);
    else if (a.F <= 128) launch_agg<32>(a, st);
    else launch_agg<64>(a, st);
    return;
  }
  if (a.F <= 64) launch_spmm_v<1>(a, st);
  else if (a.F <= 128) launch_spmm_v<4, true>(a, st);
  else launch_spmm_v<4>(a, st);
}

void launch_gather(const Segment* segs, int64_t nseg, const int32_t* halo_idx, const int64_t* halo_ptr,
                   int64_t total_halo, int64_t N, const float* C, int64_t ldc, int32_t F, float* halo,
                   int64_t ldh, hipStream_t st) {
  const int32_t f4 = (F + 3) / 4;
  const int64_t n = total_halo * f4;
  if (n > 0)
    hipLaunchKernelGGL(k_gather, (unsigned)((n + 255) / 256), 256, 0, st, segs, nseg, halo_idx, halo_ptr,
                       total_halo, N, C, ldc, f4, halo, ldh);
}

}  // namespace dgc
