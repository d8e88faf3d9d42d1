// Internal declarations shared by the HIP translation units of libdgc.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "dgc.h"

namespace dgc {

constexpr int kWave = 64;
constexpr int kTileRows = 64;      // rows of one tile of the workgroup-tile dense kernel
constexpr int kWaveTileRows = 32;  // rows of one tile of the wave-private dense kernel

// One (chunk, snapshot) pair of the fused batch.
struct Segment {
  int64_t row_off;   // first packed row
  int64_t nnz_off;   // first packed non-zero
  int64_t e0;        // rowptr[t][v_lo]: first stored non-zero of the segment in snapshot t
  int64_t halo_off;  // first packed halo slot
  int64_t v_lo, v_hi;
  int32_t t;
  int32_t chunk;
};

// Per-chunk data used by the dense kernels.
struct ChunkInfo {
  int64_t v_lo;
  int64_t nv;
  int64_t row_off0;  // packed row of (first snapshot, v_lo); snapshot s adds s*nv
  int64_t state_off; // first row of the chunk in H0 / HN
  int32_t t_lo;
  int32_t w;
};

// A tile of up to kTileRows consecutive vertices of one chunk; the dense kernel walks the
// chunk's window for it.
struct DenseTile {
  int32_t chunk;
  int32_t v0;     // first vertex, relative to the chunk's v_lo
  int32_t nrows;
  int32_t pad;
};

struct GraphDev {
  int32_t T;
  int64_t N;
  const int64_t* const* rowptr;  // device array [T] of device pointers
  const int32_t* const* colidx;
};

#define DGC_HIP_TRY(expr)                                             \
  do {                                                                \
    hipError_t e_ = (expr);                                           \
    if (e_ != hipSuccess) {                                           \
      return fail(DGC_ERR_DEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    }                                                                 \
  } while (0)

// text that dgc_last_error(NULL) returns on the calling thread (dgc_api.hip)
void set_thread_error(const std::string& msg);

// ---- packing (dgc_pack.hip)
void launch_segment_bounds(const GraphDev& g, Segment* segs, int64_t nseg, hipStream_t st);
void launch_deg_inv_sqrt(const GraphDev& g, float* dinv, hipStream_t st);
void launch_mark_halo(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_nnz,
                      int64_t words_per_seg, uint32_t* bitmap, int32_t* flags /*[4]*/, hipStream_t st);
void launch_validate_rowptr(const GraphDev& g, int32_t* flags /*[4]*/, hipStream_t st);
// exclusive scan of `n` int64 counts (in place); total written to *total_dev (device int64).
// tmp must hold ceil(n/2048)+2 int64.
void launch_exclusive_scan(int64_t* data, int64_t n, int64_t* tmp, int64_t* total_dev, hipStream_t st);
int64_t scan_tmp_elems(int64_t n);
void launch_popcount_words(const uint32_t* bitmap, int64_t n_words, int64_t* counts, hipStream_t st);
void launch_fill_halo(const uint32_t* bitmap, const int64_t* word_rank, int64_t nseg,
                      int64_t words_per_seg, int32_t* halo_idx, hipStream_t st);
void launch_seg_halo_off(const int64_t* word_rank, int64_t nseg, int64_t words_per_seg,
                         int64_t total_words, const int64_t* total_dev, Segment* segs,
                         int64_t* halo_ptr, hipStream_t st);
void launch_col_local(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_nnz,
                      int64_t words_per_seg, const uint32_t* bitmap, const int64_t* word_rank,
                      int32_t* col_local, hipStream_t st);
void launch_long_count(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_rows,
                       int32_t long_nnz, int32_t part_nnz, int64_t* counts, hipStream_t st);
void launch_long_fill(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_rows,
                      int32_t long_nnz, int32_t part_nnz, const int64_t* offs, int32_t* work_long,
                      hipStream_t st);
void launch_validate_graph(const GraphDev& g, int32_t* flags /*[4]*/, hipStream_t st);

// ---- redundant-loading estimate between chunks (dgc_fusion.hip)
// mask: T*N*ceil(n_chunks/64) words, out: n_chunks*n_chunks counters (upper triangle is filled)
int64_t shared_rows_mask_words(int32_t T, int64_t N, int32_t n_chunks);
void launch_shared_rows(const Segment* segs, int64_t nseg, const int64_t* halo_ptr, const int32_t* halo_idx, int32_t T,
                        int64_t N, int32_t n_chunks, unsigned long long* mask, unsigned long long* out, hipStream_t st);

// ---- aggregation / gather (dgc_spmm.hip)
// Spare entries after the last non-zero of the edge table: a lane group reads whole batches of 8
// entries, up to 8 * (groups per wave) - 1 entries past the end of the row it works on.
constexpr int64_t kEtabPad = 32;

struct SpmmArgs {
  GraphDev g;
  const Segment* segs;
  const int32_t* work_short;  // [n_short][3]
  int64_t n_short;
  const int32_t* work_long;   // [n_long][4]
  int64_t n_long;
  const float* dinv;          // [T*N]
  const float* fresh; int64_t ld_fresh;   // [T,N,ld]: rows inside the chunk range
  const float* stale; int64_t ld_stale;   // [T,N,ld]: cache rows (IN_PLACE)
  const float* halo; int64_t ld_halo;     // packed halo rows (STAGED) or nullptr
  const int32_t* col_local;               // STAGED only
  const int32_t* col_signed;              // generated chunks: stored columns marked j (fresh) / ~j (cache), or nullptr
  int32_t F;
  int32_t long_nnz, part_nnz;
  float* partial;             // [n_long][ldm] scratch for split rows
  float* M; int64_t ldm;      // [rows, ldm]; columns F..ldm-1 are written as zero
  const int64_t* row_map;     // nullptr, or [rows]: row of M that packed row r goes to (< 0: skip the row)
  int64_t ld_out;             // pitch of the rows of M if it differs from the written width ldm (0 = ldm)
  bool skip_stale;            // neighbours outside the row's chunk range contribute nothing
  // Edge table (IN_PLACE and generated chunks): one 8-byte entry per packed non-zero, in packed order
  // with kEtabPad spare entries at the end: .x = the stored column j if the neighbour is read fresh, ~j if it
  // is read from the cache; .y = the bits of the neighbour's degree scaling d_j^-1/2.  nullptr: the
  // kernels walk colidx and look the scaling up.
  const int2* etab;
};
void launch_spmm(const SpmmArgs& a, hipStream_t st);
// etab[p] for every packed non-zero p (col_signed: the marked columns of generated chunks, or nullptr:
// mark by the segment's vertex range); the kEtabPad spare entries are (0, 0).
void launch_edge_table(const GraphDev& g, const Segment* segs, int64_t nseg, int64_t total_nnz, const float* dinv,
                       const int32_t* col_signed, int2* etab, hipStream_t st);

void launch_gather(const Segment* segs, int64_t nseg, const int32_t* halo_idx, const int64_t* halo_ptr,
                   int64_t total_halo, int64_t N, const float* C, int64_t ldc, int32_t F, float* halo,
                   int64_t ldh, hipStream_t st);

// ---- dense part (dgc_dense.hip)
// Weights are kept in "fragment order" for the 32x32x2 fp32 MFMA: for W [n_out][n_in]
// (row-major), packed[(jb*nkb + kb)*64 + lane] is the float4
//   W[jb*32 + lane%32][kb*8 + (lane/32)*4 + 0..3]   (zero beyond n_in),  nkb = ceil(n_in/8).
void launch_pack_weight(const float* W, int32_t n_out, int32_t n_in, float4* packed, hipStream_t st);
inline int64_t packed_weight_elems(int32_t n_out, int32_t n_in) {
  return (int64_t)(n_out / 32) * ((n_in + 7) / 8) * 64 * 4;
}

struct DenseArgs {
  const DenseTile* tiles;       // 64-row tiles
  int64_t n_tiles;
  const DenseTile* tiles32;     // 32-row tiles
  int64_t n_tiles32;
  int32_t variant;              // DGC_DENSE_*
  const ChunkInfo* chunks;
  int64_t N;
  int64_t total_state_rows;     // V = sum of chunk vertex counts
  const float* M; int64_t ldm;  // packed aggregated rows
  int32_t K0;                   // columns of M that are used (input dim of the GCN layer)
  int32_t S, H;
  int32_t act;                  // activation after the GCN transform
  int32_t time_kind;
  const float4* Wg;             // packed GCN weight [S][K0] (one per snapshot if wg_step_bytes != 0)
  int64_t wg_bytes;             // size of the packed GCN weights
  int32_t wg_step_bytes;        // distance between consecutive snapshots' packed weights, or 0
  const float* bg;              // [S]
  const float4* Wih;            // packed [gH][S] ([gH][2S] with X2)
  const float4* Whh;            // packed [gH][H]
  const float* bih; const float* bhh;
  const float* H0;
  const uint8_t* reset_mask;
  float* Y; int64_t ldy;        // [T,N,ldy]
  float* HN;
  // Sequences inside the window (temporal fusion with states), indexed like reset_mask; both set or
  // both nullptr.  seq_in[t*N + v] >= 0: the row starts a sequence whose state row that is (the
  // incoming state becomes H0's row, or zero without H0); seq_out[...] >= 0: the row ends the
  // sequence of that state row (the new state goes to HN's row).  H0 / HN are then read / written
  // only through these tables.
  const int64_t* seq_in;
  const int64_t* seq_out;
  // With the sequence tables only: y_map[t*N + v] = row of Y (pitch ldy) that the output of (t, v)
  // goes to, negative = not stored; nullptr = row t*N + v.
  const int64_t* y_map;
  // Second half of the time encoder's input (the first structure layer's output), or nullptr: the
  // time encoder then reads [X2 row, Z] and Wih is packed [gH][2S].  Row of (t, v) in X2:
  // x2_map[t*N + v] (negative: any row, the output is not used), or t*N + v without a map.
  const float* X2; int64_t ldx2;
  const int64_t* x2_map;
  // A stacked recurrent layer (wave-private kernel only): the rows of M are rows t*N + v of a
  // [T,N,ldm] tensor (m_by_vertex) and are the time encoder's input as they are (input_is_z: no
  // transform, K0 = 0; Wg must still name readable packed weights, its fragments are prefetched).
  // M may be Y itself: a wave reads row (t, v) in step t and writes it one step later.
  bool m_by_vertex;
  bool input_is_z;
};
// returns false if the (S,H,K0) combination has no kernel
bool launch_dense(const DenseArgs& a, hipStream_t st, std::string* why);
bool dense_wave_supported(const DenseArgs& a);
bool launch_dense_wave(const DenseArgs& a, hipStream_t st, std::string* why);
size_t dense_lds_bytes(int32_t K0, int32_t S, int32_t H);
int dense_ld(int32_t K0, int32_t S, int32_t H);

// ---- EvolveGCN-O (dgc_evolve.hip)
enum { EV_W = 0, EV_UZ, EV_VZ, EV_BZ, EV_UR, EV_VR, EV_BR, EV_UH, EV_VH, EV_BH, EV_NPAR };

struct EvolveWs {
  int32_t T, F, S;
  const float* P[EV_NPAR];   // parameters (device, fp32): W_init, Uz, Vz, Bz, Ur, Vr, Br, Uh, Vh, Bh
  float* G[EV_NPAR];         // their gradients (fp32, what the caller reads)
  double* Pd[EV_NPAR];       // the parameters widened to double for the weight recurrence
  double* Gd[EV_NPAR];       // gradient accumulators of the back-propagation through time
  double *Wt, *Zg, *Rg, *Wc; // [T][F][S]: evolved weights and the gates that produced them
  float* Wt_f32;             // [T][F][S]: W_t rounded to fp32
  float4* Wt_packed;         // every W_t^T (fp32) in MFMA fragment order
  double* tmp[6];            // [F][S] scratch
  float* dWd;                // [T][F][S] direct gradient of each W_t
  float* partial;            // [T][split][F][S]
  float* loss_partial;       // [T][split]
  const DenseTile* items;    // 32-row tiles ordered by snapshot
  const int64_t* item_ptr;   // [T+1]
};

struct EvolveBwdIn {
  const ChunkInfo* chunks;
  int64_t N;
  const float* M; int64_t ldm;
  const float* Y; int64_t ldy;
  const float* dY; int64_t lddy;
  const float* target; int64_t ldt;
  int64_t count;             // number of output elements the loss averages over
  float* loss_out;           // device, or nullptr
};

int64_t evolve_partial_elems(int32_t T, int32_t F, int32_t S);
int64_t evolve_loss_partial_elems(int32_t T);
void evolve_forward_weights(const EvolveWs& ws, hipStream_t st);
bool evolve_backward_dw(const EvolveWs& ws, const EvolveBwdIn& in, hipStream_t st, std::string* why);
// input-gradient pass: dP = dL/d(pre-activation) of every covered row into packed rows [rows][ldp];
// the packed-row -> t*N + v table; every W_t as (out = F, in = S) fragments for dM = dP W_t^T
void evolve_backward_dp(const EvolveBwdIn& in, int32_t n_chunks, int64_t max_nv, int32_t max_w, int32_t S, float* dP,
                        int64_t ldp, hipStream_t st);
void evolve_row_index(const ChunkInfo* chunks, int32_t n_chunks, int64_t max_nv, int32_t max_w, int64_t N, int64_t* idx,
                      hipStream_t st);
void evolve_pack_weights_plain(const EvolveWs& ws, float4* packed, hipStream_t st);
void evolve_backward_bptt(const EvolveWs& ws, hipStream_t st);

// ---- graph attention + temporal self-attention, bf16 (dgc_dysat.hip)
enum { DY_W = 0, DY_ASRC, DY_ADST, DY_POS, DY_WQ, DY_WK, DY_WV, DY_NPAR };

struct DysatWs {
  int32_t T; int64_t N; int32_t n_chunks;
  GraphDev g;
  const Segment* segs; int64_t nseg;
  const ChunkInfo* chunks;
  const int32_t* work_short; int64_t n_short;   // row groups of the segments (segment, first row, rows)
  const int64_t* tile_ptr; int64_t n_tiles;     // tiles of the temporal kernels, per chunk: 2 vertices each, 1 if wide
  bool wide;                                    // some chunk's window is longer than 16 snapshots (at most 32)
  const int32_t* owner;                         // [T*N] covering chunk or -1
  const int32_t* used_t; int32_t n_used;        // snapshots some chunk covers
  int64_t total_rows;
  const float* P[DY_NPAR];   // fp32 parameters: gat.weight, att_src, att_dst, pos, W_q, W_k, W_v
  float* G[DY_NPAR];         // their gradients
  uint4 *Wp, *Wqp, *Wkp, *Wvp;   // bf16 operand fragments (row operand)
  uint4 *WqT, *WkT, *WvT, *WT;   // bf16 fragments of the transposes (backward)
  uint4* WTlo;                   // low part of W^T (W minus its bf16 rounding), for the input gradient
  uint16_t *zX, *zC;         // [T*N][128] half-precision projections of input and cache rows
  float *sX, *sC;            // attention scalars
  float* U;                  // [T*N][128] fp32 structure-encoder output before ELU
  float* lse;                // [T*N][8]
  // backward
  const void* X; int64_t ldx;                // inputs of the last forward (read again by backward)
  const void* C; int64_t ldc;
  uint16_t *dU, *dQ, *dK, *dV, *dzX, *dzC;   // [T*N][128] bf16
  uint16_t* dzXlo;                           // what dzX lost to rounding, for the input gradient (allocated on demand)
  float* st2;                // [T*N][8][4]: per head (s_dst, lse, c, d s_dst) of every covered row
  float* dss;                // [T*N][16]: d s_src of every vertex, as in-chunk neighbour [8] and as cache row [8]
  float* partial;            // scratch for the parameter-gradient reductions
  int64_t partial_elems;
  float* loss_partial;
  // rows longer than long_nnz are cut into parts of part_nnz non-zeros
  int32_t long_nnz, part_nnz;
  const int32_t* work_long; int64_t n_long;        // covered rows: (segment, local row, part, parts)
  const int32_t* cols_long; int64_t n_cols_long;   // all vertices: (snapshot, vertex, part, parts)
  float* long_partial;                             // one record per part
  // per stored non-zero (j, i) of the snapshots in use: 0 = row i not covered, 1 = i and j rows of
  // the same chunk, 2 = rows of different chunks; snapshot t starts at ecode_off[t]
  const uint8_t* ecode; const int64_t* ecode_off;
};
void dysat_edge_code(const GraphDev& g, const int32_t* used_t, int32_t n_used, const int32_t* owner,
                     const int64_t* ecode_off, uint8_t* ecode, hipStream_t st);

int64_t dysat_partial_elems(const DysatWs& ws);
int64_t dysat_long_partial_elems(const DysatWs& ws);
// list of the split rows among all vertices of the snapshots in use; *counter (device, zero on
// entry) receives the number of parts; list may be NULL (count only)
void dysat_cols_long(const GraphDev& g, const int32_t* used_t, int32_t n_used, int32_t long_nnz, int32_t part_nnz,
                     int32_t* counter, int32_t* list, hipStream_t st);
int64_t dysat_loss_partial_elems(const DysatWs& ws);
// ev: NULL or 4 events recorded around the three backward stages
void dysat_backward(const DysatWs& ws, const void* Y, int64_t ldy, const void* dY, int64_t lddy, const void* target,
                    int64_t ldt, float* loss_out, void* dX, int64_t lddx, hipEvent_t* ev, hipStream_t st);
void dysat_build_owner(const Segment* segs, int64_t nseg, int32_t T, int64_t N, int32_t* owner, hipStream_t st);
void dysat_pack_params(const DysatWs& ws, hipStream_t st);
// ev: NULL or 4 events recorded around the three forward stages
void dysat_forward(const DysatWs& ws, const void* X, int64_t ldx, const void* C, int64_t ldc, void* Y, int64_t ldy,
                   hipEvent_t* ev, hipStream_t st);

// ---- temporal fusion (dgc_tfusion.hip)
struct TFusion {
  bool built = false;
  int64_t n_lanes = 0;       // lanes of all chunks
  int32_t Lmax = 0;          // longest window
  int64_t rows_v = 0;        // sum over chunks of lanes x window
  int64_t* lane_ptr = nullptr;    // [n_chunks+1] first lane of every chunk
  int64_t* slot_row = nullptr;    // [Lmax][n_lanes] t*N + i of the row in the slot, -1 = empty
  int64_t* row_map = nullptr;     // [total rows] inverse: packed row -> row of Mv (lane order), -1 = absent
  int64_t* seq_in = nullptr;      // [Lmax][n_lanes] state row of the sequence that starts in the slot, else -1
  int64_t* seq_out = nullptr;     // [Lmax][n_lanes] state row of the sequence that ends in the slot, else -1
  int32_t* seq_len = nullptr;     // [state rows] present snapshots of every (chunk, vertex)
  uint8_t* slot_reset = nullptr;  // [Lmax][n_lanes] 1 on the first slot of every sequence
  ChunkInfo* chunks_v = nullptr;  // the lanes of chunk k as a chunk: v_lo = first lane, nv = lanes, t_lo = 0
  DenseTile* tiles_v = nullptr; int64_t n_tiles_v = 0;
  DenseTile* tiles32_v = nullptr; int64_t n_tiles32_v = 0;
  float* Mv = nullptr;            // [rows_v][ldm] aggregated rows in lane order
};
void tf_lengths(const uint8_t* present, const ChunkInfo* chunks, int32_t n_chunks, int64_t max_nv, int64_t N,
                int32_t* seq_len, hipStream_t st);
void tf_fill(const uint8_t* present, const ChunkInfo* chunks, int32_t n_chunks, int64_t max_nv, int64_t N,
             const int32_t* seq_lane, const int32_t* seq_off, int64_t n_lanes, int32_t Lmax, const ChunkInfo* chunks_v,
             int64_t total_rows, int64_t* slot_row, int64_t* row_map, uint8_t* slot_reset, int64_t* seq_in,
             int64_t* seq_out, hipStream_t st);
void tf_carry(const int32_t* seq_len, int64_t V, int32_t n_state, int32_t H, const float* H0, float* HN, hipStream_t st);
// temporal fusion over generated chunks: sequences = runs of present instances with one label
void lp_sequences(const uint8_t* present, const int32_t* labels, int32_t T, int64_t N, int32_t* seq_len, int32_t* first_t,
                  int32_t* pos, uint8_t* last, hipStream_t st);
void lp_fill(const uint8_t* present, const int32_t* first_t, const int32_t* pos, const uint8_t* last,
             const int32_t* seq_lane, const int32_t* seq_off, int32_t T, int64_t N, int64_t n_lanes, int64_t* slot_row,
             int64_t* row_map, uint8_t* slot_reset, int64_t* seq_in, int64_t* seq_out, hipStream_t st);

// ---- generated chunks (dgc_labels.hip)
struct Labelled {
  bool built = false;
  int32_t* col_signed = nullptr;  // [total nnz] see SpmmArgs
  int64_t* seq_in = nullptr;      // [T*N] see DenseArgs
  int64_t* seq_out = nullptr;
  int32_t* labels = nullptr;      // [T*N] copy of the labels (a later dgc_layer_set_presence reads them)
};
void labels_build(const GraphDev& g, const Segment* segs, const int32_t* labels, int32_t* col_signed,
                  int64_t* seq_in, int64_t* seq_out, hipStream_t st);

}  // namespace dgc
