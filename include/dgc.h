/*
 * dgc.h - C ABI of the fused-chunk dynamic-GNN layer for AMD MI355X (gfx950).
 *
 * The layer is the DGNN block of the paper's Section 2.1 (a structure encoder over every
 * snapshot followed by a time encoder over every vertex's sequence), executed over a fused
 * batch of graph chunks (Section 4: a chunk is a sub-graph across spatial and temporal
 * boundaries; here a vertex range x a window of snapshots).  All chunks of a batch run in the
 * same launches (spatial fusion, Section 5.1.1); a neighbour outside a row's own chunk range
 * is read from a cache of earlier ("last transmitted") embeddings instead of the fresh input
 * (Section 5.2); the recurrent state entering a step can be masked off per row (temporal
 * fusion mask, Section 5.1.2).  Encoders: GCN convolution, GRU, LSTM (Section 6).
 *
 * Conventions
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *    host memory.  The library never frees caller memory and only borrows it while the work
 *    it enqueued is running.
 *  - Floating tensors are row-major with a base address aligned to 16 bytes; their element type
 *    is the layer's dtype: fp32 (row pitch ld*, in elements, a multiple of 4) or bfloat16 (pitch a
 *    multiple of 8), passed as void*.  Parameters and their gradients are always fp32.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - forward / backward / aggregate / gather / stale_filter only enqueue work: they return
 *    argument errors at once and never synchronise the device, so a caller may record them into a
 *    HIP graph (backward allocates workspace on its first call with dX: make one eager call
 *    first).  create / set_param / get_param / packing / set_presence / set_labels /
 *    shared_rows / chunk_generate synchronise.
 *  - Every function returns DGC_OK (0) or an error code; dgc_last_error gives the text.
 *  - A layer object is not thread-safe; different layers may be used from different threads.
 */
#ifndef DGC_H_
#define DGC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dgc_layer dgc_layer_t; /* opaque, owned by the library */

typedef enum {
  DGC_OK = 0,
  DGC_ERR_INVALID_ARG = 1, /* null pointer, bad size, pitch or alignment, unknown name      */
  DGC_ERR_BAD_GRAPH = 2,   /* CSR arrays violate the graph contract                          */
  DGC_ERR_BAD_CHUNK = 3,   /* chunk empty, outside [0,N) x [0,T), or overlapping another     */
  DGC_ERR_UNSUPPORTED = 4, /* a combination of options that is not built                     */
  DGC_ERR_OOM = 5,         /* device or host allocation failed                               */
  DGC_ERR_DEVICE = 6,      /* a HIP call failed (no device, launch error)                    */
  DGC_ERR_STATE = 7        /* call order (backward before forward, ...)                      */
} dgc_status_t;

/* Structure encoder: GCN convolution with fixed weights, or EvolveGCN-O (the GCN weight matrix
 * is the state of a matrix GRU and evolves from snapshot to snapshot; Section 1 lists EvolveGCN
 * among the DGNNs the method targets). */
enum { DGC_STRUCT_GCN = 0, DGC_STRUCT_EVOLVE_GCN_O = 1, DGC_STRUCT_GAT = 2 };
enum { DGC_TIME_NONE = 0, DGC_TIME_GRU = 1, DGC_TIME_LSTM = 2, DGC_TIME_SELF_ATTN = 3 };
enum { DGC_ACT_NONE = 0, DGC_ACT_RELU = 1 };
enum { DGC_DTYPE_F32 = 0, DGC_DTYPE_BF16 = 1 };
/* DGC_STRUCT_GAT + DGC_TIME_SELF_ATTN + DGC_DTYPE_BF16 (the three go together) is the DySAT-style
 * DGNN of Sections 2.1 and 6: a one-layer graph attention structure encoder and a one-layer
 * scaled dot-product self-attention time encoder in which every vertex attends, causally, to
 * its own embeddings in the snapshots of the chunk's window.  Built for F = S = 128, heads = 8,
 * windows of at most 32 snapshots (two vertices share a 32-row tile while every window is at
 * most 16, else a tile is one vertex); act_hidden / act_out / gather_mode / dense_kernel are ignored
 * (ELU follows the structure encoder; neighbours are read in place):
 *   z = W x for rows inside the chunk range, W c for cache rows;
 *   e_ij^h = LeakyReLU_0.2(a_dst^h . z_i^h + a_src^h . z_j^h), alpha = softmax over the stored row,
 *   g_i = ELU(sum_j alpha_ij z_j);  p_s = g_s + pos[s] (s = absolute snapshot index);
 *   q, k, v = W_q p, W_k p, W_v p;  y_s^h = sum_{r <= s, r in window} softmax_r(q_s^h . k_r^h / 4) v_r^h. */
/* How rows of neighbours outside the chunk reach the aggregation (Section 5.2):
 *  IN_PLACE the aggregation kernel reads the cache tensor directly;
 *  STAGED   a gather kernel first copies each segment's de-duplicated halo rows (loaded once
 *           per segment, Section 5.1.1) into a buffer that the aggregation then indexes
 *           through the packed local column ids. */
enum { DGC_GATHER_IN_PLACE = 0, DGC_GATHER_STAGED = 1 };
/* Which kernel runs the dense transform + time encoder:
 *  AUTO  the wave-private kernel where it applies, else the workgroup-tile kernel;
 *  TILE  64 vertices per workgroup, operands shared through LDS (any S, H up to 256);
 *  WAVE  32 vertices per wavefront, hidden state kept in registers, no barriers
 *        (S = H in {32, 64, 128}); DGC_ERR_UNSUPPORTED at forward otherwise. */
enum { DGC_DENSE_AUTO = 0, DGC_DENSE_TILE = 1, DGC_DENSE_WAVE = 2 };
/* Which kernels aggregate in IN_PLACE mode (STAGED always takes WALK):
 *  TABLE  kernels that read a per-non-zero table built at create (8 bytes per stored non-zero: the column,
 *         marked fresh / cache, and the neighbour's degree scaling); needs equal pitches of X and C and
 *         F <= 256, else WALK runs;
 *  WALK   kernels that walk colidx, test the chunk range and look the scaling up (no table).
 * Results differ only in summation order. */
enum { DGC_AGG_TABLE = 0, DGC_AGG_WALK = 1 };

/* A chunk: vertices [v_lo, v_hi) over snapshots [t_lo, t_hi). */
typedef struct {
  int64_t v_lo, v_hi;
  int32_t t_lo, t_hi;
} dgc_chunk_t;

/* A dynamic graph (Section 2.1): T snapshots over the same N vertex ids.  rowptr / colidx
 * are HOST arrays of T DEVICE pointers.  Snapshot t: rowptr[t] is int64[N+1] with
 * rowptr[t][0] = 0; colidx[t] is int32[rowptr[t][N]], ascending and unique within a row, the
 * self-loop (i,i) stored for every vertex, symmetric (undirected).  The arrays must stay
 * valid and unchanged for the life of the layer. */
typedef struct {
  int32_t T;
  int64_t N;
  const int64_t* const* rowptr;
  const int32_t* const* colidx;
} dgc_graph_t;

typedef struct {
  int32_t struct_kind;     /* DGC_STRUCT_*                                                   */
  int32_t n_struct_layers; /* 1 or 2 stacked GCN layers                                      */
  int32_t time_kind;       /* DGC_TIME_*                                                     */
  int32_t dtype;           /* DGC_DTYPE_*: element type of X, C, Y, dY, target               */
  int32_t F, S, H;         /* input dim, structure-encoder output dim, hidden dim.  S and H
                              multiples of 32, at most 256; F at most 512.  Where the
                              workgroup-tile kernel runs (DGC_DENSE_TILE, or S, H outside what
                              DGC_DENSE_WAVE takes) its operand tile lives in LDS:
                              max(F rounded up to 8, S, H) <= 304, else DGC_ERR_UNSUPPORTED   */
  int32_t act_hidden;      /* activation between stacked GCN layers                          */
  int32_t act_out;         /* activation after the last GCN layer                            */
  int32_t gather_mode;     /* DGC_GATHER_*                                                   */
  int32_t validate_level;  /* 0: O(chunks) checks; 1: also O(nnz) checks of the CSR contract */
  int32_t rows_per_group;  /* work list: rows per group, at most 32 (0 = default: 16, halved
                              down to 1 while the batch has fewer than 8192 groups)          */
  int32_t long_nnz;        /* work list: rows longer than this are split (0 = default 1024)  */
  int32_t part_nnz;        /* work list: non-zeros per part of a split row (0 = default 512) */
  int32_t dense_kernel;    /* DGC_DENSE_*                                                    */
  int32_t heads;           /* attention heads (DGC_STRUCT_GAT: 8; otherwise ignored)         */
  int32_t lstm_input_concat; /* 1: the LSTM reads both GCN layers' outputs side by side, first
                              layer first (Section 6, MPNN-LSTM); rnn.weight_ih is then
                              [4H, 2S].  Needs DGC_STRUCT_GCN, two layers, DGC_TIME_LSTM
                              (else DGC_ERR_INVALID_ARG) and S = H in {32, 64, 128} with
                              dense_kernel not DGC_DENSE_TILE (else DGC_ERR_UNSUPPORTED)     */
  int32_t agg_kernel;      /* DGC_AGG_*                                                      */
  int32_t n_time_layers;   /* 0 or 1: one recurrent layer; 2: a second GRU / LSTM layer of the same
                              width stacked on the first (Section 6: MPNN-LSTM has two LSTM layers),
                              reading its output step by step; Y is the second layer's output.
                              Needs DGC_STRUCT_GCN, a recurrent time_kind (else
                              DGC_ERR_INVALID_ARG) and S = H in {32, 64, 128} with dense_kernel not
                              DGC_DENSE_TILE (else DGC_ERR_UNSUPPORTED).  With dgc_layer_set_presence /
                              dgc_layer_set_labels the second layer steps through the same sequences;
                              its state blocks follow the first layer's in H0 / HN               */
} dgc_layer_desc_t;

/* Build a layer for a fixed graph and a fixed set of chunks (the paper partitions once per
 * training job, Section 7.5).  Validates, runs chunk-fusion packing on the device (Section
 * 5.1.1: segment offsets, de-duplicated halo lists, local column ids, the row-group work
 * list, per-row degree scaling), allocates the workspace and zero-initialised parameters.
 *  desc, graph, chunks: host.  chunks must be non-empty, inside the graph and pairwise
 *  disjoint in (vertex, snapshot) space, else DGC_ERR_BAD_CHUNK.
 *  *out receives the layer (NULL on failure).  Synchronises `stream`. */
dgc_status_t dgc_layer_create(const dgc_layer_desc_t* desc, const dgc_graph_t* graph,
                              const dgc_chunk_t* chunks, int32_t n_chunks, void* stream,
                              dgc_layer_t** out);

/* Release the layer, its workspace and parameters.  NULL is accepted. */
dgc_status_t dgc_layer_destroy(dgc_layer_t* layer);

/* Parameters, fp32, (out, in) row-major as in the recurrent units Section 6 names:
 *  "gcn0.weight" [S,F]  "gcn0.bias" [S]   "gcn1.weight" [S,S]  "gcn1.bias" [S]  (2 layers)
 *  "rnn.weight_ih" [gH,S] ([gH,2S] with lstm_input_concat)  "rnn.weight_hh" [gH,H]
 *  "rnn.bias_ih" [gH]  "rnn.bias_hh" [gH]
 *  g = 3 (GRU, gate order r,z,n) or 4 (LSTM, gate order i,f,g,o).
 *  n_time_layers = 2 adds "rnn1.weight_ih" [gH,H] "rnn1.weight_hh" [gH,H] "rnn1.bias_ih" "rnn1.bias_hh".
 * DGC_STRUCT_EVOLVE_GCN_O (needs F = S, time_kind NONE, one layer, act_out RELU) has instead
 *  "evolve.W_init" [F,S] (in, out)   "evolve.U_z" "evolve.V_z" "evolve.U_r" "evolve.V_r"
 *  "evolve.U_h" "evolve.V_h" [F,F]   "evolve.B_z" "evolve.B_r" "evolve.B_h" [F,S]:
 *    Zg = sig(U_z W + V_z W + B_z)  Rg = sig(U_r W + V_r W + B_r)
 *    Wc = tanh(U_h W + V_h (Rg*W) + B_h)   W_t = (1 - Zg)*W + Zg*Wc,   W = W_{t-1}, W_{-1} = W_init,
 *  for t = 0..T-1 whatever the chunk windows are, and Y[t,i] = relu(M[t,i] W_t).
 * DGC_STRUCT_GAT has "gat.weight" [S,F] (out, in)  "gat.att_src" "gat.att_dst" [heads, S/heads]
 *  "attn.pos" [T,S]  "attn.weight_q" "attn.weight_k" "attn.weight_v" [S,S] (out, in); values are
 *  rounded to bfloat16 where the kernels use them as matrix operands.
 *  After dgc_layer_backward, "<name>.grad" reads the gradient of that parameter (get only).
 * host_src / host_dst: host, numel elements; numel must equal the parameter's size. */
dgc_status_t dgc_layer_set_param(dgc_layer_t* layer, const char* name, const float* host_src,
                                 int64_t numel);
dgc_status_t dgc_layer_get_param(dgc_layer_t* layer, const char* name, float* host_dst,
                                 int64_t numel);

/* Forward pass of the whole layer over the fused batch.
 *  X  device [T,N,ldx]: input features x_{i,t} (Section 2.1).
 *  C  device [T,N,ldc]: cache of stale input embeddings, read for every neighbour outside the
 *     row's chunk vertex range (Section 5.2); may alias X (then chunking is invisible).
 *  C1 device [T,N,ldc1]: cache of stale inputs of the second GCN layer; NULL unless
 *     n_struct_layers = 2.
 *  H0 device [n_state * V, H], V = sum of chunk vertex counts, chunk k's rows starting at the
 *     sum of earlier chunks' vertex counts: state entering each chunk's first snapshot; for
 *     LSTM n_state = 2, hidden states first, then cell states.  With n_time_layers = 2 the second
 *     layer's n_state blocks follow the first layer's ([2 * n_state * V, H]).  NULL = zeros.
 *  reset_mask device uint8 [T,N] or NULL: a non-zero byte at (t,i) zeroes the state entering
 *     step t of vertex i (Section 5.1.2).
 *  Y  device [T,N,ldy]: output h_t (or the structure encoder's output if time_kind = NONE);
 *     only rows covered by a chunk are written.
 *  HN device, same shape as H0, or NULL: state after each chunk's last snapshot.
 * X, C, C1, H0, reset_mask must not overlap Y or HN. */
dgc_status_t dgc_layer_forward(dgc_layer_t* layer, const void* X, int64_t ldx, const void* C,
                               int64_t ldc, const void* C1, int64_t ldc1, const float* H0,
                               const uint8_t* reset_mask, void* Y, int64_t ldy, float* HN,
                               void* stream);

/* Temporal fusion (Section 5.1.2).  present device uint8 [T,N]: a non-zero byte says that vertex
 * i exists in snapshot t.  The sequence of a vertex in a chunk is then the ascending list of the
 * window's snapshots in which it is present; instead of padding every sequence to the window,
 * the sequences of a chunk are concatenated into lanes as long as the window (first-fit
 * decreasing: sequences by length descending then vertex ascending, each into the first lane in
 * order of creation with room for all of it) and the first slot of every sequence carries a reset
 * flag (the paper's mask: the previous sequence's state does not enter that step).  After this
 * call dgc_layer_forward runs the time encoder over the lanes: Y is written only for present rows
 * of the chunks and a vertex's state is carried over the snapshots it is absent from.  H0 and HN
 * keep the layout they have without fusion (one row per (chunk, vertex)): a sequence starts from
 * its row of H0 (zero if H0 is NULL), HN receives the state after the vertex's last present
 * snapshot of the window, and a vertex that is absent throughout the window keeps its state
 * (HN row = H0 row), so chained windows equal one long window.  reset_mask must be NULL
 * (DGC_ERR_INVALID_ARG).  For DGC_STRUCT_GCN with DGC_TIME_GRU / DGC_TIME_LSTM; can be called
 * once per layer (DGC_ERR_STATE otherwise); `present` is only read during the call.
 * Synchronises `stream`.
 * On a layer that has labels (dgc_layer_set_labels before this call; Sections 5.1.2 and 4.1
 * together) the sequences are a vertex's maximal runs of PRESENT instances that carry one label
 * (the label of an absent instance plays no part; the state is carried over the gaps inside a
 * run); all sequences, ordered by (length descending, vertex ascending, first snapshot ascending),
 * go first-fit into lanes of T slots.  H0 / HN keep the labelled layer's layout [n_state * T*N, H]:
 * a sequence starts from row t*N + i of its first instance (zero if H0 is NULL) and HN's row of
 * its last instance receives its final state; other rows are not written.  The labels cannot be
 * set again afterwards (DGC_ERR_STATE). */
dgc_status_t dgc_layer_set_presence(dgc_layer_t* layer, const uint8_t* present, void* stream);

/* Generated chunks as the layer's input (Sections 4.1 and 5.2): labels device int32 [T*N], any
 * values (what dgc_chunk_generate wrote, for instance); a chunk is the set of (snapshot, vertex)
 * pairs with one label.  For a layer created with DGC_STRUCT_GCN or DGC_STRUCT_EVOLVE_GCN_O (there
 * only the aggregation changes: forward, backward and the input gradient read a neighbour's fresh
 * row where the labels agree and the cache row, a constant, where they do not), DGC_GATHER_IN_PLACE and the
 * single chunk [0,N) x [0,T) (DGC_ERR_STATE otherwise; the rectangle only says which rows exist).
 * After this call dgc_layer_forward computes, for every (t, i):
 *   aggregation: neighbour j of snapshot t contributes X[t,j] (for the second GCN layer the first
 *     one's output) if labels[t,j] == labels[t,i], else the cache row C[t,j] (C1[t,j]);
 *   time encoder: the state entering step t is the vertex's own state after step t-1 if
 *     labels[t-1,i] == labels[t,i]; else, and at t = 0, it is row t*N + i of H0 (zero if H0 is
 *     NULL): H0 is then the stale-state cache, [n_state * T*N, H], cell rows after all hidden rows;
 *   HN (optional, same shape): row t*N + i receives the state after step t wherever the next step
 *     belongs to another chunk (t = T-1 or labels[t+1,i] != labels[t,i]); other rows are not written.
 * reset_mask must be NULL.  May be called again with other labels; `labels` is only read during
 * the call, until dgc_layer_set_presence has been called on the layer (then DGC_ERR_STATE: labels
 * come first).  The packing arrays of the chunk-fusion packing and dgc_layer_shared_rows keep
 * describing the single rectangular chunk.  Synchronises `stream`. */
dgc_status_t dgc_layer_set_labels(dgc_layer_t* layer, const int32_t* labels, void* stream);

/* Backward pass: gradients of a scalar loss with respect to the layer's parameters, for the
 * batch of the last dgc_layer_forward on this layer (the layer keeps the aggregated rows of that
 * pass; a forward in between invalidates them).  Built for DGC_STRUCT_EVOLVE_GCN_O and
 * DGC_STRUCT_GAT; other layers return DGC_ERR_UNSUPPORTED.  DGC_ERR_STATE if no forward has run.
 * DGC_STRUCT_GAT needs a symmetric adjacency (its gradient with respect to a neighbour's
 * projection is gathered through the reverse edge).
 *  Y      device [T,N,ldy]: the output that forward wrote, unchanged.
 *  Exactly one of
 *   dY     device [T,N,lddy]: gradient of the loss with respect to Y (rows not covered by a
 *          chunk are ignored), or
 *   target device [T,N,ldt]: the loss is the mean squared error between Y and target over all
 *          covered elements; *loss_out (device float, may be NULL) receives its value.
 *  dX     device [T,N,lddx], element type as X, or NULL: gradient with respect to the input
 *          rows.  Rows covered by a chunk are written (a row's gradient comes from the rows of its
 *          own chunk that store it as a neighbour), other rows and the pitch padding are left
 *          alone.  DGC_STRUCT_EVOLVE_GCN_O: computing it uses up the aggregated rows the layer
 *          kept, so a further backward needs a forward first (DGC_ERR_STATE); the first such
 *          call allocates T*N*F floats of workspace.  DGC_STRUCT_GAT: bfloat16, lddx a multiple
 *          of 8; one more product per row on top of the parameter gradients.
 * The cache is a constant: no gradient flows into C.  Gradients are read with
 * dgc_layer_get_param(layer, "<name>.grad", ...).  Enqueues work only. */
dgc_status_t dgc_layer_backward(dgc_layer_t* layer, const void* Y, int64_t ldy, const void* dY,
                                int64_t lddy, const void* target, int64_t ldt, float* loss_out,
                                void* dX, int64_t lddx, void* stream);

/* Steps of the path on their own (for measurement and element-wise checks).
 * dgc_layer_aggregate: the normalised neighbour aggregation of the first GCN layer,
 *   M[row] = sum_j (d_i d_j)^(-1/2) src(t,j), d = stored row length in the full snapshot,
 *   for every row of the fused batch in packed order (segment after segment, rows of a segment
 *   in vertex order).  M device [rows, ldm], ldm >= F.
 * dgc_layer_gather: the stale-cache gather of STAGED mode: halo device [halo_rows, ldh]
 *   receives C[t, halo_idx[p], :] for every packed halo slot p.  Works in either mode. */
dgc_status_t dgc_layer_aggregate(dgc_layer_t* layer, const float* X, int64_t ldx, const float* C,
                                 int64_t ldc, float* M, int64_t ldm, void* stream);
dgc_status_t dgc_layer_gather(dgc_layer_t* layer, const float* C, int64_t ldc, float* halo,
                              int64_t ldh, void* stream);

/* Per-stage device time, from HIP events recorded on the caller's stream (for measurement;
 * adds no synchronisation to forward / backward themselves).  Stages:
 *  0 aggregation of the first GCN layer (gather + split-row reduction included)
 *  1 first GCN layer's dense transform            (0 ms unless n_struct_layers = 2)
 *  2 aggregation of the second GCN layer          (0 ms unless n_struct_layers = 2)
 *  3 last GCN layer's dense transform fused with the time encoder
 *  4 evolution of the GCN weights over the T snapshots   (EvolveGCN-O forward, else 0 ms)
 *  5 backward: weight-gradient reduction over the rows of every snapshot (+ loss)
 *  6 backward: back-propagation through time over the weight recurrence
 *  7 graph attention: projection of input and cache rows       (DGC_STRUCT_GAT forward)
 *  8 graph attention: edge softmax + aggregation
 *  9 temporal self-attention
 * 10 backward: temporal self-attention and its weight gradients
 * 11 backward: graph attention, gradients of the attention logits (row pass)
 * 12 backward: graph attention, gradients of the projections (reverse-edge pass) and of W
 * dgc_layer_set_profiling: enable != 0 makes every later forward / backward record the events.
 * dgc_layer_stage_times: waits for the last profiled forward (and backward, if one followed it)
 * and writes DGC_N_STAGES durations in milliseconds to host_ms (host); stages that did not run
 * read 0; DGC_ERR_STATE if no profiled forward was enqueued. */
#define DGC_N_STAGES 13
dgc_status_t dgc_layer_set_profiling(dgc_layer_t* layer, int32_t enable);
dgc_status_t dgc_layer_stage_times(dgc_layer_t* layer, float* host_ms);

/* Read back a packing array (host_dst: host).  `what` and element types:
 *  "seg_row_off" "seg_nnz_off" "halo_ptr"  int64 [n_segments+1]
 *  "halo_idx" int32 [halo_ptr[n_segments]]   "col_local" int32 [seg_nnz_off[n_segments]]
 *  "work_short" int32 [n][3] (segment, first local row, rows)
 *  "work_long"  int32 [n][4] (segment, local row, part, parts)
 *  "deg_inv_sqrt" fp32 [T*N]
 *  after dgc_layer_set_presence (DGC_ERR_STATE before): "lane_ptr" int64 [n_chunks+1] first lane of
 *  every chunk; "slot_row" int64 [Lmax][n_lanes] (Lmax = longest window, n_lanes = lane_ptr[n_chunks]):
 *  t*N + i of the row in that slot, -1 = empty; "slot_reset" uint8 [Lmax][n_lanes]
 * *needed_bytes (may be NULL) receives the array's size; data is copied only if
 * capacity_bytes is large enough (else DGC_ERR_INVALID_ARG, with *needed_bytes set).
 * Segments are ordered by chunk as given, then snapshot ascending. */
dgc_status_t dgc_layer_packing(dgc_layer_t* layer, const char* what, void* host_dst,
                               int64_t capacity_bytes, int64_t* needed_bytes);

/* Chunk generation by weighted label propagation (Section 4.1).  The super-graph has one vertex
 * x = t*N + i per (snapshot, vertex), the spatial edges of every snapshot (weight w_s; the stored
 * self-loops are not edges) and a virtual temporal edge between (t, i) and (t+1, i) (weight w_t);
 * the weights are the traffic an edge of each kind causes in the DGNN at hand, integers in
 * [0, 2^20] with (largest degree + 2) x weight below 2^32 (DGC_ERR_UNSUPPORTED otherwise: scores
 * are 32-bit sums).  Labels start all different (label of x = x, the section's initialisation with equal
 * snapshot sizes).  Every iteration works on the labels of the one before: a vertex scores each
 * neighbour label by the total weight of the edges to the neighbours carrying it; its candidate is
 * the label carried by fewer than `cap` vertices with the largest score (ties: the label carried
 * by fewer vertices, then the smaller label); it wants to change if the candidate scores strictly
 * more than its own label; of two adjacent vertices that want to change only the one that comes
 * first in the iteration's order does (iteration r, 0-based: by a fixed 32-bit mix of
 * x xor (r * 0x9E3779B9 mod 2^32), then by x).  Vertices whose answer cannot have changed are
 * skipped; the labels are those of looking at every vertex every time.  Ends when no vertex wants to change (*converged_out = 1) or after max_iters
 * iterations.  `cap` is soft: several vertices may join a label in the iteration in which it
 * reaches the limit.
 *  graph: as for dgc_layer_create (host struct of device arrays), checked against the graph contract
 *  (DGC_ERR_BAD_GRAPH); T*N < 2^31.  labels: device int32 [T*N], receives the label of every
 *  super-vertex (vertices with equal labels form a chunk).  iters_out, converged_out: host, may be
 *  NULL.  Allocates its workspace (24 bytes per super-vertex), synchronises `stream` once per
 *  iteration.  Errors: text in dgc_last_error(NULL). */
dgc_status_t dgc_chunk_generate(const dgc_graph_t* graph, int32_t w_s, int32_t w_t, int64_t cap,
                                int32_t max_iters, int32_t* labels, int32_t* iters_out,
                                int32_t* converged_out, void* stream);

/* Spatial-fusion selection (Section 5.1.1) and chunk assignment (Section 4.2, Algorithm 1).
 *
 * dgc_layer_shared_rows: the estimate of redundant loading between the chunks of the layer.  A
 *   chunk loads its own (snapshot, vertex) rows and, per snapshot of its window, the neighbours of
 *   its rows outside its vertex range; host_out (host int64 [n_chunks][n_chunks], symmetric, zero
 *   diagonal) entry (a, b) receives the number of rows both a and b load - loaded twice when the
 *   two are processed one after the other, once when they are fused.  Computed on the device from
 *   the packing; the first call allocates a bitmap of T*N*ceil(n_chunks/64) 8-byte words that the
 *   layer keeps (DGC_ERR_OOM if it does not fit); synchronises `stream`.
 *
 * dgc_fusion_select (host arithmetic): greedy fusion under a memory cap.  Every chunk starts as
 *   its own group; repeatedly, among the pairs of groups whose memories (sums of mem[], the
 *   per-chunk memory the caller measured) add up to at most `cap`, the pair with the largest shared
 *   amount (sum of shared[] over the members) is fused; ties go to the pair with the smallest
 *   (first, second) group, a group being named by its smallest member; stops when no pair fits.
 *   shared: int64 [n][n] symmetric, non-negative.  group_out int32 [n]: group of every chunk,
 *   groups numbered in ascending order of their smallest member.
 *
 * dgc_chunk_assign (host arithmetic): Algorithm 1.  Chunks in decreasing order of the predicted
 *   workload g[] (ties: smaller index first); chunk a goes to the GPU m with the largest
 *   s_m = (g_bar - sum of g over Q_m) * (sum of h(a, a') over a' in Q_m), g_bar = sum(g) / n_gpus,
 *   Q_m = the chunks already on m; equal scores go to the GPU with the smaller assigned load, then
 *   the smaller index.  g double [n], h double [n][n], x_out int32 [n].
 * The last two return DGC_ERR_INVALID_ARG with the text in dgc_last_error(NULL). */
dgc_status_t dgc_layer_shared_rows(dgc_layer_t* layer, int64_t* host_out, void* stream);
dgc_status_t dgc_fusion_select(int32_t n, const int64_t* shared, const int64_t* mem, int64_t cap,
                               int32_t* group_out);
dgc_status_t dgc_chunk_assign(int32_t n, const double* g, const double* h, int32_t n_gpus, int32_t* x_out);

/* Adaptive stale-embedding filter (Section 5.2): an embedding is transmitted again only if its L2
 * distance to the copy transmitted last exceeds a threshold that follows the training loss.  The
 * paper computes the distances on the CPU; here the whole step runs on the device.
 *
 * dgc_stale_theta_factor (host arithmetic): theta_r / D_r of the section's threshold equation from
 *   the initial loss l1 (> 0) and the loss of the epoch before, norm = (l1 - l_prev) / l1:
 *   DGC_THETA_PRINTED 1 / (1 + exp(norm)), the equation as printed (falls from 1/2 while the loss falls);
 *   DGC_THETA_SIGMOID 1 / (1 + exp(-norm)), the sign under which the threshold grows as the text
 *   around the equation says.  Returns a negative value for arguments outside the domain.
 *
 * dgc_stale_filter: E device [R, lde] current embeddings, L device [R, ldl] the copies transmitted
 *   last (updated in place; must not overlap E); element type `dtype` (DGC_DTYPE_F32 or
 *   DGC_DTYPE_BF16), pitches in elements and multiples of 16 bytes, 16-byte aligned.  Candidates: the rows listed in `rows`
 *   (device int64 [n_rows], ascending; entries outside [0, R) are skipped and counted in
 *   result->n_invalid), or every row if rows = NULL (then n_rows = 0).  For candidate c:
 *     dist[c] = || E[row] - L[row] ||_2 over the first F columns (fp32 arithmetic);
 *     D = max dist;  threshold = factor * D if factor >= 0, else `theta` (>= 0);
 *     row is transmitted iff dist[c] > threshold (compared in fp32).
 *   send_idx (device int64, room for every candidate) receives the transmitted row numbers in
 *   candidate order; send_buf (device [n, lds], same element type, may be NULL) row k receives E[send_idx[k]]; L[row]
 *   <- E[row] for the transmitted rows, every other row of L is left as it is.  result (device)
 *   receives the count, D and the threshold used.  dist device fp32 [candidates], 16-byte aligned.
 *   workspace: device, 8-byte aligned, at least dgc_stale_workspace_bytes(candidates) bytes,
 *   contents irrelevant before and after.  Enqueues work only (no synchronisation, no allocation,
 *   no memset); argument errors return at once with the text in dgc_last_error(NULL). */
enum { DGC_THETA_PRINTED = 0, DGC_THETA_SIGMOID = 1 };
typedef struct {
  int64_t n_send;    /* rows transmitted                        */
  float D;           /* largest distance among the candidates   */
  float theta;       /* threshold the selection used            */
  int64_t n_invalid; /* listed rows outside [0, R)              */
} dgc_stale_result_t;
double dgc_stale_theta_factor(double l1, double l_prev, int32_t variant);
int64_t dgc_stale_workspace_bytes(int64_t n_candidates);
dgc_status_t dgc_stale_filter(const void* E, int64_t lde, void* L, int64_t ldl, int64_t R, int32_t F,
                              int32_t dtype, const int64_t* rows, int64_t n_rows, double factor, double theta,
                              float* dist, int64_t* send_idx, void* send_buf, int64_t lds,
                              dgc_stale_result_t* result, void* workspace, int64_t workspace_bytes,
                              void* stream);

/* dgc_stale_filter for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same filter
 * with the same arguments and results, except that the block counts and scan temporaries live in a
 * fixed device array inside the library (272 KiB per GPU, held until the process ends) instead of
 * `workspace`.  At most dgc_stale_static_max_candidates() = 2^26 candidates (DGC_ERR_UNSUPPORTED
 * beyond, nothing enqueued).  Calls no hipMalloc / hipFree and no memset; the first call on a
 * device looks the array's address up (hipGetSymbolAddress, DGC_ERR_DEVICE if that fails).  Every
 * call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (two
 * streams, two threads) race and give undefined send lists - serialise them.  The array keeps the
 * last call's contents; nothing in it has to start at zero. */
int64_t dgc_stale_static_max_candidates(void);
dgc_status_t dgc_stale_filter_static(const void* E, int64_t lde, void* L, int64_t ldl, int64_t R, int32_t F,
                                     int32_t dtype, const int64_t* rows, int64_t n_rows, double factor,
                                     double theta, float* dist, int64_t* send_idx, void* send_buf, int64_t lds,
                                     dgc_stale_result_t* result, void* stream);

/* Text of the last error on this layer, or (layer = NULL) of the last failed create or layer-less
 * call on the calling thread.  Never NULL; valid until the next call on the same layer / thread. */
const char* dgc_last_error(const dgc_layer_t* layer);

/* Library version, e.g. "dgc 0.1 gfx950". */
const char* dgc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DGC_H_ */
