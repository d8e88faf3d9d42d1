/*
 * CPU oracle of the fused-chunk DGNN layer.  TEST INFRASTRUCTURE ONLY: the tests, the smoke
 * check and the benchmark's cpu_baseline leg call it; the product path never does.  It shares
 * no code with the HIP library.
 *
 * What it computes (the DGNN block of Section 2.1: a structure encoder over each snapshot,
 * then a time encoder over each vertex's sequence), restricted to chunks (Section 4: a chunk
 * is a sub-graph across spatial and temporal boundaries; here a vertex range x a snapshot
 * window), with neighbours outside the chunk's vertex range read from the cache of last
 * transmitted embeddings (Section 5.2).  The encoders are the ones Section 6 names: GCN
 * convolution, GRU, LSTM.  Section 5.1.2's mask multiplies the incoming hidden state.
 *
 * Everything is the plain definition: loops over rows and edges, double accumulation, no
 * blocking, no reordering.  Floating-point inputs and outputs are fp32; intermediates stay
 * in double.
 *
 * Parity pins (tests/test_oracle_*.py): dense-adjacency matmul on tiny graphs, a hand-worked
 * 4-vertex x 3-snapshot example, the sqrt-degree eigenvector, zero-in/zero-out, torch.nn.GRU
 * and torch.nn.LSTM in float64, concatenated-with-mask == separate sequences, cache == input
 * => chunked == unchunked, fused == one chunk at a time, brute-force packing with Python sets.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { TIME_NONE = 0, TIME_GRU = 1, TIME_LSTM = 2 };
enum { ACT_NONE = 0, ACT_RELU = 1 };

/* chunks: int64 [n][4] = v_lo, v_hi, t_lo, t_hi (half-open) */
#define CH_VLO(c, k) ((c)[4 * (k) + 0])
#define CH_VHI(c, k) ((c)[4 * (k) + 1])
#define CH_TLO(c, k) ((c)[4 * (k) + 2])
#define CH_THI(c, k) ((c)[4 * (k) + 3])

int64_t dgc_oracle_num_segments(const int64_t *chunks, int32_t n_chunks) {
  int64_t n = 0;
  for (int32_t k = 0; k < n_chunks; ++k) n += CH_THI(chunks, k) - CH_TLO(chunks, k);
  return n;
}

/* ---------------------------------------------------------------- chunk-fusion packing
 * Section 5.1.1: fused chunks are loaded and executed together and a vertex another chunk
 * depends on is loaded once.  One segment per (chunk, snapshot of its window), ordered by
 * chunk as given, then snapshot ascending.
 *   seg_row_off[s]  exclusive sum of segment row counts        [nseg+1]
 *   seg_nnz_off[s]  exclusive sum of segment stored non-zeros  [nseg+1]
 *   halo_ptr[s]     exclusive sum of segment halo sizes        [nseg+1]
 *   halo_idx        per segment: ascending, de-duplicated global ids of the columns that
 *                   fall outside the chunk's vertex range      [halo_ptr[nseg]]  (may be NULL)
 *   col_local       per stored non-zero, in packed order: j - v_lo if j is inside the range,
 *                   else (v_hi - v_lo) + position of j in the segment's halo list
 *                                                              [seg_nnz_off[nseg]] (may be NULL)
 * Call once with halo_idx = col_local = NULL to learn the sizes, then again to fill. */
int dgc_oracle_pack(int32_t T, int64_t N, const int64_t *const *rowptr, const int32_t *const *col,
                    const int64_t *chunks, int32_t n_chunks, int64_t *seg_row_off,
                    int64_t *seg_nnz_off, int64_t *halo_ptr, int32_t *halo_idx, int32_t *col_local) {
  int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
  if (!pos) return -1;
  int64_t s = 0;
  seg_row_off[0] = seg_nnz_off[0] = halo_ptr[0] = 0;
  for (int32_t k = 0; k < n_chunks; ++k) {
    const int64_t v_lo = CH_VLO(chunks, k), v_hi = CH_VHI(chunks, k);
    for (int64_t t = CH_TLO(chunks, k); t < CH_THI(chunks, k); ++t, ++s) {
      if (t < 0 || t >= T) { free(pos); return -2; }
      const int64_t e0 = rowptr[t][v_lo], e1 = rowptr[t][v_hi];
      for (int64_t j = 0; j < N; ++j) pos[j] = -1;
      for (int64_t e = e0; e < e1; ++e) {
        const int32_t j = col[t][e];
        if (j < v_lo || j >= v_hi) pos[j] = 0; /* marked */
      }
      int64_t n_halo = 0;
      for (int64_t j = 0; j < N; ++j) {
        if (pos[j] == 0) {
          if (halo_idx) halo_idx[halo_ptr[s] + n_halo] = (int32_t)j;
          pos[j] = (int32_t)n_halo++;
        }
      }
      if (col_local) {
        for (int64_t e = e0; e < e1; ++e) {
          const int32_t j = col[t][e];
          col_local[seg_nnz_off[s] + (e - e0)] =
              (j >= v_lo && j < v_hi) ? (int32_t)(j - v_lo) : (int32_t)(v_hi - v_lo) + pos[j];
        }
      }
      seg_row_off[s + 1] = seg_row_off[s] + (v_hi - v_lo);
      seg_nnz_off[s + 1] = seg_nnz_off[s] + (e1 - e0);
      halo_ptr[s + 1] = halo_ptr[s] + n_halo;
    }
  }
  free(pos);
  return 0;
}

/* Row-group work list of the fused launch (the rule is this build's own; the paper only asks
 * that fused chunks execute together, Section 5.1.1).  Two lists:
 *  short list: segments are visited snapshot by snapshot (t ascending; within a snapshot in
 *              chunk order), so that the rows being aggregated at any moment read the same
 *              snapshot's features.  Every segment is cut into groups of `rows_per_group`
 *              consecutive rows (the last group of a segment may be smaller):
 *              (segment, first local row, rows).  Rows longer than `long_nnz` stored non-zeros
 *              are left out of the sum there;
 *  long list : every such row, in packed (segment, row) order, is cut into ceil(nnz/part_nnz)
 *              parts of part_nnz non-zeros (the last may be smaller): (segment, local row,
 *              part, parts).
 * Segment numbers are those of dgc_oracle_pack (chunk as given, then snapshot).
 * Output arrays may be NULL to count only.  Returns 0; counts through n_short / n_long. */
int dgc_oracle_worklist(int32_t T, int64_t N, const int64_t *const *rowptr, const int64_t *chunks,
                        int32_t n_chunks, int32_t rows_per_group, int32_t long_nnz,
                        int32_t part_nnz, int32_t *short_list /*[n][3]*/, int64_t *n_short,
                        int32_t *long_list /*[n][4]*/, int64_t *n_long) {
  (void)N;
  int64_t ns = 0, nl = 0, s = 0;
  for (int32_t t = 0; t < T; ++t) {
    int64_t seg0 = 0; /* first segment of chunk k */
    for (int32_t k = 0; k < n_chunks; ++k) {
      const int64_t v_lo = CH_VLO(chunks, k), v_hi = CH_VHI(chunks, k);
      const int64_t t_lo = CH_TLO(chunks, k), t_hi = CH_THI(chunks, k);
      if (t >= t_lo && t < t_hi) {
        const int64_t seg = seg0 + (t - t_lo);
        for (int64_t r = 0; r < v_hi - v_lo; r += rows_per_group) {
          int64_t n = v_hi - v_lo - r;
          if (n > rows_per_group) n = rows_per_group;
          if (short_list) {
            short_list[3 * ns + 0] = (int32_t)seg;
            short_list[3 * ns + 1] = (int32_t)r;
            short_list[3 * ns + 2] = (int32_t)n;
          }
          ++ns;
        }
      }
      seg0 += t_hi - t_lo;
    }
  }
  for (int32_t k = 0; k < n_chunks; ++k) {
    const int64_t v_lo = CH_VLO(chunks, k), v_hi = CH_VHI(chunks, k);
    for (int64_t t = CH_TLO(chunks, k); t < CH_THI(chunks, k); ++t, ++s) {
      for (int64_t i = v_lo; i < v_hi; ++i) {
        const int64_t nnz = rowptr[t][i + 1] - rowptr[t][i];
        if (nnz > long_nnz) {
          const int64_t parts = (nnz + part_nnz - 1) / part_nnz;
          for (int64_t p = 0; p < parts; ++p) {
            if (long_list) {
              long_list[4 * nl + 0] = (int32_t)s;
              long_list[4 * nl + 1] = (int32_t)(i - v_lo);
              long_list[4 * nl + 2] = (int32_t)p;
              long_list[4 * nl + 3] = (int32_t)parts;
            }
            ++nl;
          }
        }
      }
    }
  }
  *n_short = ns;
  *n_long = nl;
  return 0;
}

/* ---------------------------------------------------------------- structure encoder: GCN
 * Symmetric-normalised aggregation of the GCN convolution (Section 6 names the operator):
 *   M[t,i] = sum over stored columns j of row i of snapshot t of
 *            (d[t,i] * d[t,j])^(-1/2) * src(t,j),
 * d = stored row length in the FULL snapshot (the self-loop is stored, so d >= 1);
 * src(t,j) = fresh[t,j] if v_lo <= j < v_hi, else the cache row stale[t,j] (Section 5.2).
 * `fresh` and `stale` are addressed as base + (t*N + j)*ld. */
static void aggregate_row(int64_t N, const int64_t *rp, const int32_t *cj, int64_t t, int64_t i,
                          int64_t v_lo, int64_t v_hi, const float *fresh, int64_t ld_fresh,
                          const double *fresh_d, const float *stale, int64_t ld_stale, int32_t F,
                          double *out) {
  for (int32_t f = 0; f < F; ++f) out[f] = 0.0;
  const double d_i = (double)(rp[i + 1] - rp[i]);
  for (int64_t e = rp[i]; e < rp[i + 1]; ++e) {
    const int64_t j = cj[e];
    const double d_j = (double)(rp[j + 1] - rp[j]);
    const double w = 1.0 / sqrt(d_i * d_j);
    if (j >= v_lo && j < v_hi) {
      if (fresh_d) { /* in-chunk rows of a previous layer, kept in double: [w][nv][F] slice */
        const double *src = fresh_d + (j - v_lo) * (int64_t)F;
        for (int32_t f = 0; f < F; ++f) out[f] += w * src[f];
      } else {
        const float *src = fresh + (t * N + j) * ld_fresh;
        for (int32_t f = 0; f < F; ++f) out[f] += w * (double)src[f];
      }
    } else {
      const float *src = stale + (t * N + j) * ld_stale;
      for (int32_t f = 0; f < F; ++f) out[f] += w * (double)src[f];
    }
  }
}

/* Aggregation only, for one chunk: M [w][nv][F] in double. */
int dgc_oracle_aggregate_chunk(int32_t T, int64_t N, const int64_t *const *rowptr,
                               const int32_t *const *col, const int64_t *chunk, const float *X,
                               int64_t ldx, const float *C, int64_t ldc, int32_t F, double *M) {
  const int64_t v_lo = chunk[0], v_hi = chunk[1], t_lo = chunk[2], t_hi = chunk[3];
  if (v_lo < 0 || v_hi > N || t_lo < 0 || t_hi > T) return -2;
  const int64_t nv = v_hi - v_lo;
  for (int64_t t = t_lo; t < t_hi; ++t) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = v_lo; i < v_hi; ++i)
      aggregate_row(N, rowptr[t], col[t], t, i, v_lo, v_hi, X, ldx, NULL, C, ldc, F,
                    M + ((t - t_lo) * nv + (i - v_lo)) * (int64_t)F);
  }
  return 0;
}

/* out[o] = act(b[o] + sum_k W[o][k] * in[k]);  W is [n_out][n_in] row-major (out, in). */
static void dense_row(const float *W, const float *b, int32_t n_out, int32_t n_in,
                      const double *in, int32_t act, double *out) {
  for (int32_t o = 0; o < n_out; ++o) {
    double acc = b ? (double)b[o] : 0.0;
    const float *w = W + (int64_t)o * n_in;
    for (int32_t k = 0; k < n_in; ++k) acc += (double)w[k] * in[k];
    if (act == ACT_RELU && acc < 0.0) acc = 0.0;
    out[o] = acc;
  }
}

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* One GRU step (the recurrent unit Section 6 names; gate order r, z, n in the stacked
 * weights).  hm is the incoming state already multiplied by the mask of Section 5.1.2.
 *   r = sig(W_ir x + b_ir + W_hr hm + b_hr)      z = sig(W_iz x + b_iz + W_hz hm + b_hz)
 *   n = tanh(W_in x + b_in + r * (W_hn hm + b_hn))     h' = (1 - z) * n + z * hm          */
static void gru_step(const float *Wih, const float *Whh, const float *bih, const float *bhh,
                     int32_t S, int32_t H, const double *x, const double *hm, double *gx,
                     double *gh, double *h_out) {
  dense_row(Wih, bih, 3 * H, S, x, ACT_NONE, gx);
  dense_row(Whh, bhh, 3 * H, H, hm, ACT_NONE, gh);
  for (int32_t j = 0; j < H; ++j) {
    const double r = sigmoid(gx[j] + gh[j]);
    const double z = sigmoid(gx[H + j] + gh[H + j]);
    const double n = tanh(gx[2 * H + j] + r * gh[2 * H + j]);
    h_out[j] = (1.0 - z) * n + z * hm[j];
  }
}

/* One LSTM step (gate order i, f, g, o).  hm, cm: masked incoming states.
 *   i,f,o = sig(W_i* x + b_i* + W_h* hm + b_h*)   g = tanh(...)
 *   c' = f * cm + i * g        h' = o * tanh(c')                                         */
static void lstm_step(const float *Wih, const float *Whh, const float *bih, const float *bhh,
                      int32_t S, int32_t H, const double *x, const double *hm, const double *cm,
                      double *gx, double *gh, double *h_out, double *c_out) {
  dense_row(Wih, bih, 4 * H, S, x, ACT_NONE, gx);
  dense_row(Whh, bhh, 4 * H, H, hm, ACT_NONE, gh);
  for (int32_t j = 0; j < H; ++j) {
    const double ig = sigmoid(gx[j] + gh[j]);
    const double fg = sigmoid(gx[H + j] + gh[H + j]);
    const double gg = tanh(gx[2 * H + j] + gh[2 * H + j]);
    const double og = sigmoid(gx[3 * H + j] + gh[3 * H + j]);
    c_out[j] = fg * cm[j] + ig * gg;
    h_out[j] = og * tanh(c_out[j]);
  }
}

/* The whole layer over a list of chunks.
 *  n_struct_layers 1: Z = act_out(M(X|C) W0^T + b0)
 *                  2: Z1 = act_hidden(M(X|C) W0^T + b0) for every row of the chunk, then
 *                     Z = act_out(M(Z1|C1) W1^T + b1); C1 is the cache of layer-1 inputs.
 *  input_concat (2 layers with a time encoder): the time encoder's input is the row [Z1, Z]
 *  of width 2S, both structure layers' outputs side by side as Section 6 describes for
 *  MPNN-LSTM, and Wih is [gH][2S]; otherwise it is Z and Wih is [gH][S].
 *  time_kind NONE: Y[t,i] = Z;  GRU / LSTM: per vertex recurrence over the chunk's window,
 *  starting from H0 (packed: chunk k's rows start at sum of earlier chunks' vertex counts;
 *  for LSTM the cell states follow all hidden states), Y[t,i] = h_t.
 *  reset_mask[t*N+i] != 0 zeroes the state entering step t (Section 5.1.2); NULL = none.
 *  subset_ptr/subset_idx (optional): per chunk, the vertices whose time encoder and last
 *  structure layer are evaluated (others are left untouched in Y); NULL = all.
 *  hN (optional): final states, packed like H0.
 *  n_time_layers 2 (stacked time encoder, as the two LSTM layers of Section 6's MPNN-LSTM): the
 *  second recurrent layer reads the first one's output h_t of the same step, has its own weights
 *  Wih2 [gH][H], Whh2 [gH][H], bih2, bhh2 and its own state, and Y[t,i] is ITS h_t.  H0 / hN then
 *  hold the first layer's states (hidden, then cell for the LSTM) followed by the second layer's,
 *  each block tot_v rows; the reset mask zeroes the incoming state of both layers.
 * Weights are (out, in) row-major fp32.  Returns 0, or <0 on a bad argument. */
static int forward_impl(int32_t T, int64_t N, const int64_t *const *rowptr,
                       const int32_t *const *col, const int64_t *chunks, int32_t n_chunks,
                       int32_t n_struct_layers, int32_t time_kind, int32_t act_hidden,
                       int32_t act_out, int32_t F, int32_t S, int32_t H, const float *X,
                       int64_t ldx, const float *C, int64_t ldc, const float *C1, int64_t ldc1,
                       const float *W0, const float *b0, const float *W1, const float *b1,
                       const float *Wih, const float *Whh, const float *bih, const float *bhh,
                       const float *H0, const uint8_t *reset_mask, const int64_t *subset_ptr,
                       const int64_t *subset_idx, float *Y, int64_t ldy, float *hN,
                       int32_t input_concat, int32_t n_time_layers, const float *Wih2,
                       const float *Whh2, const float *bih2, const float *bhh2) {
  if (n_struct_layers < 1 || n_struct_layers > 2) return -3;
  if (n_time_layers < 1 || n_time_layers > 2) return -3;
  if (n_time_layers == 2 && (time_kind == TIME_NONE || !Wih2 || !Whh2 || !bih2 || !bhh2)) return -3;
  const int64_t n_state = time_kind == TIME_LSTM ? 2 : 1;   /* state blocks per recurrent layer */
  if (n_struct_layers == 2 && (!C1 || !W1)) return -3;
  if (input_concat && (n_struct_layers != 2 || time_kind == TIME_NONE)) return -3;
  const int32_t Sx = input_concat ? 2 * S : S;   /* width of the time encoder's input */
  int64_t tot_v = 0;
  for (int32_t k = 0; k < n_chunks; ++k) tot_v += CH_VHI(chunks, k) - CH_VLO(chunks, k);
  int64_t row_base = 0;
  for (int32_t k = 0; k < n_chunks; ++k) {
    const int64_t v_lo = CH_VLO(chunks, k), v_hi = CH_VHI(chunks, k);
    const int64_t t_lo = CH_TLO(chunks, k), t_hi = CH_THI(chunks, k);
    if (v_lo < 0 || v_hi > N || v_lo >= v_hi || t_lo < 0 || t_hi > T || t_lo >= t_hi) return -2;
    const int64_t nv = v_hi - v_lo, w = t_hi - t_lo;
    double *Z1 = NULL;
    if (n_struct_layers == 2) {
      Z1 = (double *)malloc(sizeof(double) * (size_t)(w * nv * S));
      if (!Z1) return -1;
      /* With a subset, only the first-layer rows that a subset vertex reads are evaluated: its
       * own row and those of its neighbours inside the chunk range, snapshot by snapshot.  The
       * others would never be looked at; their slots of Z1 stay unset. */
      uint8_t *need = NULL;
      if (subset_ptr) {
        need = (uint8_t *)calloc((size_t)(w * nv), 1);
        if (!need) { free(Z1); return -1; }
        for (int64_t q = subset_ptr[k]; q < subset_ptr[k + 1]; ++q) {
          const int64_t i = subset_idx[q];
          if (i < v_lo || i >= v_hi) { free(need); free(Z1); return -2; }
          for (int64_t t = t_lo; t < t_hi; ++t) {
            need[(t - t_lo) * nv + (i - v_lo)] = 1;
            for (int64_t e = rowptr[t][i]; e < rowptr[t][i + 1]; ++e) {
              const int64_t j = col[t][e];
              if (j >= v_lo && j < v_hi) need[(t - t_lo) * nv + (j - v_lo)] = 1;
            }
          }
        }
      }
      for (int64_t t = t_lo; t < t_hi; ++t) {
#pragma omp parallel for schedule(dynamic, 64)
        for (int64_t i = v_lo; i < v_hi; ++i) {
          if (need && !need[(t - t_lo) * nv + (i - v_lo)]) continue;
          double *m = (double *)malloc(sizeof(double) * (size_t)F);
          aggregate_row(N, rowptr[t], col[t], t, i, v_lo, v_hi, X, ldx, NULL, C, ldc, F, m);
          dense_row(W0, b0, S, F, m, act_hidden, Z1 + ((t - t_lo) * nv + (i - v_lo)) * (int64_t)S);
          free(m);
        }
      }
      free(need);
    }
    const int64_t n_sub = subset_ptr ? subset_ptr[k + 1] - subset_ptr[k] : nv;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < n_sub; ++q) {
      const int64_t i = subset_ptr ? subset_idx[subset_ptr[k] + q] : v_lo + q;
      const int32_t Fl = n_struct_layers == 2 ? S : F;
      const int32_t g = time_kind == TIME_LSTM ? 4 : 3;
      double *buf = (double *)malloc(sizeof(double) * (size_t)(Fl + 2 * S + 2 * g * H + 10 * H + 8));
      double *m = buf, *x = m + Fl, *gx = x + 2 * S, *gh = gx + g * H, *h = gh + g * H, *c = h + H,
             *hm = c + H, *cm = hm + H, *h2 = cm + H, *c2 = h2 + H;
      double *hb = c2 + H, *cb = hb + H, *hb2 = cb + H, *cb2 = hb2 + H;   /* second recurrent layer */
      double *z = input_concat ? x + S : x;   /* the last structure layer's output inside x */
      const int64_t slot = row_base + (i - v_lo);
      for (int32_t j = 0; j < H; ++j) {
        h[j] = (H0 && time_kind != TIME_NONE) ? (double)H0[slot * H + j] : 0.0;
        c[j] = (H0 && time_kind == TIME_LSTM) ? (double)H0[(tot_v + slot) * H + j] : 0.0;
        hb[j] = (H0 && n_time_layers == 2) ? (double)H0[(n_state * tot_v + slot) * H + j] : 0.0;
        cb[j] = (H0 && n_time_layers == 2 && time_kind == TIME_LSTM) ? (double)H0[((n_state + 1) * tot_v + slot) * H + j] : 0.0;
      }
      for (int64_t t = t_lo; t < t_hi; ++t) {
        if (n_struct_layers == 2) {
          aggregate_row(N, rowptr[t], col[t], t, i, v_lo, v_hi, NULL, 0,
                        Z1 + (t - t_lo) * nv * (int64_t)S, C1, ldc1, S, m);
          dense_row(W1, b1, S, S, m, act_out, z);
          if (input_concat)
            for (int32_t j = 0; j < S; ++j) x[j] = Z1[((t - t_lo) * nv + (i - v_lo)) * (int64_t)S + j];
        } else {
          aggregate_row(N, rowptr[t], col[t], t, i, v_lo, v_hi, X, ldx, NULL, C, ldc, F, m);
          dense_row(W0, b0, S, F, m, act_out, z);
        }
        float *y = Y + (t * N + i) * ldy;
        if (time_kind == TIME_NONE) {
          for (int32_t j = 0; j < S; ++j) y[j] = (float)z[j];
          continue;
        }
        const double mk = (reset_mask && reset_mask[t * N + i]) ? 0.0 : 1.0;
        for (int32_t j = 0; j < H; ++j) { hm[j] = mk * h[j]; cm[j] = mk * c[j]; }
        if (time_kind == TIME_GRU) {
          gru_step(Wih, Whh, bih, bhh, Sx, H, x, hm, gx, gh, h2);
        } else {
          lstm_step(Wih, Whh, bih, bhh, Sx, H, x, hm, cm, gx, gh, h2, c2);
          for (int32_t j = 0; j < H; ++j) c[j] = c2[j];
        }
        for (int32_t j = 0; j < H; ++j) h[j] = h2[j];
        if (n_time_layers == 2) {
          /* the second recurrent layer: input = the first layer's new hidden state */
          for (int32_t j = 0; j < H; ++j) { hm[j] = mk * hb[j]; cm[j] = mk * cb[j]; }
          if (time_kind == TIME_GRU) {
            gru_step(Wih2, Whh2, bih2, bhh2, H, H, h, hm, gx, gh, hb2);
          } else {
            lstm_step(Wih2, Whh2, bih2, bhh2, H, H, h, hm, cm, gx, gh, hb2, cb2);
            for (int32_t j = 0; j < H; ++j) cb[j] = cb2[j];
          }
          for (int32_t j = 0; j < H; ++j) { hb[j] = hb2[j]; y[j] = (float)hb[j]; }
        } else {
          for (int32_t j = 0; j < H; ++j) y[j] = (float)h[j];
        }
      }
      if (hN && time_kind != TIME_NONE) {
        for (int32_t j = 0; j < H; ++j) {
          hN[slot * H + j] = (float)h[j];
          if (time_kind == TIME_LSTM) hN[(tot_v + slot) * H + j] = (float)c[j];
          if (n_time_layers == 2) {
            hN[(n_state * tot_v + slot) * H + j] = (float)hb[j];
            if (time_kind == TIME_LSTM) hN[((n_state + 1) * tot_v + slot) * H + j] = (float)cb[j];
          }
        }
      }
      free(buf);
    }
    free(Z1);
    row_base += nv;
  }
  return 0;
}

int dgc_oracle_forward(int32_t T, int64_t N, const int64_t *const *rowptr,
                       const int32_t *const *col, const int64_t *chunks, int32_t n_chunks,
                       int32_t n_struct_layers, int32_t time_kind, int32_t act_hidden,
                       int32_t act_out, int32_t F, int32_t S, int32_t H, const float *X,
                       int64_t ldx, const float *C, int64_t ldc, const float *C1, int64_t ldc1,
                       const float *W0, const float *b0, const float *W1, const float *b1,
                       const float *Wih, const float *Whh, const float *bih, const float *bhh,
                       const float *H0, const uint8_t *reset_mask, const int64_t *subset_ptr,
                       const int64_t *subset_idx, float *Y, int64_t ldy, float *hN,
                       int32_t input_concat) {
  return forward_impl(T, N, rowptr, col, chunks, n_chunks, n_struct_layers, time_kind, act_hidden, act_out, F,
                      S, H, X, ldx, C, ldc, C1, ldc1, W0, b0, W1, b1, Wih, Whh, bih, bhh, H0, reset_mask,
                      subset_ptr, subset_idx, Y, ldy, hN, input_concat, 1, NULL, NULL, NULL, NULL);
}

/* The layer with a stacked time encoder (see forward_impl): the same arguments plus the second
 * recurrent layer's parameters. */
int dgc_oracle_forward_stacked(int32_t T, int64_t N, const int64_t *const *rowptr,
                               const int32_t *const *col, const int64_t *chunks, int32_t n_chunks,
                               int32_t n_struct_layers, int32_t time_kind, int32_t act_hidden,
                               int32_t act_out, int32_t F, int32_t S, int32_t H, const float *X,
                               int64_t ldx, const float *C, int64_t ldc, const float *C1, int64_t ldc1,
                               const float *W0, const float *b0, const float *W1, const float *b1,
                               const float *Wih, const float *Whh, const float *bih, const float *bhh,
                               const float *H0, const uint8_t *reset_mask, const int64_t *subset_ptr,
                               const int64_t *subset_idx, float *Y, int64_t ldy, float *hN,
                               int32_t input_concat, const float *Wih2, const float *Whh2,
                               const float *bih2, const float *bhh2) {
  return forward_impl(T, N, rowptr, col, chunks, n_chunks, n_struct_layers, time_kind, act_hidden, act_out, F,
                      S, H, X, ldx, C, ldc, C1, ldc1, W0, b0, W1, b1, Wih, Whh, bih, bhh, H0, reset_mask,
                      subset_ptr, subset_idx, Y, ldy, hN, input_concat, 2, Wih2, Whh2, bih2, bhh2);
}

int dgc_oracle_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ================================================================ EvolveGCN-O layer
 * The paper names EvolveGCN among the DGNNs it targets (Section 1) without defining it; the
 * definition used here is the "-O" variant of the work it cites: the GCN weight matrix is
 * itself the state of a matrix GRU and evolves from snapshot to snapshot,
 *     Zg = sig(Uz W + Vz W + Bz)        Rg = sig(Ur W + Vr W + Br)
 *     Wc = tanh(Uh W + Vh (Rg * W) + Bh)   W' = (1 - Zg) * W + Zg * Wc        (* elementwise)
 * with W = W_{t-1} [F][S] (W_{-1} = W_init), U., V. [F][F], B. [F][S]; the input of the GRU is
 * the state itself.  Note the reset gate multiplies W BEFORE Vh (unlike the vertex GRU above).
 * The weights are global: W_t is evolved over all T snapshots whatever the chunk windows are.
 *     Y[t,i] = relu(M[t,i] W_t),  M = the chunked, cache-reading aggregation defined above.
 * Loss: mean squared error against targets over all covered (t, i, s).
 * Parameters are passed as one array P of 10 matrices in the order
 *   W_init, Uz, Vz, Bz, Ur, Vr, Br, Uh, Vh, Bh      (row-major, double). */
enum { EV_W = 0, EV_UZ, EV_VZ, EV_BZ, EV_UR, EV_VR, EV_BR, EV_UH, EV_VH, EV_BH, EV_NPAR };

static int64_t ev_size(int k, int32_t F, int32_t S) {
  return (k == EV_W || k == EV_BZ || k == EV_BR || k == EV_BH) ? (int64_t)F * S : (int64_t)F * F;
}

/* C[F][S] (+)= op(A)[F][F] * B[F][S];  ta: use A transposed */
static void mm_fs(const double *A, const double *B, double *C, int32_t F, int32_t S, int ta, int add) {
#pragma omp parallel for
  for (int32_t i = 0; i < F; ++i)
    for (int32_t j = 0; j < S; ++j) {
      double acc = add ? C[(int64_t)i * S + j] : 0.0;
      for (int32_t k = 0; k < F; ++k) acc += (ta ? A[(int64_t)k * F + i] : A[(int64_t)i * F + k]) * B[(int64_t)k * S + j];
      C[(int64_t)i * S + j] = acc;
    }
}
/* C[F][F] += A[F][S] * B[F][S]^T */
static void mm_abt_add(const double *A, const double *B, double *C, int32_t F, int32_t S) {
#pragma omp parallel for
  for (int32_t i = 0; i < F; ++i)
    for (int32_t j = 0; j < F; ++j) {
      double acc = C[(int64_t)i * F + j];
      for (int32_t k = 0; k < S; ++k) acc += A[(int64_t)i * S + k] * B[(int64_t)j * S + k];
      C[(int64_t)i * F + j] = acc;
    }
}

/* Evolve the weights: Wt [T][F][S]; optionally the gates Zg, Rg, Wc [T][F][S] (for backward). */
static void ev_weights(int32_t T, int32_t F, int32_t S, const double *const *P, double *Wt, double *Zg,
                       double *Rg, double *Wc) {
  const int64_t n = (int64_t)F * S;
  double *z = (double *)malloc(sizeof(double) * n), *r = (double *)malloc(sizeof(double) * n);
  double *c = (double *)malloc(sizeof(double) * n), *rw = (double *)malloc(sizeof(double) * n);
  for (int32_t t = 0; t < T; ++t) {
    const double *W = t ? Wt + (int64_t)(t - 1) * n : P[EV_W];
    mm_fs(P[EV_UZ], W, z, F, S, 0, 0); mm_fs(P[EV_VZ], W, z, F, S, 0, 1);
    mm_fs(P[EV_UR], W, r, F, S, 0, 0); mm_fs(P[EV_VR], W, r, F, S, 0, 1);
    for (int64_t e = 0; e < n; ++e) {
      z[e] = sigmoid(z[e] + P[EV_BZ][e]);
      r[e] = sigmoid(r[e] + P[EV_BR][e]);
      rw[e] = r[e] * W[e];
    }
    mm_fs(P[EV_UH], W, c, F, S, 0, 0); mm_fs(P[EV_VH], rw, c, F, S, 0, 1);
    for (int64_t e = 0; e < n; ++e) {
      c[e] = tanh(c[e] + P[EV_BH][e]);
      Wt[(int64_t)t * n + e] = (1.0 - z[e]) * W[e] + z[e] * c[e];
      if (Zg) { Zg[(int64_t)t * n + e] = z[e]; Rg[(int64_t)t * n + e] = r[e]; Wc[(int64_t)t * n + e] = c[e]; }
    }
  }
  free(z); free(r); free(c); free(rw);
}

/* Forward (Y, loss) and, if grads != NULL, the gradient of the loss w.r.t. the 10 parameter
 * matrices (grads: array of 10 double arrays, overwritten).  Wt_out (optional): [T][F][S].
 * dX (optional, [T][N][F] doubles, zero on entry): the gradient w.r.t. the input rows; a row's
 * gradient comes from the rows of its own chunk that read it as a neighbour - the cache is a
 * constant.  target may be NULL (then loss = 0 and no backward).  Returns 0 or <0. */
int dgc_oracle_evolve(int32_t T, int64_t N, const int64_t *const *rowptr, const int32_t *const *col,
                      const int64_t *chunks, int32_t n_chunks, int32_t F, int32_t S, const float *X,
                      int64_t ldx, const float *C, int64_t ldc, const double *const *P,
                      const float *target, int64_t ldt, float *Y, int64_t ldy, double *loss_out,
                      double *const *grads, double *Wt_out, double *dX) {
  const int64_t n = (int64_t)F * S;
  double *Wt = (double *)malloc(sizeof(double) * T * n);
  double *Zg = (double *)malloc(sizeof(double) * T * n), *Rg = (double *)malloc(sizeof(double) * T * n);
  double *Wc = (double *)malloc(sizeof(double) * T * n);
  double *dWd = (double *)calloc((size_t)(T * n), sizeof(double)); /* direct gradient of each W_t */
  if (!Wt || !Zg || !Rg || !Wc || !dWd) return -1;
  ev_weights(T, F, S, P, Wt, Zg, Rg, Wc);
  if (Wt_out) memcpy(Wt_out, Wt, sizeof(double) * T * n);
  int64_t count = 0;
  for (int32_t k = 0; k < n_chunks; ++k)
    count += (CH_VHI(chunks, k) - CH_VLO(chunks, k)) * (CH_THI(chunks, k) - CH_TLO(chunks, k)) * S;
  double loss = 0.0;
  for (int32_t k = 0; k < n_chunks; ++k) {
    const int64_t v_lo = CH_VLO(chunks, k), v_hi = CH_VHI(chunks, k);
    if (v_lo < 0 || v_hi > N || v_lo >= v_hi || CH_TLO(chunks, k) < 0 || CH_THI(chunks, k) > T) return -2;
    for (int64_t t = CH_TLO(chunks, k); t < CH_THI(chunks, k); ++t) {
      const double *W = Wt + t * n;
      double *dW = dWd + t * n;
      double *m = (double *)malloc(sizeof(double) * (size_t)F);
      double *dp = (double *)malloc(sizeof(double) * (size_t)S);
      double *dm = (double *)malloc(sizeof(double) * (size_t)F);
      for (int64_t i = v_lo; i < v_hi; ++i) { /* serial: the dW sum is taken in row order */
        aggregate_row(N, rowptr[t], col[t], t, i, v_lo, v_hi, X, ldx, NULL, C, ldc, F, m);
        float *y = Y + (t * N + i) * ldy;
        for (int32_t s = 0; s < S; ++s) {
          double acc = 0.0;
          for (int32_t f = 0; f < F; ++f) acc += m[f] * W[(int64_t)f * S + s];
          const double out = acc > 0.0 ? acc : 0.0;
          y[s] = (float)out;
          dp[s] = 0.0;
          if (target) {
            const double d = out - (double)target[(t * N + i) * ldt + s];
            loss += d * d;
            dp[s] = acc > 0.0 ? 2.0 * d / (double)count : 0.0;
          }
        }
        if (target && grads)
          for (int32_t f = 0; f < F; ++f)
            for (int32_t s = 0; s < S; ++s) dW[(int64_t)f * S + s] += m[f] * dp[s];
        if (target && dX) { /* dL/dm_i = W_t dp_i, handed to the in-chunk neighbours with the edge's weight */
          const int64_t *rp = rowptr[t];
          const double d_i = (double)(rp[i + 1] - rp[i]);
          for (int32_t f = 0; f < F; ++f) {
            double acc = 0.0;
            for (int32_t s = 0; s < S; ++s) acc += W[(int64_t)f * S + s] * dp[s];
            dm[f] = acc;
          }
          for (int64_t e = rp[i]; e < rp[i + 1]; ++e) {
            const int64_t j = col[t][e];
            if (j < v_lo || j >= v_hi) continue;
            const double w = 1.0 / sqrt(d_i * (double)(rp[j + 1] - rp[j]));
            for (int32_t f = 0; f < F; ++f) dX[(t * N + j) * (int64_t)F + f] += w * dm[f];
          }
        }
      }
      free(m); free(dp); free(dm);
    }
  }
  if (loss_out) *loss_out = target ? loss / (double)count : 0.0;
  if (target && grads) {
    /* back-propagation through time over the weight recurrence */
    for (int k = 0; k < EV_NPAR; ++k) memset(grads[k], 0, sizeof(double) * (size_t)ev_size(k, F, S));
    double *G = (double *)calloc((size_t)n, sizeof(double));   /* dL/dW_t, total */
    double *dWp = (double *)malloc(sizeof(double) * n), *dAz = (double *)malloc(sizeof(double) * n);
    double *dAr = (double *)malloc(sizeof(double) * n), *dAh = (double *)malloc(sizeof(double) * n);
    double *rw = (double *)malloc(sizeof(double) * n), *tmp = (double *)malloc(sizeof(double) * n);
    for (int32_t t = T - 1; t >= 0; --t) {
      const double *Wp = t ? Wt + (int64_t)(t - 1) * n : P[EV_W];
      const double *z = Zg + (int64_t)t * n, *r = Rg + (int64_t)t * n, *c = Wc + (int64_t)t * n;
      for (int64_t e = 0; e < n; ++e) {
        G[e] += dWd[(int64_t)t * n + e];
        const double dz = G[e] * (c[e] - Wp[e]), dc = G[e] * z[e];
        dWp[e] = G[e] * (1.0 - z[e]);
        dAh[e] = dc * (1.0 - c[e] * c[e]);
        dAz[e] = dz * z[e] * (1.0 - z[e]);
        rw[e] = r[e] * Wp[e];
      }
      mm_abt_add(dAh, Wp, grads[EV_UH], F, S);
      mm_abt_add(dAh, rw, grads[EV_VH], F, S);
      mm_fs(P[EV_VH], dAh, tmp, F, S, 1, 0); /* d(Rg * W) = Vh^T dAh */
      for (int64_t e = 0; e < n; ++e) {
        grads[EV_BH][e] += dAh[e];
        dAr[e] = tmp[e] * Wp[e] * r[e] * (1.0 - r[e]);
        dWp[e] += tmp[e] * r[e];
      }
      mm_fs(P[EV_UH], dAh, dWp, F, S, 1, 1);
      mm_abt_add(dAz, Wp, grads[EV_UZ], F, S); mm_abt_add(dAz, Wp, grads[EV_VZ], F, S);
      mm_abt_add(dAr, Wp, grads[EV_UR], F, S); mm_abt_add(dAr, Wp, grads[EV_VR], F, S);
      for (int64_t e = 0; e < n; ++e) { grads[EV_BZ][e] += dAz[e]; grads[EV_BR][e] += dAr[e]; }
      mm_fs(P[EV_UZ], dAz, dWp, F, S, 1, 1); mm_fs(P[EV_VZ], dAz, dWp, F, S, 1, 1);
      mm_fs(P[EV_UR], dAr, dWp, F, S, 1, 1); mm_fs(P[EV_VR], dAr, dWp, F, S, 1, 1);
      for (int64_t e = 0; e < n; ++e) G[e] = dWp[e];
    }
    for (int64_t e = 0; e < n; ++e) grads[EV_W][e] = G[e];
    free(G); free(dWp); free(dAz); free(dAr); free(dAh); free(rw); free(tmp);
  }
  free(Wt); free(Zg); free(Rg); free(Wc); free(dWd);
  return 0;
}
