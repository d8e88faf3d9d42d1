// Temporal fusion (Section 5.1.2 of the paper): the sequences of the vertices of a chunk (the
// snapshots of the window in which a vertex is present) are concatenated into lanes as long as
// the window instead of being padded, and a reset flag on the first slot of every sequence keeps
// the state of one sequence out of the next (the paper's mask).  The lanes of a chunk form a
// "virtual chunk" (lanes x window) that the dense + recurrent kernels walk like any chunk: the
// aggregation writes its rows directly in lane order (and skips the rows of absent vertices), the
// recurrent kernel takes and leaves states per sequence and stores every slot's output straight to
// its (snapshot, vertex) row.
//
// Device side here: sequence lengths, the slot tables and the row map, idle vertices' states.  The packing
// rule itself (first-fit decreasing, see tf_assign_lanes in dgc_api.hip) is host arithmetic on
// the lengths.
#include "dgc_internal.h"

namespace dgc {
namespace {

unsigned nblocks(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// seq_len[state row of (chunk k, vertex)] = number of snapshots of the window with the vertex present
__global__ void k_tf_lengths(const uint8_t* present, const ChunkInfo* chunks, int64_t N, int32_t* seq_len) {
  const ChunkInfo c = chunks[blockIdx.y];
  const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= c.nv) return;
  int32_t n = 0;
  for (int32_t s = 0; s < c.w; ++s) n += present[(int64_t)(c.t_lo + s) * N + c.v_lo + v] != 0;
  seq_len[c.state_off + v] = n;
}

// slot tables from the lane / first slot assigned to every sequence
__global__ void k_tf_fill(const uint8_t* present, const ChunkInfo* chunks, int64_t N, const int32_t* seq_lane,
                          const int32_t* seq_off, int64_t n_lanes, const ChunkInfo* chunks_v, int64_t* slot_row,
                          int64_t* row_map, uint8_t* slot_reset, int64_t* seq_in, int64_t* seq_out) {
  const ChunkInfo c = chunks[blockIdx.y];
  const ChunkInfo cv = chunks_v[blockIdx.y];
  const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= c.nv) return;
  const int32_t lane = seq_lane[c.state_off + v];
  if (lane < 0) return;
  int32_t slot = seq_off[c.state_off + v];
  slot_reset[(int64_t)slot * n_lanes + lane] = 1;
  seq_in[(int64_t)slot * n_lanes + lane] = c.state_off + v;     // the sequence's state row enters here
  for (int32_t s = 0; s < c.w; ++s) {
    const int64_t t = c.t_lo + s;
    if (!present[t * N + c.v_lo + v]) continue;
    slot_row[(int64_t)slot * n_lanes + lane] = t * N + c.v_lo + v;
    row_map[c.row_off0 + (int64_t)s * c.nv + v] = cv.row_off0 + (int64_t)slot * cv.nv + (lane - cv.v_lo);
    ++slot;
  }
  seq_out[(int64_t)(slot - 1) * n_lanes + lane] = c.state_off + v;   // ... and leaves after its last slot
}

// HN row = H0 row (or zero) for every (chunk, vertex) that is absent throughout its window; one
// thread per float4, n_state blocks of V rows (hidden, then cell for the LSTM)
__global__ void k_tf_carry(const int32_t* seq_len, int64_t V, int32_t n_state, int32_t H, const float* H0, float* HN) {
  const int64_t q = H / 4;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)n_state * V * q) return;
  const int64_t row = idx / q, c4 = idx - row * q;
  if (seq_len[row % V] != 0) return;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (H0) v = reinterpret_cast<const float4*>(H0 + row * H)[c4];
  reinterpret_cast<float4*>(HN + row * H)[c4] = v;
}

__global__ void k_tf_fill_i64(int64_t* p, int64_t v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Temporal fusion over generated chunks (Sections 5.1.2 and 4.1 together): a vertex's sequences
// are its maximal runs of present instances that carry one label (the label of an absent instance
// plays no part).  One thread per vertex walks its snapshots and writes, per instance x = t*N + i:
// the snapshot its sequence starts in (-1: absent), its position in the sequence, whether it is the
// sequence's last instance, and, at a sequence's first instance, the sequence's length (else 0).
__global__ void k_lp_sequences(const uint8_t* present, const int32_t* labels, int32_t T, int64_t N, int32_t* seq_len,
                               int32_t* first_t, int32_t* pos, uint8_t* last) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  int32_t start = -1, n = 0, prev_label = 0;
  int64_t prev = -1;
  for (int32_t t = 0; t < T; ++t) {
    const int64_t x = (int64_t)t * N + i;
    seq_len[x] = 0; first_t[x] = -1; pos[x] = 0; last[x] = 0;
    if (!present[x]) continue;
    const int32_t lab = labels[x];
    if (start < 0 || lab != prev_label) {
      if (start >= 0) { seq_len[(int64_t)start * N + i] = n; last[prev] = 1; }
      start = t; n = 0;
    }
    first_t[x] = start; pos[x] = n; ++n;
    prev = x; prev_label = lab;
  }
  if (start >= 0) { seq_len[(int64_t)start * N + i] = n; last[prev] = 1; }
}

// slot tables from the lane / first slot assigned to every sequence (indexed by the sequence's
// first instance); one thread per instance.  The layer's single chunk is [0,N) x [0,T), so the
// packed row of instance x is x itself.
__global__ void k_lp_fill(const uint8_t* present, const int32_t* first_t, const int32_t* pos, const uint8_t* last,
                          const int32_t* seq_lane, const int32_t* seq_off, int64_t TN, int64_t N, int64_t n_lanes,
                          int64_t* slot_row, int64_t* row_map, uint8_t* slot_reset, int64_t* seq_in, int64_t* seq_out) {
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= TN || !present[x]) return;
  const int64_t start = (int64_t)first_t[x] * N + x % N;
  const int64_t slot = (int64_t)(seq_off[start] + pos[x]) * n_lanes + seq_lane[start];
  slot_row[slot] = x;
  row_map[x] = slot;
  if (pos[x] == 0) { slot_reset[slot] = 1; seq_in[slot] = x; }      // the state enters from the cache row of (t, i)
  if (last[x]) seq_out[slot] = x;                                    // ... and leaves to the row of the last instance
}

}  // namespace

void lp_sequences(const uint8_t* present, const int32_t* labels, int32_t T, int64_t N, int32_t* seq_len, int32_t* first_t,
                  int32_t* pos, uint8_t* last, hipStream_t st) {
  hipLaunchKernelGGL(k_lp_sequences, nblocks(N, 256), 256, 0, st, present, labels, T, N, seq_len, first_t, pos, last);
}

void lp_fill(const uint8_t* present, const int32_t* first_t, const int32_t* pos, const uint8_t* last,
             const int32_t* seq_lane, const int32_t* seq_off, int32_t T, int64_t N, int64_t n_lanes, int64_t* slot_row,
             int64_t* row_map, uint8_t* slot_reset, int64_t* seq_in, int64_t* seq_out, hipStream_t st) {
  const int64_t n = (int64_t)T * n_lanes, TN = (int64_t)T * N;
  if (n > 0) {
    hipLaunchKernelGGL(k_tf_fill_i64, nblocks(n, 256), 256, 0, st, slot_row, (int64_t)-1, n);
    hipLaunchKernelGGL(k_tf_fill_i64, nblocks(n, 256), 256, 0, st, seq_in, (int64_t)-1, n);
    hipLaunchKernelGGL(k_tf_fill_i64, nblocks(n, 256), 256, 0, st, seq_out, (int64_t)-1, n);
    (void)hipMemsetAsync(slot_reset, 0, (size_t)n, st);
  }
  hipLaunchKernelGGL(k_tf_fill_i64, nblocks(TN, 256), 256, 0, st, row_map, (int64_t)-1, TN);
  if (n > 0)
    hipLaunchKernelGGL(k_lp_fill, nblocks(TN, 256), 256, 0, st, present, first_t, pos, last, seq_lane, seq_off, TN, N,
                       n_lanes, slot_row, row_map, slot_reset, seq_in, seq_out);
}

void tf_lengths(const uint8_t* present, const ChunkInfo* chunks, int32_t n_chunks, int64_t max_nv, int64_t N,
                int32_t* seq_len, hipStream_t st) {
  hipLaunchKernelGGL(k_tf_lengths, dim3(nblocks(max_nv, 256), n_chunks), 256, 0, st, present, chunks, N, seq_len);
}

void tf_fill(const uint8_t* present, const ChunkInfo* chunks, int32_t n_chunks, int64_t max_nv, int64_t N,
             const int32_t* seq_lane, const int32_t* seq_off, int64_t n_lanes, int32_t Lmax, const ChunkInfo* chunks_v,
             int64_t total_rows, int64_t* slot_row, int64_t* row_map, uint8_t* slot_reset, int64_t* seq_in,
             int64_t* seq_out, hipStream_t st) {
  const int64_t n = (int64_t)Lmax * n_lanes;
  if (n > 0) {   // no lanes: nobody present
    hipLaunchKernelGGL(k_tf_fill_i64, nblocks(n, 256), 256, 0, st, slot_row, (int64_t)-1, n);
    hipLaunchKernelGGL(k_tf_fill_i64, nblocks(n, 256), 256, 0, st, seq_in, (int64_t)-1, n);
    hipLaunchKernelGGL(k_tf_fill_i64, nblocks(n, 256), 256, 0, st, seq_out, (int64_t)-1, n);
  }
  hipLaunchKernelGGL(k_tf_fill_i64, nblocks(total_rows, 256), 256, 0, st, row_map, (int64_t)-1, total_rows);
  if (n > 0) (void)hipMemsetAsync(slot_reset, 0, (size_t)n, st);
  hipLaunchKernelGGL(k_tf_fill, dim3(nblocks(max_nv, 256), n_chunks), 256, 0, st, present, chunks, N, seq_lane, seq_off,
                     n_lanes, chunks_v, slot_row, row_map, slot_reset, seq_in, seq_out);
}

void tf_carry(const int32_t* seq_len, int64_t V, int32_t n_state, int32_t H, const float* H0, float* HN, hipStream_t st) {
  const int64_t n = (int64_t)n_state * V * (H / 4);
  if (n > 0) hipLaunchKernelGGL(k_tf_carry, nblocks(n, 256), 256, 0, st, seq_len, V, n_state, H, H0, HN);
}

}  // namespace dgc
