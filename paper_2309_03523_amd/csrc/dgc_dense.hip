// Dense part of the layer on the fp32 matrix cores: the GCN feature transform
// Z = act(M W^T + b) and the time encoder (GRU / LSTM, the units Section 6 names) with the
// temporal-fusion mask of Section 5.1.2 on the incoming state.
//
// The recurrence is per vertex, so a workgroup that owns 64 vertices of one chunk can walk the
// chunk's whole window by itself: per step it loads the 64 aggregated rows, transforms them,
// multiplies [Z | h] with the gate weights and applies the gate arithmetic in registers.  Z, the
// gate pre-activations and h never travel through HBM; h lives in LDS between steps.  All
// chunks of the fused batch are tiles of the same launch.
//
// MFMA: v_mfma_f32_32x32x2f32 computes D = A x B with lane l supplying A[l%32][l/32] and
// B[l/32][l%32] and receiving D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v.
// The WEIGHTS are the A operand and the activations (M, Z, h) the B operand, so a lane ends up
// with one activation row (l%32) and four consecutive output columns per register quad: Z and h
// go back to the row-major LDS tile as float4.  Activations are read from LDS as float4 (four
// consecutive k per lane); weights come straight from global memory / L2 in a pre-packed
// fragment order, one contiguous 1 KiB per wave and load, with no LDS staging and no barrier.
#include "dgc_internal.h"

namespace dgc {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kMaxPrefetch = 8;  // float4 per thread of the next step's aggregated rows

__global__ void k_pack_weight(const float* W, int32_t n_out, int32_t n_in, float4* packed) {
  const int nkb = (n_in + 7) / 8;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)(n_out / 32) * nkb * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const int64_t f = idx >> 6;
  const int kb = (int)(f % nkb);
  const int jb = (int)(f / nkb);
  const int row = jb * 32 + (lane & 31);
  const int k0 = kb * 8 + (lane >> 5) * 4;
  float v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = (k0 + q < n_in) ? W[(int64_t)row * n_in + k0 + q] : 0.f;
  packed[idx] = make_float4(v[0], v[1], v[2], v[3]);
}

// Gate non-linearities on the hardware exp2 / reciprocal units (about 1 ulp each): the
// absolute error is ~1e-7, far inside the fp32 tolerance of the layer.
__device__ __forceinline__ float sigmoid_fast(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ __forceinline__ float tanh_fast(float x) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x)); }

__device__ __forceinline__ float f4get(const float4& v, int q) {
  return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w;
}

// Visit every (row, float4 column) of a [64][wf4] tile once (wf4 <= 64), a whole row per half
// wave or wave so that global accesses are contiguous; no integer division.
template <class F>
__device__ __forceinline__ void for_tile_f4(int tid, int wf4, F&& body) {
  const int lane = tid & 63, wave = tid >> 6;
  if (wf4 <= 32) {
    const int c4 = lane & 31;
    if (c4 < wf4)
      for (int r = wave * 2 + (lane >> 5); r < kTileRows; r += 2 * kWaves) body(r, c4);
  } else {
    for (int r = wave; r < kTileRows; r += kWaves)
      for (int c4 = lane; c4 < wf4; c4 += kWave) body(r, c4);
  }
}

// Waves that are not issuing matrix instructions run at raised priority: their short VALU /
// LDS / memory phases then are not starved by the other workgroup's MFMA stream on the same
// SIMD, and they return to matrix work sooner.
__device__ __forceinline__ void prio_matrix() { __builtin_amdgcn_s_setprio(0); }
__device__ __forceinline__ void prio_other() { __builtin_amdgcn_s_setprio(2); }

// One block of 8 k: acc[rb][slot g] += W_g (A operand) x activations (B operand).
template <int NRB, int NG, int S0, int S1, int S2, int S3>
__device__ __forceinline__ void mma_block(floatx16 (&acc)[NRB][4], const float4 (&w)[NG], const float4 (&x)[NRB]) {
  constexpr int slot[4] = {S0, S1, S2, S3};
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
        acc[rb][slot[g]] =
            __builtin_amdgcn_mfma_f32_32x32x2f32(f4get(w[g], q), f4get(x[rb], q), acc[rb][slot[g]], 0, 0, 0);
}

// acc[rb][slot g] += X[rows of block rb][k] * W_g[cols][k], k over nkb blocks of 8.
//  ldsX : LDS address of X[row l%32 of block 0][(l/32)*4]; block rb adds rb*32*ld
//  wp[g]: packed weight fragments of gate g for this column block, already offset by lane;
//         fragment kb is wp[g][kb*64]
// Two register sets alternate so that the weight loads (L2 latency) of block kb+1 are in flight
// while the 8*NG*NRB MFMAs of block kb issue.
template <int NRB, int NG, int S0, int S1, int S2, int S3>
__device__ __forceinline__ void mma_k_loop(floatx16 (&acc)[NRB][4], const float* ldsX, int ld, int nkb,
                                           const float4* const (&wp)[NG]) {
  float4 w0[NG], w1[NG], x0[NRB], x1[NRB];
#pragma unroll
  for (int g = 0; g < NG; ++g) w0[g] = wp[g][0];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) x0[rb] = *reinterpret_cast<const float4*>(ldsX + rb * 32 * ld);
  int kb = 0;
  for (; kb + 1 < nkb; kb += 2) {
#pragma unroll
    for (int g = 0; g < NG; ++g) w1[g] = wp[g][(int64_t)(kb + 1) * 64];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) x1[rb] = *reinterpret_cast<const float4*>(ldsX + rb * 32 * ld + (kb + 1) * 8);
    __builtin_amdgcn_sched_barrier(0);
    mma_block<NRB, NG, S0, S1, S2, S3>(acc, w0, x0);
    __builtin_amdgcn_sched_barrier(0);
    const int kn = kb + 2 < nkb ? kb + 2 : nkb - 1;
#pragma unroll
    for (int g = 0; g < NG; ++g) w0[g] = wp[g][(int64_t)kn * 64];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) x0[rb] = *reinterpret_cast<const float4*>(ldsX + rb * 32 * ld + kn * 8);
    __builtin_amdgcn_sched_barrier(0);
    mma_block<NRB, NG, S0, S1, S2, S3>(acc, w1, x1);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (kb < nkb) mma_block<NRB, NG, S0, S1, S2, S3>(acc, w0, x0);
}

// KIND: DGC_TIME_*.  NRB: 32-row blocks per unit (1 or 2).  UPW: units per wave.
// A unit is NRB row blocks x one 32-column block (x all gates).
//
// LDS holds two [64][ld] buffers that swap roles every step:
//   P: the state h entering the step;   Q: the aggregated rows, then Z, then the new state.
// Per step: mask P | Z = act(Q W^T + b) in registers | Z -> Q | gate GEMMs read Q and P | the
// next step's aggregated rows start loading into registers | gate arithmetic | new h -> Q and
// the prefetched rows -> P | Q -> Y | swap(P, Q).
// SEQ: the rows of a tile hold several sequences one after the other (temporal fusion with
// states): states enter and leave through the tables seq_in / seq_out instead of at the window's
// ends; mask_row then holds 1 + the state row of a sequence that starts at this step, end_row
// 1 + the state row of a sequence that ends at it (0 = none).
template <int KIND, int NRB, int UPW, bool SEQ>
// (the two-units-per-wave variants, S or H above 128, hold a tile of up to 133 KB in LDS: one
//  workgroup per CU either way, so they may use the whole register file)
__global__ __launch_bounds__(kThreads, (UPW >= 2 ? 1 : 2)) void k_dense(DenseArgs a, int ld) {
  extern __shared__ float smem[];
  float* P = smem;
  float* Q = smem + kTileRows * ld;
  int* mask_row = reinterpret_cast<int*>(smem + 2 * kTileRows * ld);   // [64]
  int* end_rows = mask_row + kTileRows;                                // [2][64], by step parity: the output
                                                                       // store of a step still reads its table
                                                                       // when the next step's is written
  float* gate_bias = smem + 2 * kTileRows * ld + 3 * kTileRows;        // [4][H]

  prio_other();
  const DenseTile tile = a.tiles[blockIdx.x];
  const ChunkInfo ch = a.chunks[tile.chunk];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int nrows = tile.nrows;
  const int K0 = a.K0, S = a.S, H = a.H;
  const int nkb0 = (K0 + 7) / 8, nkbS = S / 8, nkbH = H / 8;
  const int njbS = S / 32, njbH = H / 32;
  constexpr int RBU = 2 / NRB;  // units per column block
  const int unitsS = njbS * RBU, unitsH = njbH * RBU;
  const int64_t V = a.total_state_rows;
  const int64_t vbase = ch.v_lo + tile.v0;            // first vertex of the tile
  const int64_t sbase = ch.state_off + tile.v0;       // first state row of the tile
  const int nf4 = nkb0 * 2;                           // float4 per aggregated row in LDS
  // The next step's rows are prefetched through registers when a row is a power-of-two number
  // of float4 (K0 = 8..128): thread -> (row r0 + i*rpp, float4 column c4), no column masking.
  const bool prefetch = KIND != DGC_TIME_NONE && K0 % 8 == 0 && (nf4 & (nf4 - 1)) == 0 && nf4 <= 32;
  const int pf_c4 = tid & (nf4 - 1), pf_r0 = tid / nf4, pf_rpp = kThreads / nf4;

  auto load_rows = [&](int s, float4 (&r)[kMaxPrefetch]) {
    const float* src = a.M + (ch.row_off0 + (int64_t)s * ch.nv + tile.v0 + pf_r0) * a.ldm + 4 * pf_c4;
#pragma unroll
    for (int i = 0; i < kMaxPrefetch; ++i) {
      const int row = pf_r0 + i * pf_rpp;
      r[i] = row < nrows ? *reinterpret_cast<const float4*>(src + (int64_t)i * pf_rpp * a.ldm)
                         : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto store_rows = [&](float* buf, const float4 (&r)[kMaxPrefetch]) {
#pragma unroll
    for (int i = 0; i < kMaxPrefetch; ++i) {
      const int row = pf_r0 + i * pf_rpp;
      if (row < kTileRows) *reinterpret_cast<float4*>(buf + row * ld + 4 * pf_c4) = r[i];
    }
  };
  // the same, any width, straight to LDS
  auto load_rows_direct = [&](int s, float* buf) {
    const float* Mrow0 = a.M + (ch.row_off0 + (int64_t)s * ch.nv + tile.v0) * a.ldm;
    for (int row = wave; row < kTileRows; row += kWaves) for (int c4 = lane; c4 < nf4; c4 += kWave) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row < nrows && 4 * c4 < a.ldm) {
        v = *reinterpret_cast<const float4*>(Mrow0 + (int64_t)row * a.ldm + 4 * c4);
        if (4 * c4 + 1 >= K0) v.y = 0.f;
        if (4 * c4 + 2 >= K0) v.z = 0.f;
        if (4 * c4 + 3 >= K0) v.w = 0.f;
        if (4 * c4 >= K0) v.x = 0.f;
      }
      *reinterpret_cast<float4*>(buf + row * ld + 4 * c4) = v;
    }
  };

  // LSTM cell state stays in registers, in accumulator layout, for the whole window
  float cst[UPW][NRB][16];
  if constexpr (KIND == DGC_TIME_LSTM) {
#pragma unroll
    for (int ui = 0; ui < UPW; ++ui) {
      const int u = wave + kWaves * ui;
      const int jb = u / RBU, rb0 = (u % RBU) * NRB;
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = (rb0 + rb) * 32 + l32;
          const int col = jb * 32 + 8 * (v / 4) + 4 * half + (v % 4);
          cst[ui][rb][v] = (!SEQ && a.H0 && u < unitsH && row < nrows) ? a.H0[(V + sbase + row) * H + col] : 0.f;
        }
    }
  }
  if constexpr (KIND != DGC_TIME_NONE) {
    for_tile_f4(tid, H / 4, [&](int r, int c4) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (!SEQ && a.H0 && r < nrows) v = *reinterpret_cast<const float4*>(a.H0 + (sbase + r) * H + 4 * c4);
      *reinterpret_cast<float4*>(P + r * ld + 4 * c4) = v;
    });
    // gate biases, pre-summed where the gate adds both: GRU rows r, z, n(input), n(hidden);
    // LSTM rows i, f, g, o
    for (int idx = tid; idx < 4 * H; idx += kThreads) {
      const int g = idx / H, c = idx - g * H;
      float b;
      if (KIND == DGC_TIME_GRU) {
        b = g < 2 ? a.bih[g * H + c] + a.bhh[g * H + c] : (g == 2 ? a.bih[2 * H + c] : a.bhh[2 * H + c]);
      } else {
        b = a.bih[g * H + c] + a.bhh[g * H + c];
      }
      gate_bias[idx] = b;
    }
  }
  load_rows_direct(0, Q);

  for (int s = 0; s < ch.w; ++s) {
    const int64_t t = ch.t_lo + s;
    int* end_row = end_rows + (s & 1) * kTileRows;
    if (s > 0 && !prefetch) load_rows_direct(s, Q);
    // temporal-fusion mask: zero the incoming state of masked rows (same thread <-> element
    // mapping as the Y store at the end of the previous step, so no barrier in between)
    if constexpr (KIND != DGC_TIME_NONE && !SEQ) {
      if (a.reset_mask) {
        for_tile_f4(tid, H / 4, [&](int r, int c4) {
          const int mk = r < nrows ? a.reset_mask[t * a.N + vbase + r] : 0;
          if (mk) *reinterpret_cast<float4*>(P + r * ld + 4 * c4) = make_float4(0.f, 0.f, 0.f, 0.f);
          if (c4 == 0) mask_row[r] = mk;
        });
      } else if (s == 0 && tid < kTileRows) {
        mask_row[tid] = 0;
      }
    }
    if constexpr (KIND != DGC_TIME_NONE && SEQ) {
      for_tile_f4(tid, H / 4, [&](int r, int c4) {
        const int64_t sr = r < nrows ? a.seq_in[t * a.N + vbase + r] : -1;
        if (sr >= 0) {   // a sequence starts here: its own state row, or zero
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (a.H0) v = *reinterpret_cast<const float4*>(a.H0 + sr * H + 4 * c4);
          *reinterpret_cast<float4*>(P + r * ld + 4 * c4) = v;
        }
        if (c4 == 0) {
          mask_row[r] = (int)(sr + 1);
          end_row[r] = r < nrows ? (int)(a.seq_out[t * a.N + vbase + r] + 1) : 0;
        }
      });
    }
    __syncthreads();

    // Z = act(M W^T + b) for this wave's units, kept in the accumulators over the barrier
    floatx16 zacc[UPW][NRB];
#pragma unroll
    for (int ui = 0; ui < UPW; ++ui) {
      const int u = wave + kWaves * ui;
      if (u < unitsS) {
        const int jb = u / RBU, rb0 = (u % RBU) * NRB;
        floatx16 acc[NRB][4];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) acc[rb][0] = (floatx16)(0.f);
        const float4* const wp[1] = {a.Wg + (t * a.wg_step_bytes) / 16 + ((int64_t)jb * nkb0) * 64 + lane};
        prio_matrix();
        mma_k_loop<NRB, 1, 0, 0, 0, 0>(acc, Q + (rb0 * 32 + l32) * ld + half * 4, ld, nkb0, wp);
        prio_other();
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) zacc[ui][rb] = acc[rb][0];
      }
    }
    __syncthreads();  // everyone has finished reading the aggregated rows
#pragma unroll
    for (int ui = 0; ui < UPW; ++ui) {
      const int u = wave + kWaves * ui;
      if (u < unitsS) {
        const int jb = u / RBU, rb0 = (u % RBU) * NRB;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int c0 = jb * 32 + 8 * g4 + 4 * half;
          const float4 bias = *reinterpret_cast<const float4*>(a.bg + c0);
#pragma unroll
          for (int rb = 0; rb < NRB; ++rb) {
            float4 z = make_float4(zacc[ui][rb][4 * g4 + 0] + bias.x, zacc[ui][rb][4 * g4 + 1] + bias.y,
                                   zacc[ui][rb][4 * g4 + 2] + bias.z, zacc[ui][rb][4 * g4 + 3] + bias.w);
            if (a.act == DGC_ACT_RELU) {
              z.x = fmaxf(z.x, 0.f); z.y = fmaxf(z.y, 0.f); z.z = fmaxf(z.z, 0.f); z.w = fmaxf(z.w, 0.f);
            }
            *reinterpret_cast<float4*>(Q + ((rb0 + rb) * 32 + l32) * ld + c0) = z;
          }
        }
      }
    }
    __syncthreads();

    if constexpr (KIND == DGC_TIME_NONE) {
      for_tile_f4(tid, S / 4, [&](int r, int c4) {
        if (r < nrows)
          *reinterpret_cast<float4*>(a.Y + (t * a.N + vbase + r) * a.ldy + 4 * c4) =
              *reinterpret_cast<const float4*>(Q + r * ld + 4 * c4);
      });
      __syncthreads();  // Q is overwritten by the next step's rows
    } else {
      // Gate pre-activations and gate arithmetic, four consecutive columns at a time.  The new
      // state can only be written once every wave has stopped reading Z and h, so it waits in
      // registers over the barrier.
      float4 hnew[UPW][NRB][4];
      float4 mnext[kMaxPrefetch];
#pragma unroll
      for (int ui = 0; ui < UPW; ++ui) {
        const int u = wave + kWaves * ui;
        floatx16 acc[NRB][4];
        const int jb = u / RBU, rb0 = (u % RBU) * NRB;
        if (u < unitsH) {
#pragma unroll
          for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int g = 0; g < 4; ++g) acc[rb][g] = (floatx16)(0.f);
          const float* ldsZ = Q + (rb0 * 32 + l32) * ld + half * 4;
          const float* ldsHp = P + (rb0 * 32 + l32) * ld + half * 4;
          if constexpr (KIND == DGC_TIME_GRU) {
            // slots: 0 r, 1 z, 2 input part of n, 3 hidden part of n
            const float4* const wi[3] = {a.Wih + ((int64_t)(0 * njbH + jb) * nkbS) * 64 + lane,
                                         a.Wih + ((int64_t)(1 * njbH + jb) * nkbS) * 64 + lane,
                                         a.Wih + ((int64_t)(2 * njbH + jb) * nkbS) * 64 + lane};
            const float4* const wh[3] = {a.Whh + ((int64_t)(0 * njbH + jb) * nkbH) * 64 + lane,
                                         a.Whh + ((int64_t)(1 * njbH + jb) * nkbH) * 64 + lane,
                                         a.Whh + ((int64_t)(2 * njbH + jb) * nkbH) * 64 + lane};
            prio_matrix();
            mma_k_loop<NRB, 3, 0, 1, 2, 0>(acc, ldsZ, ld, nkbS, wi);
            mma_k_loop<NRB, 3, 0, 1, 3, 0>(acc, ldsHp, ld, nkbH, wh);
            prio_other();
          } else {
            // slots: 0 i, 1 f, 2 g, 3 o
            const float4* const wi[4] = {a.Wih + ((int64_t)(0 * njbH + jb) * nkbS) * 64 + lane,
                                         a.Wih + ((int64_t)(1 * njbH + jb) * nkbS) * 64 + lane,
                                         a.Wih + ((int64_t)(2 * njbH + jb) * nkbS) * 64 + lane,
                                         a.Wih + ((int64_t)(3 * njbH + jb) * nkbS) * 64 + lane};
            const float4* const wh[4] = {a.Whh + ((int64_t)(0 * njbH + jb) * nkbH) * 64 + lane,
                                         a.Whh + ((int64_t)(1 * njbH + jb) * nkbH) * 64 + lane,
                                         a.Whh + ((int64_t)(2 * njbH + jb) * nkbH) * 64 + lane,
                                         a.Whh + ((int64_t)(3 * njbH + jb) * nkbH) * 64 + lane};
            prio_matrix();
            mma_k_loop<NRB, 4, 0, 1, 2, 3>(acc, ldsZ, ld, nkbS, wi);
            mma_k_loop<NRB, 4, 0, 1, 2, 3>(acc, ldsHp, ld, nkbH, wh);
            prio_other();
          }
        }
        if (u < unitsH) {
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            const int c0 = jb * 32 + 8 * g4 + 4 * half;
            float bs[4][4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const float4 b = *reinterpret_cast<const float4*>(gate_bias + g * H + c0);
              bs[g][0] = b.x; bs[g][1] = b.y; bs[g][2] = b.z; bs[g][3] = b.w;
            }
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
              float o[4];
              if constexpr (KIND == DGC_TIME_GRU) {
                const float4 hp4 = *reinterpret_cast<const float4*>(P + ((rb0 + rb) * 32 + l32) * ld + c0);
                const float hp[4] = {hp4.x, hp4.y, hp4.z, hp4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const int v = 4 * g4 + e;
                  const float r = sigmoid_fast(acc[rb][0][v] + bs[0][e]);
                  const float z = sigmoid_fast(acc[rb][1][v] + bs[1][e]);
                  const float n = tanh_fast(acc[rb][2][v] + bs[2][e] + r * (acc[rb][3][v] + bs[3][e]));
                  o[e] = (1.0f - z) * n + z * hp[e];
                }
              } else {
                const int mrow = mask_row[(rb0 + rb) * 32 + l32];
                const bool masked = mrow != 0;
                float cin[4] = {0.f, 0.f, 0.f, 0.f};
                if (SEQ && masked && a.H0) {   // the cell row of the sequence that starts here
                  const float4 c4v = *reinterpret_cast<const float4*>(a.H0 + (V + mrow - 1) * H + c0);
                  cin[0] = c4v.x; cin[1] = c4v.y; cin[2] = c4v.z; cin[3] = c4v.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const int v = 4 * g4 + e;
                  const float cm = masked ? cin[e] : cst[ui][rb][v];
                  const float ig = sigmoid_fast(acc[rb][0][v] + bs[0][e]);
                  const float fg = sigmoid_fast(acc[rb][1][v] + bs[1][e]);
                  const float gg = tanh_fast(acc[rb][2][v] + bs[2][e]);
                  const float og = sigmoid_fast(acc[rb][3][v] + bs[3][e]);
                  const float cn = fg * cm + ig * gg;
                  cst[ui][rb][v] = cn;
                  o[e] = og * tanh_fast(cn);
                }
                if constexpr (SEQ) {           // the cell state of a sequence that ends at this step
                  const int erow = end_row[(rb0 + rb) * 32 + l32];
                  if (erow != 0 && a.HN)
                    *reinterpret_cast<float4*>(a.HN + (V + erow - 1) * H + c0) =
                        make_float4(cst[ui][rb][4 * g4], cst[ui][rb][4 * g4 + 1], cst[ui][rb][4 * g4 + 2],
                                    cst[ui][rb][4 * g4 + 3]);
                }
              }
              hnew[ui][rb][g4] = make_float4(o[0], o[1], o[2], o[3]);
            }
          }
        }
      }
      // the accumulators are free: start fetching the next step's rows, so that their HBM latency
      // hides behind the barriers and the Y store
      if (prefetch && s + 1 < ch.w) load_rows(s + 1, mnext);
      __syncthreads();  // everyone has finished reading Z and the old state
#pragma unroll
      for (int ui = 0; ui < UPW; ++ui) {
        const int u = wave + kWaves * ui;
        if (u < unitsH) {
          const int jb = u / RBU, rb0 = (u % RBU) * NRB;
#pragma unroll
          for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
              *reinterpret_cast<float4*>(Q + ((rb0 + rb) * 32 + l32) * ld + jb * 32 + 8 * g4 + 4 * half) =
                  hnew[ui][rb][g4];
        }
      }
      __syncthreads();
      // h_t -> Y, whole rows at a time; Q becomes the state buffer of the next step
      const bool last = !SEQ && (s == ch.w - 1) && a.HN;
      for_tile_f4(tid, H / 4, [&](int r, int c4) {
        if (r < nrows) {
          const float4 v = *reinterpret_cast<const float4*>(Q + r * ld + 4 * c4);
          int64_t yr = t * a.N + vbase + r;
          if constexpr (SEQ) {
            if (a.y_map) yr = a.y_map[yr];     // temporal fusion: the slot's own row of Y, or nowhere
          }
          if (yr >= 0) *reinterpret_cast<float4*>(a.Y + yr * a.ldy + 4 * c4) = v;
          if (last) *reinterpret_cast<float4*>(a.HN + (sbase + r) * H + 4 * c4) = v;
          if constexpr (SEQ) {
            const int erow = end_row[r];
            if (erow != 0 && a.HN) *reinterpret_cast<float4*>(a.HN + (int64_t)(erow - 1) * H + 4 * c4) = v;
          }
        }
      });
      // P (the old state, no longer read) becomes the next step's Q
      if (prefetch && s + 1 < ch.w) store_rows(P, mnext);
      float* tmp = P; P = Q; Q = tmp;
    }
  }

  if constexpr (KIND == DGC_TIME_LSTM && !SEQ) {
    if (a.HN) {
#pragma unroll
      for (int ui = 0; ui < UPW; ++ui) {
        const int u = wave + kWaves * ui;
        if (u < unitsH) {
          const int jb = u / RBU, rb0 = (u % RBU) * NRB;
#pragma unroll
          for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int row = (rb0 + rb) * 32 + l32;
              const int col = jb * 32 + 8 * (v / 4) + 4 * half + (v % 4);
              if (row < nrows) a.HN[(V + sbase + row) * H + col] = cst[ui][rb][v];
            }
        }
      }
    }
  }
}

template <int KIND, int NRB, int UPW>
bool launch_k(const DenseArgs& a, hipStream_t st, std::string* why) {
  const int ld = dense_ld(a.K0, a.S, KIND == DGC_TIME_NONE ? 0 : a.H);
  const size_t lds = dense_lds_bytes(a.K0, a.S, KIND == DGC_TIME_NONE ? 0 : a.H);
  constexpr bool kSeq = KIND != DGC_TIME_NONE;
  static bool attr_done = false;  // per instantiation
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dense<KIND, NRB, UPW, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess && kSeq)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dense<KIND, NRB, UPW, kSeq>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) {
      if (why) *why = std::string("hipFuncSetAttribute: ") + hipGetErrorString(e);
      return false;
    }
    attr_done = true;
  }
  if (a.n_tiles > 0) {
    if (kSeq && a.seq_in)
      hipLaunchKernelGGL((k_dense<KIND, NRB, UPW, kSeq>), (unsigned)a.n_tiles, kThreads, lds, st, a, ld);
    else
      hipLaunchKernelGGL((k_dense<KIND, NRB, UPW, false>), (unsigned)a.n_tiles, kThreads, lds, st, a, ld);
  }
  return true;
}

template <int KIND>
bool launch_kind(const DenseArgs& a, hipStream_t st, std::string* why) {
  const int mx = KIND == DGC_TIME_NONE ? a.S : (a.S > a.H ? a.S : a.H);
  if (mx <= 64) return launch_k<KIND, 1, 1>(a, st, why);
  if (mx <= 128) return launch_k<KIND, 2, 1>(a, st, why);
  if (mx <= 256) return launch_k<KIND, 2, 2>(a, st, why);
  if (why) *why = "S and H above 256 are not supported";
  return false;
}

}  // namespace

// common row stride of the two LDS buffers: widest of the three operands, +4 floats so that
// float4 accesses of 32 consecutive rows spread over the banks
int dense_ld(int32_t K0, int32_t S, int32_t H) {
  const int Kp0 = ((K0 + 7) / 8) * 8;
  int m = Kp0 > S ? Kp0 : S;
  if (H > m) m = H;
  return m + 4;
}

size_t dense_lds_bytes(int32_t K0, int32_t S, int32_t H) {
  return sizeof(float) * ((size_t)kTileRows * 2 * dense_ld(K0, S, H) + 3 * kTileRows + 4 * (size_t)H);
}

void launch_pack_weight(const float* W, int32_t n_out, int32_t n_in, float4* packed, hipStream_t st) {
  const int64_t total = (int64_t)(n_out / 32) * ((n_in + 7) / 8) * 64;
  if (total > 0)
    hipLaunchKernelGGL(k_pack_weight, (unsigned)((total + 255) / 256), 256, 0, st, W, n_out, n_in, packed);
}

bool launch_dense(const DenseArgs& a, hipStream_t st, std::string* why) {
  if (a.variant != DGC_DENSE_TILE && dense_wave_supported(a)) return launch_dense_wave(a, st, why);
  if (a.variant == DGC_DENSE_WAVE || a.X2 || a.input_is_z || a.m_by_vertex) {
    if (why) *why = "the wave-private dense kernel needs S = H in {32, 64, 128}";
    return false;
  }
  if (a.S % 32 || (a.time_kind != DGC_TIME_NONE && a.H % 32)) {
    if (why) *why = "S and H must be multiples of 32";
    return false;
  }
  if (dense_lds_bytes(a.K0, a.S, a.time_kind == DGC_TIME_NONE ? 0 : a.H) > 160 * 1024) {
    if (why) *why = "tile does not fit in LDS";
    return false;
  }
  switch (a.time_kind) {
    case DGC_TIME_NONE: return launch_kind<DGC_TIME_NONE>(a, st, why);
    case DGC_TIME_GRU: return launch_kind<DGC_TIME_GRU>(a, st, why);
    case DGC_TIME_LSTM: return launch_kind<DGC_TIME_LSTM>(a, st, why);
  }
  if (why) *why = "unknown time encoder";
  return false;
}

}  // namespace dgc
