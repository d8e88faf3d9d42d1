// Dense part of the layer, wave-private variant (S = H = 32, 64 or 128): one WAVEFRONT owns 32
// vertices of a chunk and walks the chunk's window alone.  Rows of the GEMMs are independent,
// so nothing is shared between waves: there is no workgroup barrier and no cross-wave LDS
// traffic anywhere in the recurrence.
//
// With the weights as the MFMA's A operand and the activations as its B operand
// (v_mfma_f32_32x32x2f32: lane l supplies A[l%32][l/32], B[l/32][l%32]; receives
// D[8*(v/4) + 4*(l/32) + v%4][l%32] in register v), a lane receives, for activation row l%32,
// the output columns 8*g4 + 4*(l/32) + e (g4, e = 0..3) of a 32-column block in registers
// 4*g4 + e.  Read as the B operand of the NEXT product, the same lane has to supply
// X[row l%32][k = 8*kb + 4*(l/32) + q]: the very same registers (kb = g4, q = e).  So the hidden
// state h never leaves the registers between steps, and the gate arithmetic is elementwise in
// that layout.  Z = act(M W^T + b) makes one trip through a wave-private LDS tile (it would
// cost another 16*NJB registers), the aggregated rows M are read straight from global memory
// as B operands, and the weights stream from L2 in pre-packed fragment order.
#include "dgc_internal.h"

namespace dgc {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kRows = kWaveTileRows;  // 32
constexpr int kXAhead = 4;            // k-blocks of aggregated rows in flight (HBM latency)

__device__ __forceinline__ float sigmoid_fast(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ __forceinline__ float tanh_fast(float x) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x)); }
__device__ __forceinline__ float f4get(const float4& v, int q) { return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w; }
__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }

// acc[g] += W_g(k-block) x X(k-block) for NG weight fragments sharing one activation fragment
template <int NG>
__device__ __forceinline__ void mma8(floatx16 (&acc)[NG], const float4 (&w)[NG], const float4& x) {
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int g = 0; g < NG; ++g)
      acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(f4get(w[g], q), f4get(x, q), acc[g], 0, 0, 0);
}

// wp[g]: wave-uniform base of gate g's fragments; fragment kb of this lane is wp[g][kb*64 + lane].
// Keeping the base uniform lets the load use a scalar base register plus one small vector
// offset instead of a 64-bit vector address per load.
typedef int intx4 __attribute__((ext_vector_type(4)));

// Weights are fetched with buffer loads: one 128-bit resource descriptor per matrix in scalar
// registers, the lane's 16-byte slot as the only vector offset, and the fragment's position
// (gate, column block, k-block) as a scalar byte offset.  No 64-bit vector address exists, so
// the unrolled loops below do not drown in address registers.
struct WeightStream {
  __amdgpu_buffer_rsrc_t rsrc;
  __device__ __forceinline__ float4 frag(int lane16, int soff_bytes) const {
    const intx4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane16, soff_bytes, 0);
    return make_float4(__int_as_float(v.x), __int_as_float(v.y), __int_as_float(v.z), __int_as_float(v.w));
  }
};
__device__ __forceinline__ WeightStream make_stream(const float4* p, int64_t bytes) {
  WeightStream w;
  w.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float4*>(p), 0, (int)bytes, 0x00020000);
  return w;
}

// fragment kb of NG gates; soff[g] = byte offset of gate g's fragment 0 (wave-uniform)
template <int NG>
__device__ __forceinline__ void load_w(float4 (&w)[NG], const WeightStream& ws, const int (&soff)[NG], int kb,
                                       int lane16) {
#pragma unroll
  for (int g = 0; g < NG; ++g) w[g] = ws.frag(lane16, soff[g] + kb * 1024);
}

// The K loops below are chained: each one starts with its fragment 0 already in flight (wq,
// requested by the loop before it) and, in its last pair of k-blocks, requests fragment 0 of
// the loop that follows (ws_next / soff_next).  So the L2 latency of a loop's first weights
// hides behind the tail of the previous loop and the gate arithmetic in between.

// K loop with the activation fragments in LDS (row l%32 of a [32][ldz] tile, float4 at k).
template <int NG, int NKB, int NGN, int NWQ>
__device__ __forceinline__ void k_loop_lds(floatx16 (&acc)[NG], const float* ldsX, const WeightStream& ws,
                                           const int (&soff)[NG], int lane16, float4 (&wq)[NWQ],
                                           const WeightStream& ws_next, const int (&soff_next)[NGN]) {
  static_assert(NKB % 2 == 0 && NG <= NWQ && NGN <= NWQ, "");
  float4 w0[NG], w1[NG], x0, x1;
#pragma unroll
  for (int g = 0; g < NG; ++g) w0[g] = wq[g];
  x0 = *reinterpret_cast<const float4*>(ldsX);
#pragma unroll
  for (int kb = 0; kb < NKB; kb += 2) {
    load_w<NG>(w1, ws, soff, kb + 1, lane16);
    x1 = *reinterpret_cast<const float4*>(ldsX + (kb + 1) * 8);
    __builtin_amdgcn_sched_barrier(0);
    mma8<NG>(acc, w0, x0);
    __builtin_amdgcn_sched_barrier(0);
    if (kb + 2 < NKB) {
      load_w<NG>(w0, ws, soff, kb + 2, lane16);
      x0 = *reinterpret_cast<const float4*>(ldsX + (kb + 2) * 8);
    } else {
#pragma unroll
      for (int g = 0; g < NGN; ++g) wq[g] = ws_next.frag(lane16, soff_next[g]);
    }
    __builtin_amdgcn_sched_barrier(0);
    mma8<NG>(acc, w1, x1);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// K loop with the activation fragments in registers: x[kb] for kb = 0..NKB-1 (NKB even).
template <int NG, int NKB, int NGN, int NWQ>
__device__ __forceinline__ void k_loop_reg(floatx16 (&acc)[NG], const float4 (&x)[NKB], const WeightStream& ws,
                                           const int (&soff)[NG], int lane16, float4 (&wq)[NWQ],
                                           const WeightStream& ws_next, const int (&soff_next)[NGN]) {
  static_assert(NKB % 2 == 0 && NG <= NWQ && NGN <= NWQ, "");
  float4 w0[NG], w1[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) w0[g] = wq[g];
#pragma unroll
  for (int kb = 0; kb < NKB; kb += 2) {
    load_w<NG>(w1, ws, soff, kb + 1, lane16);
    __builtin_amdgcn_sched_barrier(0);
    mma8<NG>(acc, w0, x[kb]);
    __builtin_amdgcn_sched_barrier(0);
    if (kb + 2 < NKB) {
      load_w<NG>(w0, ws, soff, kb + 2, lane16);
    } else {
#pragma unroll
      for (int g = 0; g < NGN; ++g) wq[g] = ws_next.frag(lane16, soff_next[g]);
    }
    __builtin_amdgcn_sched_barrier(0);
    mma8<NG>(acc, w1, x[kb + 1]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// KIND: DGC_TIME_*;  NJB = S/32 = H/32.
// the state (h, and c for the LSTM) after a sequence's last row goes to that sequence's row of HN
template <int KIND, int NKB>
__device__ __forceinline__ void store_state_t(const DenseArgs& a, int64_t idx, int64_t V, int H, int half,
                                              const float4 (&h)[NKB], const float4 (&c)[NKB]) {
  if (!a.HN) return;
  const int64_t so = a.seq_out[idx];
  if (so < 0) return;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    *reinterpret_cast<float4*>(a.HN + so * H + 8 * kb + 4 * half) = h[kb];
    if constexpr (KIND == DGC_TIME_LSTM) *reinterpret_cast<float4*>(a.HN + (V + so) * H + 8 * kb + 4 * half) = c[kb];
  }
}

// SEQ: the rows of a tile hold several sequences one after the other (temporal fusion with
// states): states enter and leave through the tables seq_in / seq_out instead of at the window's ends.
// CAT: the time encoder's input is [X2 row, Z] (2S wide): X2 holds the first structure layer's
// output of the same (snapshot, vertex); it shares the Z tile in LDS, columns 0..S-1.
// STACK: this launch is a stacked second recurrent layer: no transform, the input rows are rows
// t*N + v of a [T,N,ldm] tensor (DenseArgs::m_by_vertex and input_is_z, which go together).
template <int KIND, int NJB, bool SEQ, bool CAT, bool STACK = false>
__global__ __launch_bounds__(kWave, (KIND == DGC_TIME_LSTM ? 1 : 2)) void k_dense_wave(DenseArgs a) {
  // LDS, private to this wave (the workgroup is one wave):
  //   zbuf [32][ldz] the Z tile | gbias [4][H] gate biases, pre-summed | zbias [S]
  // (biases are read from LDS inside the step loop: as global loads they would be hoisted out
  //  of it and held in hundreds of registers)
  extern __shared__ __align__(16) float zbuf[];
  constexpr int H = NJB * 32;
  constexpr int NKB = NJB * 4;     // k-blocks of 8 over S or H
  constexpr int NKX = CAT ? 2 * NKB : NKB;   // k-blocks of the time encoder's input
  constexpr int zcol = CAT ? H : 0;          // where Z starts in a row of the tile
  constexpr int ldz = H + zcol + 4;  // +4 floats: float4 accesses of 32 rows spread over the banks
  float* gbias = zbuf + (KIND == DGC_TIME_NONE ? 0 : kRows * ldz);
  float* zbias = gbias + (KIND == DGC_TIME_NONE ? 0 : 4 * H);
  for (int i = threadIdx.x; i < H; i += kWave) {
    zbias[i] = a.bg[i];
    if constexpr (KIND == DGC_TIME_GRU) {
      gbias[i] = a.bih[i] + a.bhh[i];
      gbias[H + i] = a.bih[H + i] + a.bhh[H + i];
      gbias[2 * H + i] = a.bih[2 * H + i];
      gbias[3 * H + i] = a.bhh[2 * H + i];
    }
    if constexpr (KIND == DGC_TIME_LSTM) {
#pragma unroll
      for (int g = 0; g < 4; ++g) gbias[g * H + i] = a.bih[g * H + i] + a.bhh[g * H + i];
    }
  }
  __syncthreads();

  const DenseTile tile = a.tiles32[blockIdx.x];
  const ChunkInfo ch = a.chunks[tile.chunk];
  const int lane = threadIdx.x, l32 = lane & 31, half = lane >> 5;
  const int nrows = tile.nrows;
  const bool valid = l32 < nrows;
  const int row = valid ? l32 : nrows - 1;   // rows past the tile's end recompute its last row; never stored
  const int lane16 = lane * 16;
  const int K0 = a.K0, nkb0 = (K0 + 7) / 8;
  const WeightStream wsg = make_stream(a.Wg, a.wg_bytes);
  const WeightStream wsi = make_stream(a.Wih, (int64_t)(KIND == DGC_TIME_LSTM ? 4 : 3) * NJB * NKX * 1024);
  const WeightStream wsh = make_stream(a.Whh, (int64_t)(KIND == DGC_TIME_LSTM ? 4 : 3) * NJB * NKB * 1024);
  const int64_t V = a.total_state_rows;
  const int64_t vrow = ch.v_lo + tile.v0 + row;          // this lane's vertex
  const int64_t srow = ch.state_off + tile.v0 + row;     // this lane's state row

  // state: h[kb] = columns 8*kb + 4*half .. +3 of this lane's row  (kb = 4*jb + g4)
  float4 h[NKB], c[NKB];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    h[kb] = zero4();
    c[kb] = zero4();
    if constexpr (KIND != DGC_TIME_NONE && !SEQ) {
      if (a.H0) {
        h[kb] = *reinterpret_cast<const float4*>(a.H0 + srow * H + 8 * kb + 4 * half);
        if constexpr (KIND == DGC_TIME_LSTM)
          c[kb] = *reinterpret_cast<const float4*>(a.H0 + (V + srow) * H + 8 * kb + 4 * half);
      }
    }
  }

  // Aggregated rows as B operand, straight from global memory: float4 at column 8*kb + 4*half of
  // this lane's row.  (The library's M buffer has a pitch that is a multiple of 8 with zero pad
  // columns, so a k-block never needs masking.)
  // (m_by_vertex: the input rows are not the packed aggregated rows but rows t*N + v of a [T,N,ldm]
  //  tensor - the first recurrent layer's output when this launch runs a stacked second layer)
  // (STACK over lanes, i.e. with a row map: the input row of a slot is the row of Y the slot's output
  //  goes to; the map entry of the next step is fetched one step ahead, an empty slot reads row 0)
  int yrow_next = 0;
  if constexpr (STACK && SEQ) {
    if (a.y_map) yrow_next = (int)a.y_map[(int64_t)ch.t_lo * a.N + vrow];
  }
  const float* mrow0 = STACK ? a.M + ((STACK && SEQ && a.y_map) ? (int64_t)max(yrow_next, 0)
                                                                 : (int64_t)ch.t_lo * a.N + vrow) * a.ldm + 4 * half
                             : a.M + (ch.row_off0 + tile.v0 + row) * a.ldm + 4 * half;
  const int64_t mstep = STACK ? a.N * a.ldm : ch.nv * a.ldm;
  float4 xq[kXAhead];
#pragma unroll
  for (int i = 0; i < kXAhead; ++i) xq[i] = i < nkb0 ? *reinterpret_cast<const float4*>(mrow0 + 8 * i) : zero4();
  // fragment 0 of the next K loop's weights (see k_loop_lds)
  // (with per-snapshot GCN weights, snapshot t's fragments start t * wg_step_bytes further on)
  int soffg[NJB];
#pragma unroll
  for (int jb = 0; jb < NJB; ++jb) soffg[jb] = jb * nkb0 * 1024 + ch.t_lo * a.wg_step_bytes;
  float4 wq[NJB > 4 ? NJB : 4];
#pragma unroll
  for (int jb = 0; jb < NJB; ++jb) wq[jb] = wsg.frag(lane16, soffg[jb]);

  float4 x2[CAT ? NKB : 1];
  // SEQ with a row map: row of Y that the output of the previous / the current step goes to (a table
  // entry < 0: nowhere; the host checks that the rows of Y number less than 2^31)
  int yrow_prev = 0, yrow = 0;
  for (int s = 0; s < ch.w; ++s) {
    const int64_t t = ch.t_lo + s;
    if constexpr (SEQ) {
      yrow_prev = yrow;
      if constexpr (STACK) {
        if (a.y_map) {
          yrow = yrow_next;
          if (s + 1 < ch.w) yrow_next = (int)a.y_map[(t + 1) * a.N + vrow];
        }
      } else {
        if (a.y_map) yrow = (int)a.y_map[t * a.N + vrow];   // used one step later: no wait here
      }
    }
    const float* mrow = (STACK && SEQ && a.y_map) ? a.M + (int64_t)max(yrow, 0) * a.ldm + 4 * half : mrow0 + s * mstep;
    auto load_x = [&](int kb) -> float4 { return *reinterpret_cast<const float4*>(mrow + 8 * kb); };
    if (s > 0) {
#pragma unroll
      for (int i = 0; i < kXAhead; ++i)
        if (i < nkb0) xq[i] = load_x(i);
    }
    if constexpr (CAT) {   // the other half of the time encoder's input: arrives during the transform
      int64_t r2 = t * a.N + vrow;
      if (a.x2_map) r2 = max(a.x2_map[r2], (int64_t)0);    // an empty slot reads row 0; its output is never used
      const float* p2 = a.X2 + r2 * a.ldx2 + 4 * half;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) x2[kb] = *reinterpret_cast<const float4*>(p2 + 8 * kb);
    }
    if (s > 0) {
      // h_{t-1} -> Y, issued after the loads above: memory operations retire in order, so loads
      // issued behind these stores would wait for them
      if constexpr (KIND != DGC_TIME_NONE) {
        if (valid) {
          const int64_t yr = (SEQ && a.y_map) ? (int64_t)yrow_prev : (t - 1) * a.N + vrow;
          if (yr >= 0) {
            float* y = a.Y + yr * a.ldy + 4 * half;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) *reinterpret_cast<float4*>(y + 8 * kb) = h[kb];
          }
          if constexpr (SEQ) store_state_t<KIND, NKB>(a, (t - 1) * a.N + vrow, V, H, half, h, c);
        }
      }
    }

    // temporal-fusion mask on the incoming state (Section 5.1.2)
    if constexpr (KIND != DGC_TIME_NONE && !SEQ) {
      if (a.reset_mask && a.reset_mask[t * a.N + vrow]) {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) { h[kb] = zero4(); c[kb] = zero4(); }
      }
    }
    if constexpr (KIND != DGC_TIME_NONE && SEQ) {
      const int64_t sr = a.seq_in[t * a.N + vrow];
      if (sr >= 0) {   // a sequence starts here: its own state row, or zero
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
          h[kb] = a.H0 ? *reinterpret_cast<const float4*>(a.H0 + sr * H + 8 * kb + 4 * half) : zero4();
          if constexpr (KIND == DGC_TIME_LSTM)
            c[kb] = a.H0 ? *reinterpret_cast<const float4*>(a.H0 + (V + sr) * H + 8 * kb + 4 * half) : zero4();
        }
      }
    }

    // Z = act(M W^T + b): all NJB column blocks at once, they share the activation fragment
    floatx16 zacc[NJB];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) zacc[jb] = (floatx16)(0.f);
    {
      const int (&soff)[NJB] = soffg;
      float4 w0[NJB], w1[NJB];
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb) w0[jb] = wq[jb];
      for (int kb = 0; kb < nkb0; kb += kXAhead) {
#pragma unroll
        for (int i = 0; i < kXAhead; i += 2) {
          // uniform guards: nkb0 need not be a multiple of kXAhead
          if (kb + i < nkb0) {
            load_w<NJB>(w1, wsg, soff, kb + i + 1 < nkb0 ? kb + i + 1 : kb + i, lane16);
            const float4 x = xq[i];
            if (kb + i + kXAhead < nkb0) xq[i] = load_x(kb + i + kXAhead);
            __builtin_amdgcn_sched_barrier(0);
            mma8<NJB>(zacc, w0, x);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (kb + i + 1 < nkb0) {
            load_w<NJB>(w0, wsg, soff, kb + i + 2 < nkb0 ? kb + i + 2 : kb + i + 1, lane16);
            const float4 x = xq[i + 1];
            if (kb + i + 1 + kXAhead < nkb0) xq[i + 1] = load_x(kb + i + 1 + kXAhead);
            __builtin_amdgcn_sched_barrier(0);
            mma8<NJB>(zacc, w1, x);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
    constexpr int NG = KIND == DGC_TIME_LSTM ? 4 : 3;
    if constexpr (KIND == DGC_TIME_NONE) {
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb) {   // next step's first weights
        soffg[jb] += a.wg_step_bytes;
        wq[jb] = wsg.frag(lane16, soffg[jb]);
      }
    } else {
#pragma unroll
      for (int g = 0; g < NG; ++g) wq[g] = wsi.frag(lane16, (g * NJB) * NKX * 1024);  // gates of column block 0
    }
    float4 z[NKB];
    if constexpr (STACK) {
      // no transform (K0 = 0, the loop above did nothing): the input row is the time encoder's input,
      // and its float4 at column 8*kb + 4*half is exactly this lane's fragment kb
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) z[kb] = load_x(kb);
    } else {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
        const float4 b = *reinterpret_cast<const float4*>(zbias + 8 * kb + 4 * half);
        const int jb = kb / 4, g4 = kb % 4;
        z[kb] = make_float4(zacc[jb][4 * g4 + 0] + b.x, zacc[jb][4 * g4 + 1] + b.y, zacc[jb][4 * g4 + 2] + b.z,
                            zacc[jb][4 * g4 + 3] + b.w);
        if (a.act == DGC_ACT_RELU) {
          z[kb].x = fmaxf(z[kb].x, 0.f); z[kb].y = fmaxf(z[kb].y, 0.f);
          z[kb].z = fmaxf(z[kb].z, 0.f); z[kb].w = fmaxf(z[kb].w, 0.f);
        }
      }
    }

    if constexpr (KIND == DGC_TIME_NONE) {
      if (valid) {
        float* y = a.Y + (t * a.N + vrow) * a.ldy + 4 * half;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) *reinterpret_cast<float4*>(y + 8 * kb) = z[kb];
      }
    } else {
      // Z -> wave-private LDS tile (frees its registers for the gate accumulators)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) *reinterpret_cast<float4*>(zbuf + l32 * ldz + zcol + 8 * kb + 4 * half) = z[kb];
      if constexpr (CAT) {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)   // rebuilt element by element: a whole-struct copy to LDS kept x2 in scratch memory
          *reinterpret_cast<float4*>(zbuf + l32 * ldz + 8 * kb + 4 * half) = make_float4(x2[kb].x, x2[kb].y, x2[kb].z, x2[kb].w);
      }
      __syncthreads();  // one wave: orders the LDS writes before the reads below
      const float* ldsZ = zbuf + l32 * ldz + 4 * half;

      float4 hn[NKB], cn[NKB];
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb) {
        // GRU slots: 0 r, 1 z, 2 input part of n, 3 hidden part of n.  LSTM: i, f, g, o.
        floatx16 acc[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[g] = (floatx16)(0.f);
        int soff[NG], soffx[NG];   // hidden-side and input-side fragments of this column block
#pragma unroll
        for (int g = 0; g < NG; ++g) { soff[g] = (g * NJB + jb) * NKB * 1024; soffx[g] = (g * NJB + jb) * NKX * 1024; }
        // what follows the hidden-state loop: the next column block's gates, or the next
        // step's transform
        int soff_next[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) soff_next[g] = (g * NJB + jb + 1) * NKX * 1024;
        if (jb + 1 == NJB) {
#pragma unroll
          for (int j2 = 0; j2 < NJB; ++j2) soffg[j2] += a.wg_step_bytes;
        }
        if constexpr (KIND == DGC_TIME_GRU) {
          floatx16 ai[3] = {acc[0], acc[1], acc[2]};   // r, z, input part of n
          k_loop_lds<3, NKX, 3, 4>(ai, ldsZ, wsi, soffx, lane16, wq, wsh, soff);
          floatx16 ah[3] = {ai[0], ai[1], acc[3]};     // r, z, hidden part of n
          if (jb + 1 < NJB) k_loop_reg<3, NKB, 3, 4>(ah, h, wsh, soff, lane16, wq, wsi, soff_next);
          else k_loop_reg<3, NKB, NJB, 4>(ah, h, wsh, soff, lane16, wq, wsg, soffg);
          acc[0] = ah[0]; acc[1] = ah[1]; acc[2] = ai[2]; acc[3] = ah[2];
        } else {
          k_loop_lds<4, NKX, 4, 4>(acc, ldsZ, wsi, soffx, lane16, wq, wsh, soff);
          if (jb + 1 < NJB) k_loop_reg<4, NKB, 4, 4>(acc, h, wsh, soff, lane16, wq, wsi, soff_next);
          else k_loop_reg<4, NKB, NJB, 4>(acc, h, wsh, soff, lane16, wq, wsg, soffg);
        }
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int kb = 4 * jb + g4, c0 = 8 * kb + 4 * half;
          float o[4], oc[4];
          float bs[4][4];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 b = *reinterpret_cast<const float4*>(gbias + g * H + c0);
            bs[g][0] = b.x; bs[g][1] = b.y; bs[g][2] = b.z; bs[g][3] = b.w;
          }
          if constexpr (KIND == DGC_TIME_GRU) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int v = 4 * g4 + e;
              const float r = sigmoid_fast(acc[0][v] + bs[0][e]);
              const float zg = sigmoid_fast(acc[1][v] + bs[1][e]);
              const float n = tanh_fast(acc[2][v] + bs[2][e] + r * (acc[3][v] + bs[3][e]));
              o[e] = (1.0f - zg) * n + zg * f4get(h[kb], e);
              oc[e] = 0.f;
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int v = 4 * g4 + e;
              const float ig = sigmoid_fast(acc[0][v] + bs[0][e]);
              const float fg = sigmoid_fast(acc[1][v] + bs[1][e]);
              const float gg = tanh_fast(acc[2][v] + bs[2][e]);
              const float og = sigmoid_fast(acc[3][v] + bs[3][e]);
              oc[e] = fg * f4get(c[kb], e) + ig * gg;
              o[e] = og * tanh_fast(oc[e]);
            }
          }
          hn[kb] = make_float4(o[0], o[1], o[2], o[3]);
          cn[kb] = make_float4(oc[0], oc[1], oc[2], oc[3]);
        }
      }
      __syncthreads();  // the Z tile is rewritten in the next step
      // the new state replaces the old one in place (same register layout); it is written to Y
      // at the top of the next step, behind that step's first loads
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
        h[kb] = hn[kb];
        if constexpr (KIND == DGC_TIME_LSTM) c[kb] = cn[kb];
      }
    }
  }

  if constexpr (KIND != DGC_TIME_NONE) {
    if (valid) {  // the last step's output
      const int64_t yr = (SEQ && a.y_map) ? (int64_t)yrow : (int64_t)(ch.t_lo + ch.w - 1) * a.N + vrow;
      if (yr >= 0) {
        float* y = a.Y + yr * a.ldy + 4 * half;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) *reinterpret_cast<float4*>(y + 8 * kb) = h[kb];
      }
      if constexpr (SEQ) store_state_t<KIND, NKB>(a, (int64_t)(ch.t_lo + ch.w - 1) * a.N + vrow, V, H, half, h, c);
    }
    if (!SEQ && a.HN && valid) {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
        *reinterpret_cast<float4*>(a.HN + srow * H + 8 * kb + 4 * half) = h[kb];
        if constexpr (KIND == DGC_TIME_LSTM)
          *reinterpret_cast<float4*>(a.HN + (V + srow) * H + 8 * kb + 4 * half) = c[kb];
      }
    }
  }
}

template <int KIND, int NJB>
bool launch_w(const DenseArgs& a, hipStream_t st, std::string* why) {
  constexpr bool kLstm = KIND == DGC_TIME_LSTM, kRnn = KIND != DGC_TIME_NONE;
  const bool cat = a.X2 != nullptr;
  if (cat && !kLstm) {
    if (why) *why = "the concatenated input is built for the LSTM";
    return false;
  }
  const int ldz = NJB * 32 * (cat ? 2 : 1) + 4;
  const size_t lds = sizeof(float) * ((kRnn ? kRows * ldz + 4 * NJB * 32 : 0) + NJB * 32);
  if (a.n_tiles32 > 0) {
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, (unsigned)a.n_tiles32, kWave, lds, st, a);
    };
    if (a.input_is_z != a.m_by_vertex || (a.input_is_z && (!kRnn || cat))) {
      if (why) *why = "a stacked recurrent layer runs without the concatenated input";
      return false;
    }
    if (a.input_is_z && a.seq_in) go(k_dense_wave<KIND, NJB, kRnn, false, kRnn>);
    else if (a.input_is_z) go(k_dense_wave<KIND, NJB, false, false, kRnn>);
    else if (kRnn && a.seq_in && cat) go(k_dense_wave<KIND, NJB, kRnn, kLstm>);
    else if (kRnn && a.seq_in) go(k_dense_wave<KIND, NJB, kRnn, false>);
    else if (cat) go(k_dense_wave<KIND, NJB, false, kLstm>);
    else go(k_dense_wave<KIND, NJB, false, false>);
  }
  return true;
}

template <int KIND>
bool launch_wk(const DenseArgs& a, hipStream_t st, std::string* why) {
  switch (a.S / 32) {
    case 1: return launch_w<KIND, 1>(a, st, why);
    case 2: return launch_w<KIND, 2>(a, st, why);
    case 4: return launch_w<KIND, 4>(a, st, why);
    case 8:
      if constexpr (KIND == DGC_TIME_NONE) return launch_w<KIND, 8>(a, st, why);
  }
  return false;
}

}  // namespace

bool dense_wave_supported(const DenseArgs& a) {
  const bool s_ok = a.S == 32 || a.S == 64 || a.S == 128 || (a.S == 256 && a.time_kind == DGC_TIME_NONE);
  const bool m_ok = a.ldm % 8 == 0 && a.ldm >= (a.K0 + 7) / 8 * 8;  // whole k-blocks, zero padded
  if (a.input_is_z && (a.time_kind == DGC_TIME_NONE || a.K0 != 0 || a.ldm < a.S || a.ldm % 4)) return false;
  return s_ok && (m_ok || a.input_is_z) && (a.time_kind == DGC_TIME_NONE || a.H == a.S);
}

bool launch_dense_wave(const DenseArgs& a, hipStream_t st, std::string* why) {
  switch (a.time_kind) {
    case DGC_TIME_NONE: return launch_wk<DGC_TIME_NONE>(a, st, why);
    case DGC_TIME_GRU: return launch_wk<DGC_TIME_GRU>(a, st, why);
    case DGC_TIME_LSTM: return launch_wk<DGC_TIME_LSTM>(a, st, why);
  }
  return false;
}

}  // namespace dgc
