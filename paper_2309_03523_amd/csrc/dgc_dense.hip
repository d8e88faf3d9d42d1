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
// MFMA: v_mfma_f32_32x32x2f32.  Lane l supplies A[l%32][l/32] and B[l/32][l%32]; it receives
// C[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v (0..15).  A operands (M, Z, h)
// are read from LDS as float4 (four consecutive k per lane), B operands (weights) straight
// from global memory / L2 in a pre-packed fragment order, so that every load is one contiguous
// 1 KiB per wave and no LDS staging or barrier is needed for them.
#include "dgc_internal.h"

namespace dgc {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

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

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

// acc[rb][SLOTg] += A[rows of block rb][k] * W_g[cols][k], k over nkb blocks of 8.
//  ldsA : LDS address of A[row l%32 of block 0][(l/32)*4]; block rb adds rb*32*lda
//  wp[g]: packed weight fragments of gate g for this column block, already offset by lane;
//         fragment kb is wp[g][kb*64]
template <int NRB, int NG, int S0, int S1, int S2, int S3>
__device__ __forceinline__ void mma_k_loop(floatx16 (&acc)[NRB][4], const float* ldsA, int lda, int nkb,
                                           const float4* const (&wp)[NG]) {
  constexpr int slot[4] = {S0, S1, S2, S3};
  float4 a_cur[NRB], b_cur[NG];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) a_cur[rb] = *reinterpret_cast<const float4*>(ldsA + rb * 32 * lda);
#pragma unroll
  for (int g = 0; g < NG; ++g) b_cur[g] = wp[g][0];
  for (int kb = 0; kb < nkb; ++kb) {
    float4 a_nxt[NRB], b_nxt[NG];
    const int kn = kb + 1 < nkb ? kb + 1 : kb;
#pragma unroll
    for (int g = 0; g < NG; ++g) b_nxt[g] = wp[g][(int64_t)kn * 64];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
      a_nxt[rb] = *reinterpret_cast<const float4*>(ldsA + rb * 32 * lda + kn * 8);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const float bv = q == 0 ? b_cur[g].x : q == 1 ? b_cur[g].y : q == 2 ? b_cur[g].z : b_cur[g].w;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
          const float av = q == 0 ? a_cur[rb].x : q == 1 ? a_cur[rb].y : q == 2 ? a_cur[rb].z : a_cur[rb].w;
          acc[rb][slot[g]] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[rb][slot[g]], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) a_cur[rb] = a_nxt[rb];
#pragma unroll
    for (int g = 0; g < NG; ++g) b_cur[g] = b_nxt[g];
  }
}

// KIND: DGC_TIME_*.  NRB: 32-row blocks per unit (1 or 2).  UPW: units per wave.
// A unit is NRB row blocks x one 32-column block (x all gates).
//
// LDS holds two [64][ld] buffers that swap roles every step:
//   P: the state h entering the step;   Q: the aggregated rows, then Z, then the new state.
// Per step: load M -> Q and mask P | Z = act(Q W^T + b) in registers | Z -> Q | gate GEMMs read
// Q and P | gate arithmetic writes the new h into Q | Q -> Y | swap(P, Q).
template <int KIND, int NRB, int UPW>
__global__ __launch_bounds__(kThreads, 2) void k_dense(DenseArgs a, int ld) {
  extern __shared__ float smem[];
  float* P = smem;
  float* Q = smem + kTileRows * ld;
  int* mask_row = reinterpret_cast<int*>(smem + 2 * kTileRows * ld);

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
          const int row = (rb0 + rb) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
          const int col = jb * 32 + l32;
          cst[ui][rb][v] = (a.H0 && u < unitsH && row < nrows) ? a.H0[(V + sbase + row) * H + col] : 0.f;
        }
    }
  }
  if constexpr (KIND != DGC_TIME_NONE) {
    const int hf4 = H / 4;
    for (int idx = tid; idx < kTileRows * hf4; idx += kThreads) {
      const int r = idx / hf4, c4 = idx - r * hf4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (a.H0 && r < nrows) v = *reinterpret_cast<const float4*>(a.H0 + (sbase + r) * H + 4 * c4);
      *reinterpret_cast<float4*>(P + r * ld + 4 * c4) = v;
    }
  }

  for (int s = 0; s < ch.w; ++s) {
    const int64_t t = ch.t_lo + s;
    // (a) aggregated rows of this step -> Q, zero beyond K0 and beyond nrows
    {
      const float* Mrow0 = a.M + (ch.row_off0 + (int64_t)s * ch.nv + tile.v0) * a.ldm;
      const int nf4 = nkb0 * 2;
      for (int idx = tid; idx < kTileRows * nf4; idx += kThreads) {
        const int r = idx / nf4, c4 = idx - r * nf4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < nrows && 4 * c4 < a.ldm) {
          v = *reinterpret_cast<const float4*>(Mrow0 + (int64_t)r * a.ldm + 4 * c4);
          if (4 * c4 + 1 >= K0) v.y = 0.f;
          if (4 * c4 + 2 >= K0) v.z = 0.f;
          if (4 * c4 + 3 >= K0) v.w = 0.f;
          if (4 * c4 >= K0) v.x = 0.f;
        }
        *reinterpret_cast<float4*>(Q + r * ld + 4 * c4) = v;
      }
    }
    // (b) temporal-fusion mask: zero the incoming state of masked rows (same thread <-> element
    //     mapping as the Y store at the end of the previous step, so no barrier in between)
    if constexpr (KIND != DGC_TIME_NONE) {
      const int hf4 = H / 4;
      for (int idx = tid; idx < kTileRows * hf4; idx += kThreads) {
        const int r = idx / hf4, c4 = idx - r * hf4;
        const int mk = (a.reset_mask && r < nrows) ? a.reset_mask[t * a.N + vbase + r] : 0;
        if (mk) *reinterpret_cast<float4*>(P + r * ld + 4 * c4) = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c4 == 0) mask_row[r] = mk;
      }
    }
    __syncthreads();

    // (c) Z = act(M W^T + b) for this wave's units, kept in the accumulators over the barrier
    floatx16 zacc[UPW][NRB];
#pragma unroll
    for (int ui = 0; ui < UPW; ++ui) {
      const int u = wave + kWaves * ui;
      if (u < unitsS) {
        const int jb = u / RBU, rb0 = (u % RBU) * NRB;
        floatx16 acc[NRB][4];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) acc[rb][0] = (floatx16)(0.f);
        const float4* const wp[1] = {a.Wg + ((int64_t)jb * nkb0) * 64 + lane};
        mma_k_loop<NRB, 1, 0, 0, 0, 0>(acc, Q + (rb0 * 32 + l32) * ld + half * 4, ld, nkb0, wp);
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
        const float bias = a.bg[jb * 32 + l32];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = (rb0 + rb) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            float z = zacc[ui][rb][v] + bias;
            if (a.act == DGC_ACT_RELU) z = fmaxf(z, 0.f);
            Q[row * ld + jb * 32 + l32] = z;
          }
      }
    }
    __syncthreads();

    if constexpr (KIND == DGC_TIME_NONE) {
      const int sf4 = S / 4;
      for (int idx = tid; idx < kTileRows * sf4; idx += kThreads) {
        const int r = idx / sf4, c4 = idx - r * sf4;
        if (r < nrows)
          *reinterpret_cast<float4*>(a.Y + (t * a.N + vbase + r) * a.ldy + 4 * c4) =
              *reinterpret_cast<const float4*>(Q + r * ld + 4 * c4);
      }
      __syncthreads();  // Q is overwritten by the next step's rows
    } else {
      // (e) gate pre-activations.  With UPW > 1 a wave finishes unit after unit; the new state of
      //     a unit can only be written once every wave has stopped reading Z and h, so the gate
      //     values of earlier units wait in registers.
      float hnew[UPW][NRB][16];
#pragma unroll
      for (int ui = 0; ui < UPW; ++ui) {
        const int u = wave + kWaves * ui;
        if (u < unitsH) {
          const int jb = u / RBU, rb0 = (u % RBU) * NRB;
          const int col = jb * 32 + l32;
          floatx16 acc[NRB][4];
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
            mma_k_loop<NRB, 3, 0, 1, 2, 0>(acc, ldsZ, ld, nkbS, wi);
            mma_k_loop<NRB, 3, 0, 1, 3, 0>(acc, ldsHp, ld, nkbH, wh);
            const float b_r = a.bih[col] + a.bhh[col];
            const float b_z = a.bih[H + col] + a.bhh[H + col];
            const float b_in = a.bih[2 * H + col], b_hn = a.bhh[2 * H + col];
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int row = (rb0 + rb) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                const float hp = P[row * ld + col];
                const float r = sigmoidf_(acc[rb][0][v] + b_r);
                const float z = sigmoidf_(acc[rb][1][v] + b_z);
                const float n = tanhf(acc[rb][2][v] + b_in + r * (acc[rb][3][v] + b_hn));
                hnew[ui][rb][v] = (1.0f - z) * n + z * hp;
              }
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
            mma_k_loop<NRB, 4, 0, 1, 2, 3>(acc, ldsZ, ld, nkbS, wi);
            mma_k_loop<NRB, 4, 0, 1, 2, 3>(acc, ldsHp, ld, nkbH, wh);
            float bsum[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) bsum[g] = a.bih[g * H + col] + a.bhh[g * H + col];
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int row = (rb0 + rb) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                const float cm = mask_row[row] ? 0.f : cst[ui][rb][v];
                const float ig = sigmoidf_(acc[rb][0][v] + bsum[0]);
                const float fg = sigmoidf_(acc[rb][1][v] + bsum[1]);
                const float gg = tanhf(acc[rb][2][v] + bsum[2]);
                const float og = sigmoidf_(acc[rb][3][v] + bsum[3]);
                const float cn = fg * cm + ig * gg;
                cst[ui][rb][v] = cn;
                hnew[ui][rb][v] = og * tanhf(cn);
              }
          }
        }
      }
      __syncthreads();  // everyone has finished reading Z and the old state
#pragma unroll
      for (int ui = 0; ui < UPW; ++ui) {
        const int u = wave + kWaves * ui;
        if (u < unitsH) {
          const int jb = u / RBU, rb0 = (u % RBU) * NRB;
#pragma unroll
          for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int row = (rb0 + rb) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
              Q[row * ld + jb * 32 + l32] = hnew[ui][rb][v];
            }
        }
      }
      __syncthreads();
      // (g) h_t -> Y, whole rows at a time; Q becomes the state buffer of the next step
      const int hf4 = H / 4;
      const bool last = (s == ch.w - 1) && a.HN;
      for (int idx = tid; idx < kTileRows * hf4; idx += kThreads) {
        const int r = idx / hf4, c4 = idx - r * hf4;
        if (r < nrows) {
          const float4 v = *reinterpret_cast<const float4*>(Q + r * ld + 4 * c4);
          *reinterpret_cast<float4*>(a.Y + (t * a.N + vbase + r) * a.ldy + 4 * c4) = v;
          if (last) *reinterpret_cast<float4*>(a.HN + (sbase + r) * H + 4 * c4) = v;
        }
      }
      float* tmp = P; P = Q; Q = tmp;
    }
  }

  if constexpr (KIND == DGC_TIME_LSTM) {
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
              const int row = (rb0 + rb) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
              if (row < nrows) a.HN[(V + sbase + row) * H + jb * 32 + l32] = cst[ui][rb][v];
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
  static bool attr_done = false;  // per instantiation
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dense<KIND, NRB, UPW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) {
      if (why) *why = std::string("hipFuncSetAttribute: ") + hipGetErrorString(e);
      return false;
    }
    attr_done = true;
  }
  if (a.n_tiles > 0)
    hipLaunchKernelGGL((k_dense<KIND, NRB, UPW>), (unsigned)a.n_tiles, kThreads, lds, st, a, ld);
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
// float4 reads of 32 consecutive rows spread over the banks
int dense_ld(int32_t K0, int32_t S, int32_t H) {
  const int Kp0 = ((K0 + 7) / 8) * 8;
  int m = Kp0 > S ? Kp0 : S;
  if (H > m) m = H;
  return m + 4;
}

size_t dense_lds_bytes(int32_t K0, int32_t S, int32_t H) {
  return sizeof(float) * (size_t)kTileRows * 2 * dense_ld(K0, S, H) + sizeof(int) * kTileRows;
}

void launch_pack_weight(const float* W, int32_t n_out, int32_t n_in, float4* packed, hipStream_t st) {
  const int64_t total = (int64_t)(n_out / 32) * ((n_in + 7) / 8) * 64;
  if (total > 0)
    hipLaunchKernelGGL(k_pack_weight, (unsigned)((total + 255) / 256), 256, 0, st, W, n_out, n_in, packed);
}

bool launch_dense(const DenseArgs& a, hipStream_t st, std::string* why) {
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
