// EvolveGCN-O support (the paper lists EvolveGCN among its DGNNs, Section 1; the "-O" variant of
// the cited work is used): the GCN weight matrix W [F][S] is the state of a matrix GRU,
//     Zg = sig(Uz W + Vz W + Bz)   Rg = sig(Ur W + Vr W + Br)
//     Wc = tanh(Uh W + Vh (Rg*W) + Bh)      W' = (1 - Zg)*W + Zg*Wc
// evolved once per snapshot over all T snapshots (global, independent of the chunk windows),
// Y[t,i] = relu(M[t,i] W_t), mean-squared-error loss, gradients of all ten parameter matrices.
//
// Kernels here: a wave-per-tile fp32 MFMA GEMM for the small (F x F)(F x S) products of the
// weight recurrence and of its back-propagation through time (latency-bound: 64 waves per
// launch), the elementwise gate kernels, and the one large kernel of the backward pass,
// dW_t = M_t^T dP_t reduced over all rows of snapshot t across the fused chunks.
#include "dgc_internal.h"

namespace dgc {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float f4get(const float4& v, int q) { return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w; }
__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

// C[M][N] (+)= op(A) op(B), one wave per 32 x 32 tile of C; K a multiple of 8.
//  TA = false: A stored [M][K] (lda = K)      TA = true: A stored [K][M] (lda = M)
//  TB = false: B stored [K][N] (ldb = N)      TB = true: B stored [N][K] (ldb = K)
template <bool TA, bool TB>
__global__ __launch_bounds__(64) void k_small_gemm(const float* A, const float* B, float* C, int M, int N, int K,
                                                   int accumulate) {
  const int lane = threadIdx.x, l32 = lane & 31, half = lane >> 5;
  const int n0 = blockIdx.x * 32, m0 = blockIdx.y * 32;
  const int lda = TA ? M : K, ldb = TB ? K : N;
  floatx16 acc = (floatx16)(0.f);
  for (int kb = 0; kb < K; kb += 8) {
    const int k = kb + 4 * half;
    float4 a, b;
    if (TA) {
      a = make_float4(A[(int64_t)(k + 0) * lda + m0 + l32], A[(int64_t)(k + 1) * lda + m0 + l32],
                      A[(int64_t)(k + 2) * lda + m0 + l32], A[(int64_t)(k + 3) * lda + m0 + l32]);
    } else {
      a = *reinterpret_cast<const float4*>(A + (int64_t)(m0 + l32) * lda + k);
    }
    if (TB) {
      b = *reinterpret_cast<const float4*>(B + (int64_t)(n0 + l32) * ldb + k);
    } else {
      b = make_float4(B[(int64_t)(k + 0) * ldb + n0 + l32], B[(int64_t)(k + 1) * ldb + n0 + l32],
                      B[(int64_t)(k + 2) * ldb + n0 + l32], B[(int64_t)(k + 3) * ldb + n0 + l32]);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f4get(a, q), f4get(b, q), acc, 0, 0, 0);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = m0 + 8 * (v / 4) + 4 * half + (v % 4);
    float* c = C + (int64_t)row * N + n0 + l32;
    *c = accumulate ? *c + acc[v] : acc[v];
  }
}

// forward gates: z = sig(az + Bz), r = sig(ar + Br), rw = r * W
__global__ void k_ev_zr(const float* az, const float* ar, const float* Bz, const float* Br, const float* W,
                        float* z, float* r, float* rw, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const float zz = sigmoidf_(az[e] + Bz[e]), rr = sigmoidf_(ar[e] + Br[e]);
  z[e] = zz; r[e] = rr; rw[e] = rr * W[e];
}

// c = tanh(ah + Bh),  W' = (1 - z) W + z c
__global__ void k_ev_out(const float* ah, const float* Bh, const float* z, const float* W, float* c, float* Wn,
                         int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const float cc = tanhf(ah[e] + Bh[e]);
  c[e] = cc;
  Wn[e] = (1.0f - z[e]) * W[e] + z[e] * cc;
}

// backward, first half of a step: G += direct gradient of W_t; gate gradients that need no GEMM
__global__ void k_ev_bwd1(float* G, const float* dWd, const float* z, const float* r, const float* c,
                          const float* Wp, float* dWp, float* dAh, float* dAz, float* rw, float* gBh, float* gBz,
                          int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const float g = G[e] + dWd[e];
  G[e] = g;
  const float zz = z[e], cc = c[e], wp = Wp[e];
  const float dz = g * (cc - wp), dc = g * zz;
  dWp[e] = g * (1.0f - zz);
  const float ah = dc * (1.0f - cc * cc), azv = dz * zz * (1.0f - zz);
  dAh[e] = ah; dAz[e] = azv;
  rw[e] = r[e] * wp;
  gBh[e] += ah; gBz[e] += azv;
}

// second half: tmp = Vh^T dAh is the gradient of (Rg * W)
__global__ void k_ev_bwd2(const float* tmp, const float* r, const float* Wp, float* dWp, float* dAr, float* gBr,
                          int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const float rr = r[e], tv = tmp[e];
  const float arv = tv * Wp[e] * rr * (1.0f - rr);
  dAr[e] = arv;
  dWp[e] += tv * rr;
  gBr[e] += arv;
}

__global__ void k_copy(float* dst, const float* src, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) dst[e] = src[e];
}

__global__ void k_fill(float* dst, float v, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) dst[e] = v;
}

// W_t [F][S] for all t -> fragment order of W_t^T [S][F] (the dense kernels take (out, in) weights)
__global__ void k_pack_weight_t(const float* Wt, int32_t T, int32_t F, int32_t S, float4* packed) {
  const int nkb = (F + 7) / 8;
  const int64_t per = (int64_t)(S / 32) * nkb * 64;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= per * T) return;
  const int64_t t = idx / per, i = idx - t * per;
  const int lane = (int)(i & 63);
  const int64_t f = i >> 6;
  const int kb = (int)(f % nkb), jb = (int)(f / nkb);
  const int out = jb * 32 + (lane & 31);      // column s of W_t
  const int k0 = kb * 8 + (lane >> 5) * 4;    // row f of W_t
  const float* W = Wt + t * (int64_t)F * S;
  float v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = (k0 + q < F) ? W[(int64_t)(k0 + q) * S + out] : 0.f;
  packed[idx] = make_float4(v[0], v[1], v[2], v[3]);
}

// ---------------------------------------------------------------------------------------------
// dW_t = sum over the rows (t, i) of the batch of M[row]^T dP[row],  dP = dL/d(pre-activation):
//   dP = [Y > 0] * dY                      (explicit upstream gradient), or
//   dP = [Y > 0] * 2 (Y - target) / count  (mean-squared-error loss, also summed into loss).
// MFMA-bound (2 F S flops per row against (F + S) floats read).  One workgroup of F/32 waves
// owns (snapshot t, split k) and walks every kSplit-th 32-row tile of that snapshot; wave w keeps
// rows [32w, 32w+32) x all S columns of the partial sum in its accumulators.  Both operands are
// row-major reads: lane l supplies A[m = l%32][k = l/32] = M[r0 + l/32][32w + l%32] and
// B[k][n] = dP[r0 + l/32][32 jb + l%32].  Tiles are staged through LDS; the next tile's global
// loads are in flight (in registers) while the current one is multiplied.
constexpr int kSplit = 8;
constexpr int kDwRows = 32;

struct DwArgs {
  const DenseTile* items;     // 32-row tiles ordered by snapshot
  const int64_t* item_ptr;    // [T+1]
  const int32_t* item_t;      // unused (kept for debugging)
  const ChunkInfo* chunks;
  int64_t N;
  const float* M; int64_t ldm;
  const float* Y; int64_t ldy;
  const float* dY; int64_t lddy;       // or nullptr
  const float* target; int64_t ldt;    // or nullptr
  float inv_count2;                    // 2 / count
  int32_t F, S;
  float* partial;                      // [T][kSplit][F][S]
  float* loss_partial;                 // [T][kSplit]
};

template <int NJB>  // S / 32
__global__ __launch_bounds__(512) void k_dw_partial(DwArgs a, int t_base) {
  extern __shared__ __align__(16) float lds[];
  const int F = a.F, S = NJB * 32;
  const int ldt_m = F + 4, ldt_p = S + 4;
  float* tm = lds;                        // [32][F+4]   M tile
  float* tp = lds + kDwRows * ldt_m;      // [32][S+4]   dP tile
  float* red = tp + kDwRows * ldt_p;      // [nthreads / 64] loss partials
  const int t = t_base + blockIdx.x / kSplit, ks = blockIdx.x % kSplit;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int nthreads = blockDim.x;
  const int fm4 = F / 4, fp4 = S / 4;
  constexpr int kMaxPf = 4;  // float4 per thread and operand: 32 rows x 256 floats / 512 threads
  floatx16 acc[NJB];
#pragma unroll
  for (int jb = 0; jb < NJB; ++jb) acc[jb] = (floatx16)(0.f);
  float loss = 0.f;
  const int64_t i0 = a.item_ptr[t], i1 = a.item_ptr[t + 1];

  float4 pm[kMaxPf], py[kMaxPf], pg[kMaxPf];
  auto fetch = [&](int64_t it) {
    const DenseTile tile = a.items[it];
    const ChunkInfo ch = a.chunks[tile.chunk];
    const float* mrow = a.M + (ch.row_off0 + (int64_t)(t - ch.t_lo) * ch.nv + tile.v0) * a.ldm;
    const int64_t vrow = (int64_t)t * a.N + ch.v_lo + tile.v0;
#pragma unroll
    for (int i = 0; i < kMaxPf; ++i) {
      const int idx = tid + i * nthreads;
      pm[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      py[i] = pm[i]; pg[i] = pm[i];
      if (idx < kDwRows * fm4) {
        const int r = idx / fm4, c4 = idx - r * fm4;
        if (r < tile.nrows) pm[i] = *reinterpret_cast<const float4*>(mrow + (int64_t)r * a.ldm + 4 * c4);
      }
      if (idx < kDwRows * fp4) {
        const int r = idx / fp4, c4 = idx - r * fp4;
        if (r < tile.nrows) {
          py[i] = *reinterpret_cast<const float4*>(a.Y + (vrow + r) * a.ldy + 4 * c4);
          pg[i] = a.target ? *reinterpret_cast<const float4*>(a.target + (vrow + r) * a.ldt + 4 * c4)
                           : *reinterpret_cast<const float4*>(a.dY + (vrow + r) * a.lddy + 4 * c4);
        }
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < kMaxPf; ++i) {
      const int idx = tid + i * nthreads;
      if (idx < kDwRows * fm4) {
        const int r = idx / fm4, c4 = idx - r * fm4;
        *reinterpret_cast<float4*>(tm + r * ldt_m + 4 * c4) = pm[i];
      }
      if (idx < kDwRows * fp4) {
        const int r = idx / fp4, c4 = idx - r * fp4;
        const float y[4] = {py[i].x, py[i].y, py[i].z, py[i].w};
        const float g[4] = {pg[i].x, pg[i].y, pg[i].z, pg[i].w};
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (a.target) {
            const float d = y[e] - g[e];
            loss += d * d;                      // rows past the tile's end hold zeros: add nothing
            o[e] = y[e] > 0.f ? d * a.inv_count2 : 0.f;
          } else {
            o[e] = y[e] > 0.f ? g[e] : 0.f;
          }
        }
        *reinterpret_cast<float4*>(tp + r * ldt_p + 4 * c4) = make_float4(o[0], o[1], o[2], o[3]);
      }
    }
  };

  int64_t it = i0 + ks;
  if (it < i1) fetch(it);
  for (; it < i1; it += kSplit) {
    __syncthreads();  // the previous tile has been consumed
    stage();
    __syncthreads();
    if (it + kSplit < i1) fetch(it + kSplit);
    const float* am = tm + half * ldt_m + wave * 32 + l32;
    const float* bp = tp + half * ldt_p + l32;
#pragma unroll 4
    for (int kk = 0; kk < kDwRows / 2; ++kk) {
      const float av = am[2 * kk * ldt_m];
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb)
        acc[jb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bp[2 * kk * ldt_p + jb * 32], acc[jb], 0, 0, 0);
    }
  }
  // partial sums: rows 32*wave .. of dW_t, standard accumulator layout (row by register, column = l%32)
  float* out = a.partial + ((int64_t)t * kSplit + ks) * (int64_t)F * S;
#pragma unroll
  for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wave * 32 + 8 * (v / 4) + 4 * half + (v % 4);
      out[(int64_t)row * S + jb * 32 + l32] = acc[jb][v];
    }
  // loss: wave sums in lane order, then the waves in order (fixed order, reproducible)
  for (int d = 32; d >= 1; d >>= 1) loss += __shfl_down(loss, d, 64);
  __syncthreads();
  if (lane == 0) red[wave] = loss;
  __syncthreads();
  if (tid == 0) {
    float s = 0.f;
    for (int w = 0; w < nthreads / 64; ++w) s += red[w];
    a.loss_partial[(int64_t)t * kSplit + ks] = s;
  }
}

// dWd[t] = sum_k partial[t][k]  (k ascending)
__global__ void k_dw_reduce(const float* partial, float* dWd, int64_t n_per_t, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int64_t t = e / n_per_t, i = e - t * n_per_t;
  float s = 0.f;
  for (int k = 0; k < kSplit; ++k) s += partial[(t * kSplit + k) * n_per_t + i];
  dWd[e] = s;
}

// loss = (sum of the partial sums, in index order) / count; one block
__global__ void k_loss_reduce(const float* loss_partial, int64_t n, float inv_count, float* loss_out) {
  __shared__ double sh[256];
  double s = 0.0;
  for (int64_t i = threadIdx.x; i < n; i += 256) s += (double)loss_partial[i];
  sh[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int i = 0; i < 256; ++i) tot += sh[i];
    *loss_out = (float)(tot * (double)inv_count);
  }
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

void gemm(bool ta, bool tb, const float* A, const float* B, float* C, int M, int N, int K, bool acc, hipStream_t st) {
  const dim3 grid(N / 32, M / 32);
  if (!ta && !tb) hipLaunchKernelGGL((k_small_gemm<false, false>), grid, 64, 0, st, A, B, C, M, N, K, (int)acc);
  if (ta && !tb) hipLaunchKernelGGL((k_small_gemm<true, false>), grid, 64, 0, st, A, B, C, M, N, K, (int)acc);
  if (!ta && tb) hipLaunchKernelGGL((k_small_gemm<false, true>), grid, 64, 0, st, A, B, C, M, N, K, (int)acc);
  if (ta && tb) hipLaunchKernelGGL((k_small_gemm<true, true>), grid, 64, 0, st, A, B, C, M, N, K, (int)acc);
}

}  // namespace

int64_t evolve_partial_elems(int32_t T, int32_t F, int32_t S) { return (int64_t)T * kSplit * F * S; }
int64_t evolve_loss_partial_elems(int32_t T) { return (int64_t)T * kSplit; }

// Evolve W_t for t = 0..T-1 (ws.Wt, gates ws.Zg/Rg/Wc) and pack every W_t for the dense kernels.
void evolve_forward_weights(const EvolveWs& ws, hipStream_t st) {
  const int F = ws.F, S = ws.S;
  const int64_t n = (int64_t)F * S;
  const unsigned nb = blocks_for(n);
  for (int t = 0; t < ws.T; ++t) {
    const float* W = t ? ws.Wt + (t - 1) * n : ws.P[EV_W];
    float *z = ws.Zg + t * n, *r = ws.Rg + t * n, *c = ws.Wc + t * n, *Wn = ws.Wt + t * n;
    gemm(false, false, ws.P[EV_UZ], W, ws.tmp0, F, S, F, false, st);
    gemm(false, false, ws.P[EV_VZ], W, ws.tmp0, F, S, F, true, st);
    gemm(false, false, ws.P[EV_UR], W, ws.tmp1, F, S, F, false, st);
    gemm(false, false, ws.P[EV_VR], W, ws.tmp1, F, S, F, true, st);
    hipLaunchKernelGGL(k_ev_zr, nb, 256, 0, st, ws.tmp0, ws.tmp1, ws.P[EV_BZ], ws.P[EV_BR], W, z, r, ws.tmp2, n);
    gemm(false, false, ws.P[EV_UH], W, ws.tmp0, F, S, F, false, st);
    gemm(false, false, ws.P[EV_VH], ws.tmp2, ws.tmp0, F, S, F, true, st);
    hipLaunchKernelGGL(k_ev_out, nb, 256, 0, st, ws.tmp0, ws.P[EV_BH], z, W, c, Wn, n);
  }
  const int64_t per = (int64_t)(S / 32) * ((F + 7) / 8) * 64;
  hipLaunchKernelGGL(k_pack_weight_t, blocks_for(per * ws.T), 256, 0, st, ws.Wt, ws.T, F, S, ws.Wt_packed);
}

// dWd[t] for all t (and the loss), from the saved aggregated rows and the layer's output.
bool evolve_backward_dw(const EvolveWs& ws, const EvolveBwdIn& in, hipStream_t st, std::string* why) {
  DwArgs a{};
  a.items = ws.items; a.item_ptr = ws.item_ptr; a.item_t = nullptr; a.chunks = in.chunks; a.N = in.N;
  a.M = in.M; a.ldm = in.ldm; a.Y = in.Y; a.ldy = in.ldy; a.dY = in.dY; a.lddy = in.lddy;
  a.target = in.target; a.ldt = in.ldt;
  a.inv_count2 = 2.0f / (float)in.count;
  a.F = ws.F; a.S = ws.S; a.partial = ws.partial; a.loss_partial = ws.loss_partial;
  const int threads = 64 * (ws.F / 32);
  if (ws.F % 32 || ws.F > 256 || ws.S % 32 || ws.S > 256) {
    if (why) *why = "the weight-gradient kernel needs F and S multiples of 32, at most 256";
    return false;
  }
  const size_t lds = sizeof(float) * ((size_t)kDwRows * (ws.F + 4) + (size_t)kDwRows * (ws.S + 4) + 16);
  const unsigned grid = (unsigned)ws.T * kSplit;
  switch (ws.S / 32) {
#define DGC_DW_CASE(NJB)                                                                               \
  case NJB: {                                                                                          \
    static bool attr = false;                                                                          \
    if (!attr) {                                                                                       \
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dw_partial<NJB>),                       \
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) { \
        if (why) *why = "hipFuncSetAttribute failed";                                                  \
        return false;                                                                                  \
      }                                                                                                \
      attr = true;                                                                                     \
    }                                                                                                  \
    hipLaunchKernelGGL((k_dw_partial<NJB>), grid, threads, lds, st, a, 0);                             \
    break;                                                                                             \
  }
    DGC_DW_CASE(1) DGC_DW_CASE(2) DGC_DW_CASE(3) DGC_DW_CASE(4) DGC_DW_CASE(5) DGC_DW_CASE(6) DGC_DW_CASE(7)
    DGC_DW_CASE(8)
#undef DGC_DW_CASE
    default:
      if (why) *why = "unsupported S";
      return false;
  }
  const int64_t n = (int64_t)ws.F * ws.S;
  hipLaunchKernelGGL(k_dw_reduce, blocks_for(n * ws.T), 256, 0, st, ws.partial, ws.dWd, n, n * ws.T);
  if (in.target && in.loss_out)
    hipLaunchKernelGGL(k_loss_reduce, 1, 256, 0, st, ws.loss_partial, (int64_t)ws.T * kSplit, 1.0f / (float)in.count,
                       in.loss_out);
  return true;
}

// Back-propagation through time over the weight recurrence: fills ws.G[k] for the ten parameters.
void evolve_backward_bptt(const EvolveWs& ws, hipStream_t st) {
  const int F = ws.F, S = ws.S;
  const int64_t n = (int64_t)F * S, nff = (int64_t)F * F;
  const unsigned nb = blocks_for(n);
  for (int k = 0; k < EV_NPAR; ++k) {
    const int64_t sz = (k == EV_W || k == EV_BZ || k == EV_BR || k == EV_BH) ? n : nff;
    hipLaunchKernelGGL(k_fill, blocks_for(sz), 256, 0, st, ws.G[k], 0.f, sz);
  }
  float* Gt = ws.G[EV_W];  // running dL/dW_t; ends as the gradient of W_init
  for (int t = ws.T - 1; t >= 0; --t) {
    const float* Wp = t ? ws.Wt + (t - 1) * n : ws.P[EV_W];
    const float *z = ws.Zg + t * n, *r = ws.Rg + t * n, *c = ws.Wc + t * n;
    float *dWp = ws.tmp0, *dAh = ws.tmp1, *dAz = ws.tmp2, *rw = ws.tmp3, *tmp = ws.tmp4, *dAr = ws.tmp5;
    hipLaunchKernelGGL(k_ev_bwd1, nb, 256, 0, st, Gt, ws.dWd + t * n, z, r, c, Wp, dWp, dAh, dAz, rw, ws.G[EV_BH],
                       ws.G[EV_BZ], n);
    gemm(false, true, dAh, Wp, ws.G[EV_UH], F, F, S, true, st);    // dUh += dAh Wp^T
    gemm(false, true, dAh, rw, ws.G[EV_VH], F, F, S, true, st);    // dVh += dAh (Rg*Wp)^T
    gemm(true, false, ws.P[EV_VH], dAh, tmp, F, S, F, false, st);  // Vh^T dAh
    hipLaunchKernelGGL(k_ev_bwd2, nb, 256, 0, st, tmp, r, Wp, dWp, dAr, ws.G[EV_BR], n);
    gemm(true, false, ws.P[EV_UH], dAh, dWp, F, S, F, true, st);
    gemm(false, true, dAz, Wp, ws.G[EV_UZ], F, F, S, true, st);    // dUz += dAz Wp^T  (= dVz)
    gemm(false, true, dAr, Wp, ws.G[EV_UR], F, F, S, true, st);    // dUr += dAr Wp^T  (= dVr)
    gemm(true, false, ws.P[EV_UZ], dAz, dWp, F, S, F, true, st);
    gemm(true, false, ws.P[EV_VZ], dAz, dWp, F, S, F, true, st);
    gemm(true, false, ws.P[EV_UR], dAr, dWp, F, S, F, true, st);
    gemm(true, false, ws.P[EV_VR], dAr, dWp, F, S, F, true, st);
    hipLaunchKernelGGL(k_copy, nb, 256, 0, st, Gt, dWp, n);
  }
  // the input of the GRU is the state itself, so Uz, Vz (and Ur, Vr) receive identical gradients
  hipLaunchKernelGGL(k_copy, blocks_for(nff), 256, 0, st, ws.G[EV_VZ], ws.G[EV_UZ], nff);
  hipLaunchKernelGGL(k_copy, blocks_for(nff), 256, 0, st, ws.G[EV_VR], ws.G[EV_UR], nff);
}

}  // namespace dgc
