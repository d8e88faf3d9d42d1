// EvolveGCN-O support (the paper lists EvolveGCN among its DGNNs, Section 1; the "-O" variant of
// the cited work is used): the GCN weight matrix W [F][S] is the state of a matrix GRU,
//     Zg = sig(Uz W + Vz W + Bz)   Rg = sig(Ur W + Vr W + Br)
//     Wc = tanh(Uh W + Vh (Rg*W) + Bh)      W' = (1 - Zg)*W + Zg*Wc
// evolved once per snapshot over all T snapshots (global, independent of the chunk windows),
// Y[t,i] = relu(M[t,i] W_t), mean-squared-error loss, gradients of all ten parameter matrices.
//
// Kernels here: a double-precision MFMA kernel that fuses the small (F x F)(F x S) products of
// one step of the weight recurrence, or of its back-propagation through time, with the gate
// arithmetic that follows them (latency-bound), and the one large kernel of the backward pass,
// dW_t = M_t^T dP_t reduced over all rows of snapshot t across the fused chunks.
#include "dgc_internal.h"

namespace dgc {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float f4get(const float4& v, int q) { return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w; }
__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

// ---------------------------------------------------------------------------------------------
// The weight recurrence and its back-propagation through time run in DOUBLE precision: W is the
// state of a 64-step recurrence whose rounding errors feed every output row of every snapshot,
// and the work is tiny (a handful of n x n x n products per step, n = F = S <= 256), so it is
// latency-bound whatever the precision.  One kernel does every matrix step:
//   tile(C) = [C +] sum_p op(A_p) op(B_p)   followed by an elementwise epilogue,
// on v_mfma_f64_16x16x4f64 (lane l supplies A[l%16][l/16], B[l/16][l%16]; receives
// D[4*v + l/16][l%16], v = 0..3).  A workgroup of 4 waves owns one 16 x 16 tile; the waves
// split K and wave 0 adds their partial tiles in wave order (reproducible) and applies the
// epilogue.  grid.z selects one of several independent jobs of a launch.
typedef double doublex4 __attribute__((ext_vector_type(4)));

struct EvProd { const double* A; const double* B; int ta, tb; };  // ta: A stored [K][M]; tb: B stored [N][K]
enum { EPI_ADD = 0, EPI_ZR = 1, EPI_OUT = 2, EPI_BWD2 = 3, EPI_G = 4 };
struct EvJob {
  EvProd p[5];
  int np;
  double* C;           // EPI_ADD: C += sum
  // operands of the epilogues (see k_ev_mm)
  const double* bias;  // ZR, OUT: gate bias
  const double* W;     // ZR, OUT, BWD2: previous weights
  const double* z;     // OUT: update gate      BWD2: reset gate r
  double* o0;          // ZR: gate out          OUT: Wc      BWD2: dAr     G: running gradient G
  double* o1;          // ZR(r job): Rg*W       OUT: W_t     BWD2: dWp (+=)   G: dWp (read)
  float* o2;           // OUT: W_t in fp32 (for the dense kernels)
  double* o3;          // BWD2: gradient of B_r (+=)
  int write_rw;        // ZR: this is the r job
};
struct EvJobs { EvJob j[4]; };

__device__ __forceinline__ double sigmoidd(double x) { return 1.0 / (1.0 + exp(-x)); }

template <int EPI>
__global__ __launch_bounds__(256) void k_ev_mm(EvJobs jobs, int n) {
  __shared__ double part[4][64][4];
  const EvJob& J = jobs.j[blockIdx.z];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, kq = lane >> 4;
  const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
  const int kspan = n / 4;  // K = n, a quarter per wave; n is a multiple of 32
  doublex4 acc = {0.0, 0.0, 0.0, 0.0};
  for (int p = 0; p < J.np; ++p) {
    const int ak = J.p[p].ta ? n : 1, am = J.p[p].ta ? 1 : n;   // strides of A along k and m
    const int bk = J.p[p].tb ? 1 : n, bn = J.p[p].tb ? n : 1;
    const int k0 = wave * kspan + kq;
    const double* A = J.p[p].A + (int64_t)(m0 + l16) * am + (int64_t)k0 * ak;
    const double* B = J.p[p].B + (int64_t)(n0 + l16) * bn + (int64_t)k0 * bk;
    for (int k = 0; k < kspan; k += 8) {   // kspan is a multiple of 8
      const double a0 = A[(int64_t)k * ak], a1 = A[(int64_t)(k + 4) * ak];
      const double b0 = B[(int64_t)k * bk], b1 = B[(int64_t)(k + 4) * bk];
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc, 0, 0, 0);
    }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) part[wave][lane][v] = acc[v];
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const double sum = ((part[0][lane][v] + part[1][lane][v]) + part[2][lane][v]) + part[3][lane][v];
    const int64_t e = (int64_t)(m0 + 4 * v + kq) * n + n0 + l16;
    if (EPI == EPI_ADD) {
      J.C[e] += sum;
    } else if (EPI == EPI_ZR) {
      const double g = sigmoidd(sum + J.bias[e]);
      J.o0[e] = g;
      if (J.write_rw) J.o1[e] = g * J.W[e];
    } else if (EPI == EPI_OUT) {
      const double c = tanh(sum + J.bias[e]);
      const double zz = J.z[e];
      const double wn = (1.0 - zz) * J.W[e] + zz * c;
      J.o0[e] = c;
      J.o1[e] = wn;
      J.o2[e] = (float)wn;
    } else if (EPI == EPI_BWD2) {   // sum = Vh^T dAh = gradient of (Rg * W)
      const double rr = J.z[e];
      const double dar = sum * J.W[e] * rr * (1.0 - rr);
      J.o0[e] = dar;
      J.o1[e] += sum * rr;
      J.o3[e] += dar;
    } else {                        // EPI_G: G_{t-1} = dWp + sum
      J.o0[e] = J.o1[e] + sum;
    }
  }
}

// backward, first elementwise half of a step
__global__ void k_ev_bwd1(double* G, const float* dWd, const double* z, const double* r, const double* c,
                          const double* Wp, double* dWp, double* dAh, double* dAz, double* rw, double* gBh,
                          double* gBz, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const double g = G[e] + (double)dWd[e];
  const double zz = z[e], cc = c[e], wp = Wp[e];
  const double dz = g * (cc - wp), dc = g * zz;
  dWp[e] = g * (1.0 - zz);
  const double ah = dc * (1.0 - cc * cc), azv = dz * zz * (1.0 - zz);
  dAh[e] = ah; dAz[e] = azv;
  rw[e] = r[e] * wp;
  gBh[e] += ah; gBz[e] += azv;
}

__global__ void k_to_double(double* dst, const float* src, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) dst[e] = (double)src[e];
}
__global__ void k_to_float(float* dst, const double* src, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) dst[e] = (float)src[e];
}
__global__ void k_fill_d(double* dst, double v, int64_t n) {
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

// W_t [F][S] for all t -> fragment order of W_t itself as an (out = F, in = S) weight: the dense
// kernel then computes dM = dP W_t^T
__global__ void k_pack_weight_plain(const float* Wt, int32_t T, int32_t F, int32_t S, float4* packed) {
  const int nkb = (S + 7) / 8;
  const int64_t per = (int64_t)(F / 32) * nkb * 64;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= per * T) return;
  const int64_t t = idx / per, i = idx - t * per;
  const int lane = (int)(i & 63);
  const int64_t fr = i >> 6;
  const int kb = (int)(fr % nkb), jb = (int)(fr / nkb);
  const int out = jb * 32 + (lane & 31);      // row f of W_t
  const int k0 = kb * 8 + (lane >> 5) * 4;    // column s of W_t
  const float* W = Wt + t * (int64_t)F * S + (int64_t)out * S;
  float v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = (k0 + q < S) ? W[k0 + q] : 0.f;
  packed[idx] = make_float4(v[0], v[1], v[2], v[3]);
}

// dP of every covered row, written to the packed row of (chunk, snapshot, vertex); one thread per float4
__global__ void k_ev_dp(EvolveBwdIn in, int32_t S, float inv_count2, float* dP, int64_t ldp) {
  const ChunkInfo ch = in.chunks[blockIdx.z];
  const int32_t s = blockIdx.y;
  if (s >= ch.w) return;
  const int64_t q = S / 4;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= ch.nv * q) return;
  const int64_t v = idx / q, c4 = idx - v * q;
  const int64_t row = (int64_t)(ch.t_lo + s) * in.N + ch.v_lo + v;
  const float4 y = *reinterpret_cast<const float4*>(in.Y + row * in.ldy + 4 * c4);
  const float4 g = in.target ? *reinterpret_cast<const float4*>(in.target + row * in.ldt + 4 * c4)
                             : *reinterpret_cast<const float4*>(in.dY + row * in.lddy + 4 * c4);
  const float yy[4] = {y.x, y.y, y.z, y.w}, gg[4] = {g.x, g.y, g.z, g.w};
  float o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
    o[e] = yy[e] > 0.f ? (in.target ? (yy[e] - gg[e]) * inv_count2 : gg[e]) : 0.f;
  *reinterpret_cast<float4*>(dP + (ch.row_off0 + (int64_t)s * ch.nv + v) * ldp + 4 * c4) = make_float4(o[0], o[1], o[2], o[3]);
}

__global__ void k_ev_row_index(const ChunkInfo* chunks, int64_t N, int64_t* idx) {
  const ChunkInfo ch = chunks[blockIdx.z];
  const int32_t s = blockIdx.y;
  const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= ch.w || v >= ch.nv) return;
  idx[ch.row_off0 + (int64_t)s * ch.nv + v] = (int64_t)(ch.t_lo + s) * N + ch.v_lo + v;
}

template <int EPI>
void launch_mm(const EvJobs& jobs, int n_jobs, int n, hipStream_t st) {
  hipLaunchKernelGGL((k_ev_mm<EPI>), dim3(n / 16, n / 16, n_jobs), 256, 0, st, jobs, n);
}

}  // namespace

int64_t evolve_partial_elems(int32_t T, int32_t F, int32_t S) { return (int64_t)T * kSplit * F * S; }
int64_t evolve_loss_partial_elems(int32_t T) { return (int64_t)T * kSplit; }

// Evolve W_t for t = 0..T-1 (ws.Wt, gates ws.Zg/Rg/Wc, all double) and pack every W_t, rounded
// to fp32, for the dense kernels.  Two launches per snapshot.
void evolve_forward_weights(const EvolveWs& ws, hipStream_t st) {
  const int n = ws.F;
  const int64_t nn = (int64_t)n * n;
  for (int k = 0; k < EV_NPAR; ++k) hipLaunchKernelGGL(k_to_double, blocks_for(nn), 256, 0, st, ws.Pd[k], ws.P[k], nn);
  for (int t = 0; t < ws.T; ++t) {
    const double* W = t ? ws.Wt + (t - 1) * nn : ws.Pd[EV_W];
    double *z = ws.Zg + t * nn, *r = ws.Rg + t * nn, *c = ws.Wc + t * nn, *Wn = ws.Wt + t * nn;
    EvJobs zr{};
    zr.j[0].p[0] = {ws.Pd[EV_UZ], W, 0, 0}; zr.j[0].p[1] = {ws.Pd[EV_VZ], W, 0, 0}; zr.j[0].np = 2;
    zr.j[0].bias = ws.Pd[EV_BZ]; zr.j[0].W = W; zr.j[0].o0 = z; zr.j[0].write_rw = 0;
    zr.j[1].p[0] = {ws.Pd[EV_UR], W, 0, 0}; zr.j[1].p[1] = {ws.Pd[EV_VR], W, 0, 0}; zr.j[1].np = 2;
    zr.j[1].bias = ws.Pd[EV_BR]; zr.j[1].W = W; zr.j[1].o0 = r; zr.j[1].o1 = ws.tmp[2]; zr.j[1].write_rw = 1;
    launch_mm<EPI_ZR>(zr, 2, n, st);
    EvJobs out{};
    out.j[0].p[0] = {ws.Pd[EV_UH], W, 0, 0}; out.j[0].p[1] = {ws.Pd[EV_VH], ws.tmp[2], 0, 0}; out.j[0].np = 2;
    out.j[0].bias = ws.Pd[EV_BH]; out.j[0].W = W; out.j[0].z = z; out.j[0].o0 = c; out.j[0].o1 = Wn;
    out.j[0].o2 = ws.Wt_f32 + t * nn;
    launch_mm<EPI_OUT>(out, 1, n, st);
  }
  const int64_t per = (int64_t)(ws.S / 32) * ((ws.F + 7) / 8) * 64;
  hipLaunchKernelGGL(k_pack_weight_t, blocks_for(per * ws.T), 256, 0, st, ws.Wt_f32, ws.T, ws.F, ws.S, ws.Wt_packed);
}

void evolve_backward_dp(const EvolveBwdIn& in, int32_t n_chunks, int64_t max_nv, int32_t max_w, int32_t S, float* dP,
                        int64_t ldp, hipStream_t st) {
  hipLaunchKernelGGL(k_ev_dp, dim3(blocks_for(max_nv * (S / 4)), (unsigned)max_w, (unsigned)n_chunks), 256, 0, st, in, S,
                     2.0f / (float)in.count, dP, ldp);
}

void evolve_row_index(const ChunkInfo* chunks, int32_t n_chunks, int64_t max_nv, int32_t max_w, int64_t N, int64_t* idx,
                      hipStream_t st) {
  hipLaunchKernelGGL(k_ev_row_index, dim3(blocks_for(max_nv), (unsigned)max_w, (unsigned)n_chunks), 256, 0, st, chunks, N,
                     idx);
}

void evolve_pack_weights_plain(const EvolveWs& ws, float4* packed, hipStream_t st) {
  const int64_t per = (int64_t)(ws.F / 32) * ((ws.S + 7) / 8) * 64;
  hipLaunchKernelGGL(k_pack_weight_plain, blocks_for(per * ws.T), 256, 0, st, ws.Wt_f32, ws.T, ws.F, ws.S, packed);
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

// Back-propagation through time over the weight recurrence (double precision, four launches
// per snapshot); the gradients of the ten parameters end up in ws.G[k] as fp32.
void evolve_backward_bptt(const EvolveWs& ws, hipStream_t st) {
  const int n = ws.F;
  const int64_t nn = (int64_t)n * n;
  const unsigned nb = blocks_for(nn);
  for (int k = 0; k < EV_NPAR; ++k) hipLaunchKernelGGL(k_fill_d, nb, 256, 0, st, ws.Gd[k], 0.0, nn);
  double* Gt = ws.Gd[EV_W];  // running dL/dW_t; ends as the gradient of W_init
  double *dWp = ws.tmp[0], *dAh = ws.tmp[1], *dAz = ws.tmp[2], *rw = ws.tmp[3], *dAr = ws.tmp[5];
  for (int t = ws.T - 1; t >= 0; --t) {
    const double* Wp = t ? ws.Wt + (t - 1) * nn : ws.Pd[EV_W];
    const double *z = ws.Zg + t * nn, *r = ws.Rg + t * nn, *c = ws.Wc + t * nn;
    hipLaunchKernelGGL(k_ev_bwd1, nb, 256, 0, st, Gt, ws.dWd + t * nn, z, r, c, Wp, dWp, dAh, dAz, rw, ws.Gd[EV_BH],
                       ws.Gd[EV_BZ], nn);
    EvJobs b2{};   // Vh^T dAh -> dAr, dWp += ., dB_r += .
    b2.j[0].p[0] = {ws.Pd[EV_VH], dAh, 1, 0}; b2.j[0].np = 1;
    b2.j[0].W = Wp; b2.j[0].z = r; b2.j[0].o0 = dAr; b2.j[0].o1 = dWp; b2.j[0].o3 = ws.Gd[EV_BR];
    launch_mm<EPI_BWD2>(b2, 1, n, st);
    EvJobs gr{};   // dUh += dAh Wp^T, dVh += dAh (Rg*Wp)^T, dUz += dAz Wp^T, dUr += dAr Wp^T
    gr.j[0].p[0] = {dAh, Wp, 0, 1}; gr.j[0].np = 1; gr.j[0].C = ws.Gd[EV_UH];
    gr.j[1].p[0] = {dAh, rw, 0, 1}; gr.j[1].np = 1; gr.j[1].C = ws.Gd[EV_VH];
    gr.j[2].p[0] = {dAz, Wp, 0, 1}; gr.j[2].np = 1; gr.j[2].C = ws.Gd[EV_UZ];
    gr.j[3].p[0] = {dAr, Wp, 0, 1}; gr.j[3].np = 1; gr.j[3].C = ws.Gd[EV_UR];
    launch_mm<EPI_ADD>(gr, 4, n, st);
    EvJobs g{};    // G_{t-1} = dWp + Uh^T dAh + (Uz + Vz)^T dAz + (Ur + Vr)^T dAr
    g.j[0].p[0] = {ws.Pd[EV_UH], dAh, 1, 0}; g.j[0].p[1] = {ws.Pd[EV_UZ], dAz, 1, 0};
    g.j[0].p[2] = {ws.Pd[EV_VZ], dAz, 1, 0}; g.j[0].p[3] = {ws.Pd[EV_UR], dAr, 1, 0};
    g.j[0].p[4] = {ws.Pd[EV_VR], dAr, 1, 0}; g.j[0].np = 5;
    g.j[0].o0 = Gt; g.j[0].o1 = dWp;
    launch_mm<EPI_G>(g, 1, n, st);
  }
  // the input of the GRU is the state itself, so Uz, Vz (and Ur, Vr) receive identical gradients
  for (int k = 0; k < EV_NPAR; ++k) {
    const double* src = k == EV_VZ ? ws.Gd[EV_UZ] : k == EV_VR ? ws.Gd[EV_UR] : ws.Gd[k];
    hipLaunchKernelGGL(k_to_float, nb, 256, 0, st, ws.G[k], src, nn);
  }
}

}  // namespace dgc
