// Graph-attention + causal temporal self-attention layer, bf16: backward pass (gradients of the
// seven parameter tensors; the cache is a constant and input gradients are not produced).
//
// Stages: (1) temporal attention backward per 2-vertex tile (recomputes P, Q, K, V and the
// probabilities; writes dU, dQ, dK, dV and the position-table gradient), (2) dW_q, dW_k, dW_v as
// products over all rows, (3) graph attention row pass (gradients of the destination logits),
// (4) reverse-edge pass (gradients of both projections of every vertex, of a_src and a_dst),
// (5) dW of the projection from the input and the cache rows.  Every reduction over rows goes
// through per-wave (per-workgroup) slots that are added in slot order: no floating-point atomics.
#include "dgc_dysat_dev.h"

namespace dgc {
using namespace dysat;
namespace {

__global__ void k_fill_f32(float* p, float v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

struct TemporalBwdArgs {
  const ChunkInfo* chunks; int32_t n_chunks;
  const int64_t* tile_ptr; int64_t n_tiles;
  int64_t N; int32_t T;
  const float* U; const float* pos;
  const uint4 *Wq, *Wk, *Wv;       // row-operand fragments
  const uint4 *WqT, *WkT, *WvT;    // fragments of the transposes
  const uint16_t* Y; int64_t ldy;          // with target: dY = scale * (Y - target)
  const uint16_t* dY; int64_t lddy;        // or the upstream gradient itself
  const uint16_t* target; int64_t ldt;
  float scale;
  uint16_t *dU, *dQ, *dK, *dV;
  float* dpos_partial;   // [n_waves][T][128], zero on entry
  float* loss_partial;   // [n_waves]
  int32_t n_waves;
};

// upstream gradient of n consecutive features (n = 8 or 4) of one row; adds (Y - target)^2 to *sq
template <int NV>
__device__ __forceinline__ void load_dy(const TemporalBwdArgs& a, int64_t row, int off, bool valid, float* out, float* sq) {
  if (!valid) {
#pragma unroll
    for (int i = 0; i < NV; ++i) out[i] = 0.f;
    return;
  }
  float y[8], g[8];
  if (a.dY) {
    if (NV == 8) unpack8(*reinterpret_cast<const uint4*>(a.dY + row * a.lddy + off), out);
    else {
      const uint2 u = *reinterpret_cast<const uint2*>(a.dY + row * a.lddy + off);
      out[0] = bf_lo(u.x); out[1] = bf_hi(u.x); out[2] = bf_lo(u.y); out[3] = bf_hi(u.y);
    }
    return;
  }
  if (NV == 8) {
    unpack8(*reinterpret_cast<const uint4*>(a.Y + row * a.ldy + off), y);
    unpack8(*reinterpret_cast<const uint4*>(a.target + row * a.ldt + off), g);
  } else {
    const uint2 u = *reinterpret_cast<const uint2*>(a.Y + row * a.ldy + off);
    const uint2 w = *reinterpret_cast<const uint2*>(a.target + row * a.ldt + off);
    y[0] = bf_lo(u.x); y[1] = bf_hi(u.x); y[2] = bf_lo(u.y); y[3] = bf_hi(u.y);
    g[0] = bf_lo(w.x); g[1] = bf_hi(w.x); g[2] = bf_lo(w.y); g[3] = bf_hi(w.y);
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const float d = y[i] - g[i];
    out[i] = a.scale * d;
    if (sq) *sq += d * d;
  }
}

__device__ __forceinline__ void flush_dpos(float* slot, int t_lo, int T, int lane, floatx16* acc) {
  const int n = lane & 31, hh = lane >> 5, s = n & 15;
#pragma unroll
  for (int ib = 0; ib < 4; ++ib) {
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[ib][v] += __shfl_xor(acc[ib][v], 16);   // the two vertices of the tile
    if (n < 16 && t_lo + s < T) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4* p = reinterpret_cast<float4*>(slot + (int64_t)(t_lo + s) * kS + ib * 32 + 8 * g + 4 * hh);
        float4 o = *p;
        o.x += acc[ib][4 * g]; o.y += acc[ib][4 * g + 1]; o.z += acc[ib][4 * g + 2]; o.w += acc[ib][4 * g + 3];
        *p = o;
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[ib][v] = 0.f;
  }
}

// Temporal self-attention, backward.  One wavefront (= one workgroup) walks a contiguous range
// of 2-vertex tiles.  Per tile it recomputes P, Q, K, V (Q, K also in column layout), then per
// head the score block in both orientations: "query-major" (lane = query row, registers = key
// steps) gives the softmax statistics, delta = sum_r p dp and dS for dQ; "key-major" (lane = key
// row, registers = query steps; statistics of the query rows come through LDS) gives p and dS
// for dV and dK.  dQ, dK, dV land in row layout, are stored (bf16) for the weight-gradient
// kernel and feed, as B operands, the products with the transposed weights that give dP.
// dU = dP * ELU'(U); the column sums of dP per snapshot (gradient of the position table) are
// kept in registers and flushed to the wave's own slot when the window start changes.
__global__ __launch_bounds__(64) void k_temporal_bwd(TemporalBwdArgs a) {
  __shared__ float sh[2][32];
  const int lane = threadIdx.x;
  const int hh = lane >> 5, f = lane & 31, n = lane & 31;
  const int64_t per = (a.n_tiles + a.n_waves - 1) / a.n_waves;
  const int64_t tile0 = (int64_t)blockIdx.x * per, tile1 = min(a.n_tiles, tile0 + per);
  floatx16 dpos[4] = {};
  int cur_tlo = -1;
  float sq = 0.f;
  const bf16x8 zero8 = {};
  const bf16x8 sel0 = sel_frag(0, lane), sel1 = sel_frag(1, lane);
  float* slot = a.dpos_partial + (int64_t)blockIdx.x * a.T * kS;
  for (int64_t tile = tile0; tile < tile1; ++tile) {
    const TileRow r = tile_row(a.chunks, a.n_chunks, a.tile_ptr, tile, a.N, lane);
    if (r.t_lo != cur_tlo) {
      if (cur_tlo >= 0) flush_dpos(slot, cur_tlo, a.T, lane, dpos);
      cur_tlo = r.t_lo;
    }
    bf16x8 pf[8], pl[8];
    load_p_frags<true>(a.U, a.pos, r, hh, pf, pl);
    floatx16 dP[4] = {};
#pragma unroll 1
    for (int jb = 0; jb < 4; ++jb) {
      floatx16 q = {}, k = {}, v = {}, qt = {}, kt = {}, dyt = {};
#pragma unroll
      for (int kb = 0; kb < 8; ++kb) {
        const int fi = (jb * 8 + kb) * 64 + lane;
        const bf16x8 wq = as_frag(a.Wq[fi]), wk = as_frag(a.Wk[fi]), wv = as_frag(a.Wv[fi]);
        q = mfma2b(wq, pf[kb], pl[kb], q);
        k = mfma2b(wk, pf[kb], pl[kb], k);
        v = mfma2b(wv, pf[kb], pl[kb], v);
        qt = mfma2a(pf[kb], pl[kb], wq, qt);
        kt = mfma2a(pf[kb], pl[kb], wk, kt);
      }
      {
        float d8[8];
        bf16x8 dh, dl;
        load_dy<8>(a, r.row, (2 * jb) * 16 + 8 * hh, r.valid, d8, &sq);
        split8(d8, dh, dl);
        dyt = mfma2a(dh, dl, sel0, dyt);
        load_dy<8>(a, r.row, (2 * jb + 1) * 16 + 8 * hh, r.valid, d8, &sq);
        split8(d8, dh, dl);
        dyt = mfma2a(dh, dl, sel1, dyt);
      }
      floatx16 dq = {}, dk = {}, dv = {};
#pragma unroll
      for (int hd = 0; hd < 2; ++hd) {
        bf16x8 kh, kl, qh, ql, vh, vl, dyh, dyl;
        split8v(k, 8 * hd, kh, kl);
        split8v(q, 8 * hd, qh, ql);
        split8v(v, 8 * hd, vh, vl);
        float d8[8];
        load_dy<4>(a, r.row, jb * 32 + 16 * hd + 4 * hh, r.valid, d8, nullptr);
        load_dy<4>(a, r.row, jb * 32 + 16 * hd + 8 + 4 * hh, r.valid, d8 + 4, nullptr);
        split8(d8, dyh, dyl);
        floatx16 st = {}, dpt = {};
        st = mfma3(kh, kl, qh, ql, st);         // [key row][query row]
        dpt = mfma3(vh, vl, dyh, dyl, dpt);
        float pr[8], dst[8];
        float mx = -INFINITY;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const int rk = 8 * (p >> 2) + 4 * hh + (p & 3);
          pr[p] = rk <= r.s ? 0.25f * (r.a ? st[8 + p] : st[p]) : -INFINITY;
          mx = fmaxf(mx, pr[p]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float sum = 0.f;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          pr[p] = __expf(pr[p] - mx);
          sum += pr[p];
        }
        sum += __shfl_xor(sum, 32);
        const float inv = 1.f / sum;
        float delta = 0.f;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          pr[p] *= inv;
          dst[p] = r.a ? dpt[8 + p] : dpt[p];
          delta += pr[p] * dst[p];
        }
        delta += __shfl_xor(delta, 32);
#pragma unroll
        for (int p = 0; p < 8; ++p) dst[p] = 0.25f * pr[p] * (dst[p] - delta);
        if (hh == 0) {
          sh[0][n] = mx + __logf(sum);
          sh[1][n] = delta;
        }
        __syncthreads();
        floatx16 s2 = {}, dp2 = {};
        s2 = mfma3(qh, ql, kh, kl, s2);         // [query row][key row]
        dp2 = mfma3(dyh, dyl, vh, vl, dp2);
        float p2[8], ds2[8];
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const int sq_ = 8 * (p >> 2) + 4 * hh + (p & 3);    // query step of this register
          const float lse = sh[0][16 * r.a + sq_], dl = sh[1][16 * r.a + sq_];
          const float x = 0.25f * (r.a ? s2[8 + p] : s2[p]);
          p2[p] = r.s <= sq_ ? __expf(x - lse) : 0.f;
          ds2[p] = 0.25f * p2[p] * ((r.a ? dp2[8 + p] : dp2[p]) - dl);
        }
        __syncthreads();
        bf16x8 dsth, dstl, ds2h, ds2l, p2h, p2l;
        split8(dst, dsth, dstl);
        split8(ds2, ds2h, ds2l);
        split8(p2, p2h, p2l);
        const bool mine = (f >> 4) == hd;
#pragma unroll
        for (int av = 0; av < 2; ++av) {
          const bool myv = r.a == av;
          bf16x8 ah, al;
          split8v(kt, 8 * av, ah, al);
          dq = mfma3(mine ? ah : zero8, mine ? al : zero8, myv ? dsth : zero8, myv ? dstl : zero8, dq);
          split8v(qt, 8 * av, ah, al);
          dk = mfma3(mine ? ah : zero8, mine ? al : zero8, myv ? ds2h : zero8, myv ? ds2l : zero8, dk);
          split8v(dyt, 8 * av, ah, al);
          dv = mfma3(mine ? ah : zero8, mine ? al : zero8, myv ? p2h : zero8, myv ? p2l : zero8, dv);
        }
      }
      if (r.valid) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int64_t o = r.row * kS + jb * 32 + 8 * g + 4 * hh;
          *reinterpret_cast<uint2*>(a.dQ + o) = pack4(dq[4 * g], dq[4 * g + 1], dq[4 * g + 2], dq[4 * g + 3]);
          *reinterpret_cast<uint2*>(a.dK + o) = pack4(dk[4 * g], dk[4 * g + 1], dk[4 * g + 2], dk[4 * g + 3]);
          *reinterpret_cast<uint2*>(a.dV + o) = pack4(dv[4 * g], dv[4 * g + 1], dv[4 * g + 2], dv[4 * g + 3]);
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int ks = 2 * jb + c;
        bf16x8 bqh, bql, bkh, bkl, bvh, bvl;
        split8v(dq, 8 * c, bqh, bql);
        split8v(dk, 8 * c, bkh, bkl);
        split8v(dv, 8 * c, bvh, bvl);
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) {
          const int fi = (ib * 8 + ks) * 64 + lane;
          dP[ib] = mfma2b(as_frag(a.WqT[fi]), bqh, bql, dP[ib]);
          dP[ib] = mfma2b(as_frag(a.WkT[fi]), bkh, bkl, dP[ib]);
          dP[ib] = mfma2b(as_frag(a.WvT[fi]), bvh, bvl, dP[ib]);
        }
      }
    }
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
      if (r.valid) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int64_t o = r.row * kS + ib * 32 + 8 * g + 4 * hh;
          const float4 u = *reinterpret_cast<const float4*>(a.U + o);
          *reinterpret_cast<uint2*>(a.dU + o) = pack4(dP[ib][4 * g] * delu(u.x), dP[ib][4 * g + 1] * delu(u.y),
                                                     dP[ib][4 * g + 2] * delu(u.z), dP[ib][4 * g + 3] * delu(u.w));
        }
      }
      dpos[ib] += dP[ib];
    }
  }
  if (cur_tlo >= 0) flush_dpos(slot, cur_tlo, a.T, lane, dpos);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
  if (lane == 0) a.loss_partial[blockIdx.x] = sq;
}

// ---------------------------------------------------------------------------------------------
// Weight gradients  dW_G[out][in] = sum over rows of G[row][out] * A[row][in]  for NG tensors G
// sharing one A (A = the rows of a bf16 tensor, or P = ELU(U) + pos recomputed from U).  Rows are
// the vertices of the snapshots in use, 32 per tile.  A workgroup of 4 waves walks a contiguous
// range of tiles; wave w owns output rows [32w, 32w+32) of every dW_G.  Both operands need the
// row index as contraction index, i.e. column layout: obtained from natural row fragments with
// the selection products described above.
struct DwBf16Args {
  const int32_t* used_t; int32_t n_used; int64_t N;
  const int32_t* owner; int32_t covered_only;
  const uint16_t* A; int64_t lda;        // bf16 rows, or
  const float* Uf; const float* pos;     // A = ELU(Uf) + pos (fp32 rows of pitch 128), carried as hi + lo
  const uint16_t* G[3];
  float* partial;      // [n_groups][NG][128][128]
  int32_t n_groups;
};

template <int NG, bool AU>
__global__ __launch_bounds__(256) void k_dw_bf16(DwBf16Args a) {
  const int lane = threadIdx.x & 63, ob = threadIdx.x >> 6;
  const int n = lane & 31, hh = lane >> 5;
  const int64_t tiles_per_t = (a.N + 31) / 32, n_tiles = tiles_per_t * a.n_used;
  const int64_t per = (n_tiles + a.n_groups - 1) / a.n_groups;
  const int64_t tile0 = (int64_t)blockIdx.x * per, tile1 = min(n_tiles, tile0 + per);
  const bf16x8 sel0 = sel_frag(0, lane), sel1 = sel_frag(1, lane);
  floatx16 acc[NG][4] = {};
  for (int64_t tile = tile0; tile < tile1; ++tile) {
    const int32_t t = a.used_t[tile / tiles_per_t];
    const int64_t v = (tile % tiles_per_t) * 32 + n;
    const bool valid = v < a.N;
    const int64_t row = (int64_t)t * a.N + (valid ? v : a.N - 1);
    const bool ok = valid && (!a.covered_only || a.owner[row] >= 0);
    bf16x8 at[4][2], al[4][2];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      floatx16 tr = {}, trl = {};
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int off = (2 * jb + c) * 16 + 8 * hh;
        if (AU) {
          float x[8];
          if (ok) {
            const float4 u0 = *reinterpret_cast<const float4*>(a.Uf + row * kS + off);
            const float4 u1 = *reinterpret_cast<const float4*>(a.Uf + row * kS + off + 4);
            const float4 p0 = *reinterpret_cast<const float4*>(a.pos + t * kS + off);
            const float4 p1 = *reinterpret_cast<const float4*>(a.pos + t * kS + off + 4);
            x[0] = elu(u0.x) + p0.x; x[1] = elu(u0.y) + p0.y; x[2] = elu(u0.z) + p0.z; x[3] = elu(u0.w) + p0.w;
            x[4] = elu(u1.x) + p1.x; x[5] = elu(u1.y) + p1.y; x[6] = elu(u1.z) + p1.z; x[7] = elu(u1.w) + p1.w;
          } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = 0.f;
          }
          bf16x8 xh, xl;
          split8(x, xh, xl);
          tr = mfma(xh, c ? sel1 : sel0, tr);
          trl = mfma(xl, c ? sel1 : sel0, trl);
        } else {
          uint4 u = make_uint4(0, 0, 0, 0);
          if (ok) u = *reinterpret_cast<const uint4*>(a.A + row * a.lda + off);
          tr = mfma(as_frag(u), c ? sel1 : sel0, tr);
        }
      }
      at[jb][0] = pack8v(tr, 0);
      at[jb][1] = pack8v(tr, 8);
      if (AU) {
        al[jb][0] = pack8v(trl, 0);
        al[jb][1] = pack8v(trl, 8);
      }
    }
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      floatx16 tr = {};
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        uint4 u = make_uint4(0, 0, 0, 0);
        if (ok) u = *reinterpret_cast<const uint4*>(a.G[gi] + row * kS + (2 * ob + c) * 16 + 8 * hh);
        tr = mfma(as_frag(u), c ? sel1 : sel0, tr);
      }
      const bf16x8 g0 = pack8v(tr, 0), g1 = pack8v(tr, 8);
#pragma unroll
      for (int ib = 0; ib < 4; ++ib) {
        acc[gi][ib] = mfma(g0, at[ib][0], acc[gi][ib]);
        acc[gi][ib] = mfma(g1, at[ib][1], acc[gi][ib]);
        if (AU) {
          acc[gi][ib] = mfma(g0, al[ib][0], acc[gi][ib]);
          acc[gi][ib] = mfma(g1, al[ib][1], acc[gi][ib]);
        }
      }
    }
  }
#pragma unroll
  for (int gi = 0; gi < NG; ++gi) {
    float* out = a.partial + ((int64_t)blockIdx.x * NG + gi) * kS * kS;
#pragma unroll
    for (int ib = 0; ib < 4; ++ib)
#pragma unroll
      for (int vv = 0; vv < 16; ++vv)
        out[(ob * 32 + 8 * (vv >> 2) + 4 * hh + (vv & 3)) * kS + ib * 32 + n] = acc[gi][ib][vv];
  }
}

// out[e] = scale * sum over slots (ascending) of partial[slot * stride + e]
__global__ void k_reduce_slots(const float* partial, int64_t n_slots, int64_t stride, int64_t n_elem, float scale,
                               float* out) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_elem) return;
  float s = 0.f;
  for (int64_t k = 0; k < n_slots; ++k) s += partial[k * stride + e];
  out[e] = scale * s;
}

// ---------------------------------------------------------------------------------------------
// Graph attention backward, row pass: for every covered row i, c_i^h = du_i^h . u_i^h and
// d s_dst_i^h = sum_j dpre_ij^h,  dpre = alpha (du_i^h . z_j^h - c_i^h) LeakyReLU'(e_ij^h).
// Lane = (neighbour slot lane/8, head lane%8): eight neighbours at a time, each lane reads its
// head's 32-byte slice of the neighbour's z row and does the 16-dim dot product on its own.
struct GatBwdRowsArgs {
  GraphDev g;
  const Segment* segs;
  const int32_t* work; int64_t n_work;
  const uint16_t* zX; const uint16_t* zC;
  const float* sX; const float* sC;
  const float* U; const uint16_t* dU;
  const float* lse;
  float* st2;     // [T*N][16]: d s_dst[8], c[8]
};

__device__ __forceinline__ void load16(const uint16_t* p, float* x) {
  unpack8(reinterpret_cast<const uint4*>(p)[0], x);
  unpack8(reinterpret_cast<const uint4*>(p)[1], x + 8);
}

__global__ __launch_bounds__(256) void k_gat_bwd_rows(GatBwdRowsArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_work) return;
  const int32_t si = a.work[3 * item], r0 = a.work[3 * item + 1], nr = a.work[3 * item + 2];
  const Segment s = a.segs[si];
  const int64_t N = a.g.N;
  const int64_t* rowptr = a.g.rowptr[s.t];
  const int32_t* col = a.g.colidx[s.t];
  const int64_t base = (int64_t)s.t * N;
  const int slot = lane >> 3, h = lane & 7;
  for (int rr = 0; rr < nr; ++rr) {
    const int64_t i = s.v_lo + r0 + rr;
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    float du[16], u[16];
    load16(a.dU + (base + i) * kS + 16 * h, du);
#pragma unroll
    for (int d4 = 0; d4 < 4; ++d4) {
      const float4 x = *reinterpret_cast<const float4*>(a.U + (base + i) * kS + 16 * h + 4 * d4);
      u[4 * d4] = x.x; u[4 * d4 + 1] = x.y; u[4 * d4 + 2] = x.z; u[4 * d4 + 3] = x.w;
    }
    float c = 0.f;
#pragma unroll
    for (int d = 0; d < 16; ++d) c += du[d] * u[d];
    const float sd = a.sX[(base + i) * 16 + 8 + h];
    const float lse = a.lse[(base + i) * 8 + h];
    float dsd = 0.f;
    for (int64_t eb = e0; eb < e1; eb += 64) {
      const int cnt = (int)min((int64_t)64, e1 - eb);
      const int32_t jl = lane < cnt ? col[eb + lane] : 0;
      for (int q0 = 0; q0 < cnt; q0 += 8) {
        const int32_t j = __shfl(jl, q0 + slot);
        if (q0 + slot < cnt) {
          const bool in = j >= s.v_lo && j < s.v_hi;
          float z[16];
          load16((in ? a.zX : a.zC) + (base + j) * kS + 16 * h, z);
          const float ss = in ? a.sX[(base + j) * 16 + h] : a.sC[(base + j) * 8 + h];
          const float e = sd + ss;
          const float al = __expf(lrelu(e) - lse);
          float da = 0.f;
#pragma unroll
          for (int d = 0; d < 16; ++d) da += du[d] * z[d];
          dsd += al * (da - c) * (e > 0.f ? 1.f : kSlope);
        }
      }
    }
    dsd += __shfl_xor(dsd, 8);
    dsd += __shfl_xor(dsd, 16);
    dsd += __shfl_xor(dsd, 32);
    if (slot == 0) {
      a.st2[(base + i) * 16 + h] = dsd;
      a.st2[(base + i) * 16 + 8 + h] = c;
    }
  }
}

// Graph attention backward, reverse-edge pass: for every vertex j of every snapshot in use, the
// gradients of its two projections (z_j as seen from inside its own chunk: zX; as an
// out-of-chunk neighbour: zC) are gathered over the rows i that list j, i.e. over j's own stored
// row (the adjacency is symmetric):
//   dz_j += alpha_ij du_i,   d s_src_j^h += dpre_ij^h,
// then  dzX_j += d s_dst_j a_dst + d s_srcX_j a_src,  dzC_j += d s_srcC_j a_src, and the gradients
// of a_src, a_dst are accumulated per wave.  Lanes span the 128 features (two per lane).
struct GatBwdColsArgs {
  GraphDev g;
  const int32_t* used_t; int32_t n_used;
  const int32_t* owner;
  const uint16_t* zX; const uint16_t* zC;
  const float* sX; const float* sC;
  const uint16_t* dU;
  const float* lse; const float* st2;
  const float* a_src; const float* a_dst;
  uint16_t* dzX; uint16_t* dzC;
  float* da_partial;    // [n_waves][2][128]: d a_src, d a_dst
  int32_t n_waves;
};

__global__ __launch_bounds__(256) void k_gat_bwd_cols(GatBwdColsArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t N = a.g.N;
  const int64_t groups_per_t = (N + 15) / 16, n_items = groups_per_t * a.n_used;
  const int head = lane >> 3;
  const float as0 = a.a_src[2 * lane], as1 = a.a_src[2 * lane + 1];
  const float ad0 = a.a_dst[2 * lane], ad1 = a.a_dst[2 * lane + 1];
  float gas0 = 0.f, gas1 = 0.f, gad0 = 0.f, gad1 = 0.f;
  for (int64_t item = wave; item < n_items; item += a.n_waves) {
    const int32_t t = a.used_t[item / groups_per_t];
    const int64_t j0 = (item % groups_per_t) * 16;
    const int64_t* rowptr = a.g.rowptr[t];
    const int32_t* col = a.g.colidx[t];
    const int64_t base = (int64_t)t * N;
    const int nr = (int)min((int64_t)16, N - j0);
    for (int rr = 0; rr < nr; ++rr) {
      const int64_t j = j0 + rr;
      const int32_t oj = a.owner[base + j];
      const uint32_t zc = *reinterpret_cast<const uint32_t*>(a.zC + (base + j) * kS + 2 * lane);
      const uint32_t zx = oj >= 0 ? *reinterpret_cast<const uint32_t*>(a.zX + (base + j) * kS + 2 * lane) : 0u;
      const float zx0 = bf_lo(zx), zx1 = bf_hi(zx), zc0 = bf_lo(zc), zc1 = bf_hi(zc);
      const float ssx = oj >= 0 ? a.sX[(base + j) * 16 + head] : 0.f;
      const float ssc = a.sC[(base + j) * 8 + head];
      float ax0 = 0.f, ax1 = 0.f, ac0 = 0.f, ac1 = 0.f, dsx = 0.f, dsc = 0.f;
      const int64_t e0 = rowptr[j], e1 = rowptr[j + 1];
      for (int64_t eb = e0; eb < e1; eb += 64) {
        const int cnt = (int)min((int64_t)64, e1 - eb);
        const int32_t il = lane < cnt ? col[eb + lane] : 0;
        const int32_t ol = lane < cnt ? a.owner[base + il] : -1;
        for (int q0 = 0; q0 < cnt; q0 += 8) {
          uint32_t dv[8];
          float sd[8], ls[8], cc[8];
          int same[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            same[q] = -1;   // -1: skip
            dv[q] = 0u; sd[q] = 0.f; ls[q] = 0.f; cc[q] = 0.f;
            if (q0 + q < cnt) {
              const int32_t oi = __builtin_amdgcn_readlane(ol, q0 + q);
              if (oi >= 0) {
                const int64_t ri = base + __builtin_amdgcn_readlane(il, q0 + q);
                same[q] = oi == oj ? 1 : 0;
                dv[q] = *reinterpret_cast<const uint32_t*>(a.dU + ri * kS + 2 * lane);
                sd[q] = a.sX[ri * 16 + 8 + head];
                ls[q] = a.lse[ri * 8 + head];
                cc[q] = a.st2[ri * 16 + 8 + head];
              }
            }
          }
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            if (same[q] < 0) continue;      // wave-uniform
            const bool sm = same[q] != 0;
            const float d0 = bf_lo(dv[q]), d1 = bf_hi(dv[q]);
            const float e = sd[q] + (sm ? ssx : ssc);
            const float al = __expf(lrelu(e) - ls[q]);
            float da = d0 * (sm ? zx0 : zc0) + d1 * (sm ? zx1 : zc1);
            da += __shfl_xor(da, 1);
            da += __shfl_xor(da, 2);
            da += __shfl_xor(da, 4);
            const float dpre = al * (da - cc[q]) * (e > 0.f ? 1.f : kSlope);
            if (sm) { ax0 += al * d0; ax1 += al * d1; dsx += dpre; }
            else { ac0 += al * d0; ac1 += al * d1; dsc += dpre; }
          }
        }
      }
      if (oj >= 0) {
        const float dsd = a.st2[(base + j) * 16 + head];
        *reinterpret_cast<uint32_t*>(a.dzX + (base + j) * kS + 2 * lane) =
            pack2(ax0 + dsd * ad0 + dsx * as0, ax1 + dsd * ad1 + dsx * as1);
        gad0 += dsd * zx0; gad1 += dsd * zx1;
        gas0 += dsx * zx0; gas1 += dsx * zx1;
      }
      *reinterpret_cast<uint32_t*>(a.dzC + (base + j) * kS + 2 * lane) = pack2(ac0 + dsc * as0, ac1 + dsc * as1);
      gas0 += dsc * zc0; gas1 += dsc * zc1;
    }
  }
  if (wave < a.n_waves) {
    float* o = a.da_partial + (int64_t)wave * 2 * kS;
    o[2 * lane] = gas0; o[2 * lane + 1] = gas1;
    o[kS + 2 * lane] = gad0; o[kS + 2 * lane + 1] = gad1;
  }
}

}  // namespace

namespace {
constexpr int kDwGroups = 256;     // workgroups (slots) of the weight-gradient kernel
constexpr int kTbwdWaves = 2048;   // waves (slots) of the temporal backward kernel
constexpr int kColsBlocks = 1024;  // workgroups of the reverse-edge pass (4 slots each)
}  // namespace

// scratch layout: [weight-gradient slots | position-gradient slots | attention-vector slots]
int64_t dysat_partial_elems(const DysatWs& ws) {
  return (int64_t)kDwGroups * 3 * kS * kS + (int64_t)kTbwdWaves * ws.T * kS + (int64_t)kColsBlocks * 4 * 2 * kS;
}
int64_t dysat_loss_partial_elems(const DysatWs&) { return kTbwdWaves; }

void dysat_backward(const DysatWs& ws, const void* Y, int64_t ldy, const void* dY, int64_t lddy, const void* target,
                    int64_t ldt, float* loss_out, hipEvent_t* ev, hipStream_t st) {
  float* dw_slots = ws.partial;
  float* dpos_slots = dw_slots + (int64_t)kDwGroups * 3 * kS * kS;
  float* da_slots = dpos_slots + (int64_t)kTbwdWaves * ws.T * kS;
  const int64_t count = ws.total_rows * kS;
  const int n_tw = (int)std::min<int64_t>(kTbwdWaves, ws.n_tiles);
  const int64_t tiles32 = (ws.N + 31) / 32 * ws.n_used;
  const int groups = (int)std::min<int64_t>(kDwGroups, tiles32);

  // (1) temporal attention
  hipLaunchKernelGGL(k_fill_f32, blocks_for((int64_t)n_tw * ws.T * kS, 256), 256, 0, st, dpos_slots, 0.f,
                     (int64_t)n_tw * ws.T * kS);
  if (ev) (void)hipEventRecord(ev[0], st);
  TemporalBwdArgs ta{};
  ta.chunks = ws.chunks; ta.n_chunks = ws.n_chunks; ta.tile_ptr = ws.tile_ptr; ta.n_tiles = ws.n_tiles;
  ta.N = ws.N; ta.T = ws.T; ta.U = ws.U; ta.pos = ws.P[DY_POS];
  ta.Wq = ws.Wqp; ta.Wk = ws.Wkp; ta.Wv = ws.Wvp; ta.WqT = ws.WqT; ta.WkT = ws.WkT; ta.WvT = ws.WvT;
  ta.Y = static_cast<const uint16_t*>(Y); ta.ldy = ldy;
  ta.dY = static_cast<const uint16_t*>(dY); ta.lddy = lddy;
  ta.target = static_cast<const uint16_t*>(target); ta.ldt = ldt;
  ta.scale = 2.0f / (float)count;
  ta.dU = ws.dU; ta.dQ = ws.dQ; ta.dK = ws.dK; ta.dV = ws.dV;
  ta.dpos_partial = dpos_slots; ta.loss_partial = ws.loss_partial; ta.n_waves = n_tw;
  hipLaunchKernelGGL(k_temporal_bwd, n_tw, 64, 0, st, ta);
  hipLaunchKernelGGL(k_reduce_slots, blocks_for((int64_t)ws.T * kS, 256), 256, 0, st, dpos_slots, (int64_t)n_tw,
                     (int64_t)ws.T * kS, (int64_t)ws.T * kS, 1.f, ws.G[DY_POS]);
  if (target && loss_out)
    hipLaunchKernelGGL(k_reduce_slots, 1, 64, 0, st, ws.loss_partial, (int64_t)n_tw, (int64_t)1, (int64_t)1,
                       1.0f / (float)count, loss_out);
  // (2) dW_q, dW_k, dW_v = sum over rows of d{q,k,v}^T P
  DwBf16Args da{};
  da.used_t = ws.used_t; da.n_used = ws.n_used; da.N = ws.N; da.owner = ws.owner; da.covered_only = 1;
  da.A = nullptr; da.lda = 0; da.Uf = ws.U; da.pos = ws.P[DY_POS];
  da.G[0] = ws.dQ; da.G[1] = ws.dK; da.G[2] = ws.dV;
  da.partial = dw_slots; da.n_groups = groups;
  hipLaunchKernelGGL((k_dw_bf16<3, true>), groups, 256, 0, st, da);
  for (int gi = 0; gi < 3; ++gi)
    hipLaunchKernelGGL(k_reduce_slots, blocks_for(kS * kS, 256), 256, 0, st, dw_slots + (int64_t)gi * kS * kS,
                       (int64_t)groups, (int64_t)3 * kS * kS, (int64_t)kS * kS, 1.f, ws.G[DY_WQ + gi]);
  if (ev) (void)hipEventRecord(ev[1], st);
  // (3) graph attention, row pass
  GatBwdRowsArgs ra{};
  ra.g = ws.g; ra.segs = ws.segs; ra.work = ws.work_short; ra.n_work = ws.n_short;
  ra.zX = ws.zX; ra.zC = ws.zC; ra.sX = ws.sX; ra.sC = ws.sC; ra.U = ws.U; ra.dU = ws.dU; ra.lse = ws.lse;
  ra.st2 = ws.st2;
  hipLaunchKernelGGL(k_gat_bwd_rows, blocks_for(ws.n_short, 4), 256, 0, st, ra);
  if (ev) (void)hipEventRecord(ev[2], st);
  // (4) reverse-edge pass
  const int64_t items = (ws.N + 15) / 16 * ws.n_used;
  const int cblocks = (int)std::min<int64_t>(kColsBlocks, (items + 3) / 4);
  GatBwdColsArgs ca{};
  ca.g = ws.g; ca.used_t = ws.used_t; ca.n_used = ws.n_used; ca.owner = ws.owner;
  ca.zX = ws.zX; ca.zC = ws.zC; ca.sX = ws.sX; ca.sC = ws.sC; ca.dU = ws.dU; ca.lse = ws.lse; ca.st2 = ws.st2;
  ca.a_src = ws.P[DY_ASRC]; ca.a_dst = ws.P[DY_ADST];
  ca.dzX = ws.dzX; ca.dzC = ws.dzC; ca.da_partial = da_slots; ca.n_waves = cblocks * 4;
  hipLaunchKernelGGL(k_gat_bwd_cols, cblocks, 256, 0, st, ca);
  hipLaunchKernelGGL(k_reduce_slots, 1, 128, 0, st, da_slots, (int64_t)cblocks * 4, (int64_t)2 * kS, (int64_t)kS, 1.f,
                     ws.G[DY_ASRC]);
  hipLaunchKernelGGL(k_reduce_slots, 1, 128, 0, st, da_slots + kS, (int64_t)cblocks * 4, (int64_t)2 * kS, (int64_t)kS,
                     1.f, ws.G[DY_ADST]);
  // (5) dW = sum over covered rows of dzX^T x  +  sum over all rows of dzC^T c
  DwBf16Args dx = da;
  dx.A = static_cast<const uint16_t*>(ws.X); dx.lda = ws.ldx; dx.Uf = nullptr; dx.covered_only = 1;
  dx.G[0] = ws.dzX; dx.partial = dw_slots;
  hipLaunchKernelGGL((k_dw_bf16<1, false>), groups, 256, 0, st, dx);
  DwBf16Args dc = dx;
  dc.A = static_cast<const uint16_t*>(ws.C); dc.lda = ws.ldc; dc.covered_only = 0;
  dc.G[0] = ws.dzC; dc.partial = dw_slots + (int64_t)groups * kS * kS;
  hipLaunchKernelGGL((k_dw_bf16<1, false>), groups, 256, 0, st, dc);
  hipLaunchKernelGGL(k_reduce_slots, blocks_for(kS * kS, 256), 256, 0, st, dw_slots, (int64_t)2 * groups,
                     (int64_t)kS * kS, (int64_t)kS * kS, 1.f, ws.G[DY_W]);
  if (ev) (void)hipEventRecord(ev[3], st);
}

}  // namespace dgc
