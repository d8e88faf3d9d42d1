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
  const uint16_t* Y; int64_t ldy;          // with target: dY = scale * (Y - target)
  const uint16_t* dY; int64_t lddy;        // or the upstream gradient itself
  const uint16_t* target; int64_t ldt;
  float scale;
  uint16_t *dQ, *dK, *dV;
  float* loss_partial;   // [gridDim.x * waves per block]
};

// value of lane l^32
__device__ __forceinline__ float xor32(float x, int hh) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(hh ? r[0] : r[1]);
}

// raw 16-byte pieces of the upstream gradient (or of Y and the target) of features [off, off+8)
struct DyRaw { uint4 a, b; };

__device__ __forceinline__ DyRaw load_dy_raw(const TemporalBwdArgs& a, int64_t row, int off, bool valid) {
  DyRaw r;
  r.a = make_uint4(0, 0, 0, 0);
  r.b = r.a;
  if (valid) {
    if (a.dY) {
      r.a = *reinterpret_cast<const uint4*>(a.dY + row * a.lddy + off);
    } else {
      r.a = *reinterpret_cast<const uint4*>(a.Y + row * a.ldy + off);
      r.b = *reinterpret_cast<const uint4*>(a.target + row * a.ldt + off);
    }
  }
  return r;
}
// -> dL/dY of those 8 features; adds (Y - target)^2 to sq (rows that are not valid give zeros)
__device__ __forceinline__ void dy_from_raw(const TemporalBwdArgs& a, const DyRaw& r, float* out, float& sq) {
  unpack8(r.a, out);
  if (!a.dY) {
    float g[8];
    unpack8(r.b, g);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float d = out[i] - g[i];
      out[i] = a.scale * d;
      sq += d * d;
    }
  }
}

constexpr int kFragsPerW = 4 * 8 * 64;   // uint4 fragments of one 128 x 128 weight

__device__ __forceinline__ void stage_weights(uint4* lds, const uint4* w0, const uint4* w1, const uint4* w2) {
  for (int i = threadIdx.x; i < kFragsPerW; i += blockDim.x) {
    lds[i] = w0[i];
    lds[kFragsPerW + i] = w1[i];
    lds[2 * kFragsPerW + i] = w2[i];
  }
  __syncthreads();
}

// Temporal self-attention, backward, first half: dQ, dK, dV (and the loss).  The workgroup stages
// W_q, W_k, W_v in LDS; each of its waves then walks 2-vertex tiles with a grid stride.  Per tile
// it recomputes P, Q, K, V (Q, K also in column layout).  Per head, the "query-major" score block
// (lane = query row, registers = key steps) gives the probabilities p, delta = sum_r p dp and dS;
// dQ needs dS in that orientation, dK and dV need dS and p "key-major" (lane = key row,
// registers = query steps): those are obtained by one product each with a selection operand
// (a 16 x 16 transpose per vertex on the matrix core, exact for the hi and the lo part).
// All operands are hi + lo pairs.  dQ, dK, dV land in row layout and are stored (bf16).
// WIDE (one vertex per tile, windows of up to 32 snapshots): a lane's 16 score registers are all
// keys of its own vertex, the transposes are 32 x 32 (two selection products, one per half of the
// keys), and the three final products contract over the two halves of the keys / queries instead
// of over two vertices.
template <bool WIDE>
__global__ __launch_bounds__(256) void k_temporal_bwd(TemporalBwdArgs a) {
  extern __shared__ uint4 wlds[];
  stage_weights(wlds, a.Wq, a.Wk, a.Wv);
  const int lane = threadIdx.x & 63, nw = blockDim.x >> 6, wave = threadIdx.x >> 6;
  const int hh = lane >> 5, f = lane & 31;
  float sq = 0.f;
  const uint32_t m_head[2] = {(f >> 4) == 0 ? 0xffffffffu : 0u, (f >> 4) == 1 ? 0xffffffffu : 0u};
  const bf16x8 sel0 = sel_frag(0, lane), sel1 = sel_frag(1, lane);
  constexpr int NP = WIDE ? 16 : 8, NH = NP / 8;
  // B operand: element p of lane (j, hh) is 1 where step 8 (p/4) + 4 hh + p%4 == j % 16 (WIDE: where
  // step 16 c + ... == j, one operand per half c of the steps)
  bf16x8 selT[NH];
#pragma unroll
  for (int c = 0; c < NH; ++c)
#pragma unroll
    for (int p = 0; p < 8; ++p)
      selT[c][p] = (16 * c + 8 * (p >> 2) + 4 * hh + (p & 3) == (WIDE ? (lane & 31) : (lane & 15))) ? (__bf16)1.0f : (__bf16)0.0f;
  for (int64_t tile = (int64_t)blockIdx.x * nw + wave; tile < a.n_tiles; tile += (int64_t)gridDim.x * nw) {
    const TileRow r = tile_row<WIDE>(a.chunks, a.n_chunks, a.tile_ptr, tile, a.N, lane);
    const uint32_t m_vert[2] = {r.a == 0 ? 0xffffffffu : 0u, r.a == 1 ? 0xffffffffu : 0u};
    DyRaw raw[2];
    raw[0] = load_dy_raw(a, r.row, 8 * hh, r.valid);
    raw[1] = load_dy_raw(a, r.row, 16 + 8 * hh, r.valid);
    bf16x8 pf[8], pl[8];
    load_p_frags<true>(a.U, a.pos, r, hh, pf, pl);
#pragma unroll 1
    for (int jb = 0; jb < 4; ++jb) {
      // dL/dY of features [32 jb, 32 jb + 32): d8[c] = natural fragment kb = 2 jb + c; the next
      // block's pieces are requested now
      float d8[2][8];
      dy_from_raw(a, raw[0], d8[0], sq);
      dy_from_raw(a, raw[1], d8[1], sq);
      if (jb < 3) {
        raw[0] = load_dy_raw(a, r.row, (2 * jb + 2) * 16 + 8 * hh, r.valid);
        raw[1] = load_dy_raw(a, r.row, (2 * jb + 3) * 16 + 8 * hh, r.valid);
      }
      floatx16 q = {}, k = {}, v = {}, qt = {}, kt = {}, dyt = {};
#pragma unroll
      for (int kb = 0; kb < 8; ++kb) {
        const int fi = (jb * 8 + kb) * 64 + lane;
        const bf16x8 wq = as_frag(wlds[fi]), wk = as_frag(wlds[kFragsPerW + fi]), wv = as_frag(wlds[2 * kFragsPerW + fi]);
        q = mfma2b(wq, pf[kb], pl[kb], q);
        k = mfma2b(wk, pf[kb], pl[kb], k);
        v = mfma2b(wv, pf[kb], pl[kb], v);
        qt = mfma2a(pf[kb], pl[kb], wq, qt);
        kt = mfma2a(pf[kb], pl[kb], wk, kt);
      }
      {
        bf16x8 dh, dl;
        split8(d8[0], dh, dl);
        dyt = mfma2a(dh, dl, sel0, dyt);
        split8(d8[1], dh, dl);
        dyt = mfma2a(dh, dl, sel1, dyt);
      }
      floatx16 dq = {}, dk = {}, dv = {};
#pragma unroll
      for (int hd = 0; hd < 2; ++hd) {
        bf16x8 kh, kl, qh, ql, vh, vl, dyh, dyl;
        split8v(k, 8 * hd, kh, kl);
        split8v(q, 8 * hd, qh, ql);
        split8v(v, 8 * hd, vh, vl);
        {
          // dL/dY of the head's 16 dims in row-layout order: dims 8 c + 4 hh + e; the half c == hh is
          // in the lane's own natural fragment, the other half in lane l^32's
          float x[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float lo4 = d8[hd][e], hi4 = d8[hd][4 + e];   // static indices: a lane-dependent index
            const float other = xor32(hh ? lo4 : hi4, hh);       // would be lowered to a chain of selects
            const float own = hh ? hi4 : lo4;
            x[e] = hh ? other : own;
            x[4 + e] = hh ? own : other;
          }
          split8(x, dyh, dyl);
        }
        floatx16 st = {}, dpt = {};
        st = mfma3(kh, kl, qh, ql, st);         // [key row][query row]
        dpt = mfma3(vh, vl, dyh, dyl, dpt);
        float pr[NP], dst[NP];
        float mx = -INFINITY;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int rk = 8 * (p >> 2) + 4 * hh + (p & 3);
          pr[p] = rk <= r.s ? 0.25f * (WIDE ? st[p] : pick_half(st, p, m_vert[0], m_vert[1])) : -INFINITY;
          mx = fmaxf(mx, pr[p]);
        }
        mx = fmaxf(mx, xor32(mx, hh));
        float sum = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          pr[p] = __expf(pr[p] - mx);
          sum += pr[p];
        }
        sum += xor32(sum, hh);
        const float inv = 1.f / sum;
        float delta = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          pr[p] *= inv;
          dst[p] = WIDE ? dpt[p] : pick_half(dpt, p, m_vert[0], m_vert[1]);
          delta += pr[p] * dst[p];
        }
        delta += xor32(delta, hh);
#pragma unroll
        for (int p = 0; p < NP; ++p) dst[p] = 0.25f * pr[p] * (dst[p] - delta);
        bf16x8 dsth[NH], dstl[NH], prh[NH], prl[NH];
#pragma unroll
        for (int c = 0; c < NH; ++c) {
          split8(dst + 8 * c, dsth[c], dstl[c]);
          split8(pr + 8 * c, prh[c], prl[c]);
        }
        // key-major copies: T[i = query row][j = key row]
        floatx16 t0 = {}, t1 = {}, t2 = {}, t3 = {};
#pragma unroll
        for (int c = 0; c < NH; ++c) {
          t0 = mfma(dsth[c], selT[c], t0);
          t1 = mfma(dstl[c], selT[c], t1);
          t2 = mfma(prh[c], selT[c], t2);
          t3 = mfma(prl[c], selT[c], t3);
        }
        // own-vertex half of the registers, blended arithmetically (a select here gets merged with the
        // packing below into per-element selects on 16-bit halves); WIDE: all 16 are the vertex's own
        const float fa0 = r.a ? 0.f : 1.f, fa1 = 1.f - fa0;
        float tx[4][NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          tx[0][p] = WIDE ? t0[p] : fa0 * t0[p] + fa1 * t0[8 + (p & 7)];
          tx[1][p] = WIDE ? t1[p] : fa0 * t1[p] + fa1 * t1[8 + (p & 7)];
          tx[2][p] = WIDE ? t2[p] : fa0 * t2[p] + fa1 * t2[8 + (p & 7)];
          tx[3][p] = WIDE ? t3[p] : fa0 * t3[p] + fa1 * t3[8 + (p & 7)];
        }
        bf16x8 ds2h[NH], ds2l[NH], p2h[NH], p2l[NH];
#pragma unroll
        for (int c = 0; c < NH; ++c) {
          ds2h[c] = pack8(tx[0] + 8 * c); ds2l[c] = pack8(tx[1] + 8 * c);
          p2h[c] = pack8(tx[2] + 8 * c); p2l[c] = pack8(tx[3] + 8 * c);
        }
#pragma unroll
        for (int av = 0; av < 2; ++av) {      // the two vertices, or (WIDE) the two halves of the window's steps
          const uint32_t mv = WIDE ? 0xffffffffu : m_vert[av], mh = m_head[hd];
          const int c = WIDE ? av : 0;
          bf16x8 ah, al;
          split8v(kt, 8 * av, ah, al);
          dq = mfma3(and_mask(ah, mh), and_mask(al, mh), and_mask(dsth[c], mv), and_mask(dstl[c], mv), dq);
          split8v(qt, 8 * av, ah, al);
          dk = mfma3(and_mask(ah, mh), and_mask(al, mh), and_mask(ds2h[c], mv), and_mask(ds2l[c], mv), dk);
          split8v(dyt, 8 * av, ah, al);
          dv = mfma3(and_mask(ah, mh), and_mask(al, mh), and_mask(p2h[c], mv), and_mask(p2l[c], mv), dv);
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
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
  if (lane == 0) a.loss_partial[blockIdx.x * nw + wave] = sq;
}

// Temporal self-attention, backward, second half: dP = dQ W_q + dK W_k + dV W_v from the stored
// gradients, dU = dP * ELU'(U), and the gradient of the position table (column sums of dP per
// snapshot).  Rows are the covered vertices of the snapshots in use, 32 per tile; the transposed
// weights are staged in LDS; dQ/dK/dV row fragments are B operands as they come from memory.
// Every wave sums dP over its tiles in registers (lane = row slot) and, when the snapshot
// changes, adds the 32 row slots and writes the sums to its own slot of the scratch buffer.
struct TemporalBwd2Args {
  const int32_t* used_t; int32_t n_used; int64_t N; int32_t T;
  const int32_t* owner;
  const float* U;
  const uint4 *WqT, *WkT, *WvT;
  const uint16_t *dQ, *dK, *dV;
  uint16_t* dU;
  float* dpos_partial;   // [gridDim.x * waves per block][T][128], zero on entry
};

__device__ __forceinline__ void flush_dpos(float* slot, int t, int lane, floatx16* acc) {
  const int n = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int ib = 0; ib < 4; ++ib) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float x = acc[ib][v];
      x += __shfl_xor(x, 1); x += __shfl_xor(x, 2); x += __shfl_xor(x, 4); x += __shfl_xor(x, 8); x += __shfl_xor(x, 16);
      acc[ib][v] = x;
    }
    if (n == 0) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4* p = reinterpret_cast<float4*>(slot + (int64_t)t * kS + ib * 32 + 8 * g + 4 * hh);
        float4 o = *p;
        o.x += acc[ib][4 * g]; o.y += acc[ib][4 * g + 1]; o.z += acc[ib][4 * g + 2]; o.w += acc[ib][4 * g + 3];
        *p = o;
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[ib][v] = 0.f;
  }
}

__global__ __launch_bounds__(512) void k_temporal_bwd2(TemporalBwd2Args a) {
  extern __shared__ uint4 wlds[];
  stage_weights(wlds, a.WqT, a.WkT, a.WvT);
  const int lane = threadIdx.x & 63, nw = blockDim.x >> 6, wave = threadIdx.x >> 6;
  const int n = lane & 31, hh = lane >> 5;
  const int64_t tiles_per_t = (a.N + 31) / 32, n_tiles = tiles_per_t * a.n_used;
  const int64_t gw = (int64_t)blockIdx.x * nw + wave, n_gw = (int64_t)gridDim.x * nw;
  const int64_t per = (n_tiles + n_gw - 1) / n_gw;
  const int64_t tile0 = gw * per, tile1 = min(n_tiles, tile0 + per);
  float* slot = a.dpos_partial + gw * a.T * kS;
  floatx16 dpos[4] = {};
  int cur_t = -1;
  for (int64_t tile = tile0; tile < tile1; ++tile) {
    const int32_t t = a.used_t[tile / tiles_per_t];
    if (t != cur_t) {
      if (cur_t >= 0) flush_dpos(slot, cur_t, lane, dpos);
      cur_t = t;
    }
    const int64_t v = (tile % tiles_per_t) * 32 + n;
    const bool valid = v < a.N;
    const int64_t row = (int64_t)t * a.N + (valid ? v : a.N - 1);
    const bool ok = valid && a.owner[row] >= 0;
    floatx16 dP[4] = {};
#pragma unroll 2
    for (int ks = 0; ks < 8; ++ks) {
      uint4 uq = make_uint4(0, 0, 0, 0), uk = uq, uv = uq;
      if (ok) {
        uq = *reinterpret_cast<const uint4*>(a.dQ + row * kS + ks * 16 + 8 * hh);
        uk = *reinterpret_cast<const uint4*>(a.dK + row * kS + ks * 16 + 8 * hh);
        uv = *reinterpret_cast<const uint4*>(a.dV + row * kS + ks * 16 + 8 * hh);
      }
#pragma unroll
      for (int ib = 0; ib < 4; ++ib) {
        const int fi = (ib * 8 + ks) * 64 + lane;
        dP[ib] = mfma(as_frag(wlds[fi]), as_frag(uq), dP[ib]);
        dP[ib] = mfma(as_frag(wlds[kFragsPerW + fi]), as_frag(uk), dP[ib]);
        dP[ib] = mfma(as_frag(wlds[2 * kFragsPerW + fi]), as_frag(uv), dP[ib]);
      }
    }
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
      if (ok) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int64_t o = row * kS + ib * 32 + 8 * g + 4 * hh;
          const float4 u = *reinterpret_cast<const float4*>(a.U + o);
          *reinterpret_cast<uint2*>(a.dU + o) = pack4(dP[ib][4 * g] * delu(u.x), dP[ib][4 * g + 1] * delu(u.y),
                                                     dP[ib][4 * g + 2] * delu(u.z), dP[ib][4 * g + 3] * delu(u.w));
        }
      }
      dpos[ib] += dP[ib];
    }
  }
  if (cur_t >= 0) flush_dpos(slot, cur_t, lane, dpos);
}

// ---------------------------------------------------------------------------------------------
// Weight gradients  dW_G[out][in] = sum over rows of G[row][out] * A[row][in]  for NG tensors G
// sharing one A (A = the rows of a bf16 tensor, or P = ELU(U) + pos recomputed from U).  Rows are
// the vertices of the snapshots in use, 32 per tile.  A workgroup of 4 waves walks a contiguous
// range of tiles; wave w owns output rows [32w, 32w+32) of every dW_G.  Both operands need the
// row index as contraction index, i.e. column layout: obtained from natural row fragments with
// the selection products described above.  Eight waves per workgroup: wave w owns output rows
// [32 (w%4), +32) and input columns [64 (w/4), +64) of every dW_G.
struct DwBf16Args {
  const int32_t* used_t; int32_t n_used; int64_t N;
  const int32_t* owner; int32_t covered_only;
  const uint16_t* A; int64_t lda;        // bf16 rows, or
  const float* Uf; const float* pos;     // A = ELU(Uf) + pos (fp32 rows of pitch 128), carried as hi + lo
  const uint16_t* G[3];
  float* partial;      // [n_groups][NG][128][128]
  int32_t n_groups;
};

// Raw operand rows of one 32-row tile as they come from memory, requested ahead of their use
// (loads return in order, so waiting for older registers does not wait for younger requests):
//  - bf16 x bf16 products: both sides of the next tile are requested before the current tile is
//    multiplied;
//  - the ELU(U) + pos variant with three accumulator sets has no room for a second tile: the
//    gradient rows of the current tile are requested before U is converted, and U of the next tile
//    as soon as the conversion has used up the current one; the position rows of the snapshots a
//    workgroup meets are staged in LDS once.
template <bool AU>
struct DwRawA {
  float4 u[AU ? 8 : 1];   // AU: fp32 rows of U, [jb][c][half]
  uint4 a[AU ? 1 : 4];    // otherwise: bf16 rows of A, [jb][c]
  int32_t k;              // index of the tile's snapshot among the snapshots in use
  bool ok;
};

struct DwRow {
  int64_t row;
  int32_t k;
  bool ok;
};

__device__ __forceinline__ DwRow dw_row(const DwBf16Args& a, int64_t tile, int64_t tiles_per_t, int n) {
  DwRow r;
  r.k = (int32_t)(tile / tiles_per_t);
  const int64_t v = (tile % tiles_per_t) * 32 + n;
  const bool valid = v < a.N;
  r.row = (int64_t)a.used_t[r.k] * a.N + (valid ? v : a.N - 1);    // always a row of the tensors
  r.ok = valid && (!a.covered_only || a.owner[r.row] >= 0);       // rows that do not count are zeroed when used
  return r;
}

template <bool AU>
__device__ __forceinline__ void dw_load_a(const DwBf16Args& a, const DwRow& rw, int hh, int ih, DwRawA<AU>& r) {
  r.ok = rw.ok;
  r.k = rw.k;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int off = (2 * (2 * ih + (q >> 1)) + (q & 1)) * 16 + 8 * hh;
    if (AU) {
      r.u[2 * q] = *reinterpret_cast<const float4*>(a.Uf + rw.row * kS + off);
      r.u[2 * q + 1] = *reinterpret_cast<const float4*>(a.Uf + rw.row * kS + off + 4);
    } else {
      r.a[q] = *reinterpret_cast<const uint4*>(a.A + rw.row * a.lda + off);
    }
  }
}

template <int NG>
__device__ __forceinline__ void dw_load_g(const DwBf16Args& a, const DwRow& rw, int hh, int ob, uint4 (&g)[NG][2]) {
#pragma unroll
  for (int gi = 0; gi < NG; ++gi)
#pragma unroll
    for (int c = 0; c < 2; ++c)
      g[gi][c] = *reinterpret_cast<const uint4*>(a.G[gi] + rw.row * kS + (2 * ob + c) * 16 + 8 * hh);
}

__device__ __forceinline__ uint4 keep_if(bool ok, uint4 u) {
  return make_uint4(ok ? u.x : 0u, ok ? u.y : 0u, ok ? u.z : 0u, ok ? u.w : 0u);
}

template <int NG, bool AU>
__global__ __launch_bounds__(512) void k_dw_bf16(DwBf16Args a) {
  const int lane = threadIdx.x & 63, ob = (threadIdx.x >> 6) & 3, ih = threadIdx.x >> 8;
  const int n = lane & 31, hh = lane >> 5;
  const int64_t tiles_per_t = (a.N + 31) / 32, n_tiles = tiles_per_t * a.n_used;
  const int64_t per = (n_tiles + a.n_groups - 1) / a.n_groups;
  const int64_t tile0 = (int64_t)blockIdx.x * per, tile1 = min(n_tiles, tile0 + per);
  const bf16x8 sel0 = sel_frag(0, lane), sel1 = sel_frag(1, lane);
  floatx16 acc[NG][2] = {};
  extern __shared__ float pos_lds[];   // AU: position rows of the snapshots of tiles [tile0, tile1)
  const int32_t k0 = (int32_t)(tile0 / tiles_per_t);
  if (AU) {
    if (tile0 < tile1) {
      const int32_t nk = (int32_t)((tile1 - 1) / tiles_per_t) - k0 + 1;
      for (int i = threadIdx.x; i < nk * kS; i += 512) pos_lds[i] = a.pos[(int64_t)a.used_t[k0 + i / kS] * kS + (i % kS)];
    }
    __syncthreads();
  }
  DwRawA<AU> ra;
  uint4 rg[NG][2];
  if (tile0 < tile1) {
    const DwRow rw = dw_row(a, tile0, tiles_per_t, n);
    dw_load_a<AU>(a, rw, hh, ih, ra);
    if (!AU) dw_load_g<NG>(a, rw, hh, ob, rg);
  }
  for (int64_t tile = tile0; tile < tile1; ++tile) {
    const bool ok = ra.ok;
    const bool more = tile + 1 < tile1;
    DwRow rn{};
    if (more) rn = dw_row(a, tile + 1, tiles_per_t, n);
    DwRawA<AU> na;
    uint4 ng[NG][2];
    if (AU) {
      dw_load_g<NG>(a, dw_row(a, tile, tiles_per_t, n), hh, ob, rg);
    } else if (more) {
      dw_load_a<AU>(a, rn, hh, ih, na);
      dw_load_g<NG>(a, rn, hh, ob, ng);
    }
    bf16x8 at[2][2], al[2][2];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      floatx16 tr = {}, trl = {};
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        if (AU) {
          const float4 u0 = ra.u[(jb * 2 + c) * 2], u1 = ra.u[(jb * 2 + c) * 2 + 1];
          const float* pp = pos_lds + (ra.k - k0) * kS + (2 * (2 * ih + jb) + c) * 16 + 8 * hh;
          const float4 p0 = *reinterpret_cast<const float4*>(pp), p1 = *reinterpret_cast<const float4*>(pp + 4);
          float x[8];
          x[0] = elu(u0.x) + p0.x; x[1] = elu(u0.y) + p0.y; x[2] = elu(u0.z) + p0.z; x[3] = elu(u0.w) + p0.w;
          x[4] = elu(u1.x) + p1.x; x[5] = elu(u1.y) + p1.y; x[6] = elu(u1.z) + p1.z; x[7] = elu(u1.w) + p1.w;
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = ok ? x[i] : 0.f;
          bf16x8 xh, xl;
          split8(x, xh, xl);
          tr = mfma(xh, c ? sel1 : sel0, tr);
          trl = mfma(xl, c ? sel1 : sel0, trl);
        } else {
          tr = mfma(as_frag(keep_if(ok, ra.a[jb * 2 + c])), c ? sel1 : sel0, tr);
        }
      }
      at[jb][0] = pack8v(tr, 0);
      at[jb][1] = pack8v(tr, 8);
      if (AU) {
        al[jb][0] = pack8v(trl, 0);
        al[jb][1] = pack8v(trl, 8);
      }
    }
    if (AU && more) dw_load_a<AU>(a, rn, hh, ih, ra);   // U of this tile is used up: request the next tile's
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      floatx16 tr = {};
#pragma unroll
      for (int c = 0; c < 2; ++c) tr = mfma(as_frag(keep_if(ok, rg[gi][c])), c ? sel1 : sel0, tr);
      const bf16x8 g0 = pack8v(tr, 0), g1 = pack8v(tr, 8);
#pragma unroll
      for (int ib = 0; ib < 2; ++ib) {
        acc[gi][ib] = mfma(g0, at[ib][0], acc[gi][ib]);
        acc[gi][ib] = mfma(g1, at[ib][1], acc[gi][ib]);
        if (AU) {
          acc[gi][ib] = mfma(g0, al[ib][0], acc[gi][ib]);
          acc[gi][ib] = mfma(g1, al[ib][1], acc[gi][ib]);
        }
      }
    }
    if (!AU && more) {
      ra = na;
#pragma unroll
      for (int gi = 0; gi < NG; ++gi) { rg[gi][0] = ng[gi][0]; rg[gi][1] = ng[gi][1]; }
    }
  }
#pragma unroll
  for (int gi = 0; gi < NG; ++gi) {
    float* out = a.partial + ((int64_t)blockIdx.x * NG + gi) * kS * kS;
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
      for (int vv = 0; vv < 16; ++vv)
        out[(ob * 32 + 8 * (vv >> 2) + 4 * hh + (vv & 3)) * kS + (2 * ih + ib) * 32 + n] = acc[gi][ib][vv];
  }
}

// out[e] = scale * sum over slots of partial[slot * stride + e].  A block of 1024 threads covers 64
// elements x 16 slot groups (group g adds slots g, g+16, ... in ascending order); the 16 group
// sums are then added in group order, so the result does not depend on the launch.
__global__ __launch_bounds__(1024) void k_reduce_slots(const float* partial, int64_t n_slots, int64_t stride,
                                                       int64_t n_elem, float scale, float* out) {
  __shared__ float sh[16][64];
  const int el = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int64_t e = (int64_t)blockIdx.x * 64 + el;
  float s = 0.f;
  if (e < n_elem)
    for (int64_t k = grp; k < n_slots; k += 16) s += partial[k * stride + e];
  sh[grp][el] = s;
  __syncthreads();
  if (grp == 0 && e < n_elem) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) t += sh[g][el];
    out[e] = scale * t;
  }
}

// ---------------------------------------------------------------------------------------------
// Graph attention backward, row pass: for every covered row i, c_i^h = du_i^h . u_i^h and
// d s_dst_i^h = sum_j dpre_ij^h,  dpre = alpha (du_i^h . z_j^h - c_i^h) LeakyReLU'(e_ij^h).
// Lane = (neighbour slot lane/8, head lane%8): eight neighbours at a time, each lane reads its
// head's 32-byte slice of the neighbour's z row and does the 16-dim dot product on its own.
// Rows longer than long_nnz are cut into parts (one wavefront each) whose sums a merge kernel
// adds in part order.
constexpr int kLongRec = 144;    // floats per scratch record of a part of a split row (forward, row pass)

struct GatBwdRowsArgs {
  GraphDev g;
  const Segment* segs;
  const int32_t* work; int64_t n_work;
  const int32_t* work_long; int64_t n_long;
  int32_t long_nnz, part_nnz;
  float* long_partial;
  const uint16_t* zX; const uint16_t* zC;
  const float* sX; const float* sC;
  const float* U; const uint16_t* dU;
  const float* lse;
  float4* st2;    // [T*N][8]: per head (s_dst, lse, c, d s_dst): what the reverse-edge pass needs of a row
};

__device__ __forceinline__ void load16(const uint16_t* p, float* x) {
  unpack8(reinterpret_cast<const uint4*>(p)[0], x);
  unpack8(reinterpret_cast<const uint4*>(p)[1], x + 8);
}

// du_i^h (16 values) and c_i^h for the lane's head
__device__ __forceinline__ float load_du_c(const GatBwdRowsArgs& a, int64_t row, int h, float* du) {
  load16(a.dU + row * kS + 16 * h, du);
  float c = 0.f;
#pragma unroll
  for (int d4 = 0; d4 < 4; ++d4) {
    const float4 x = *reinterpret_cast<const float4*>(a.U + row * kS + 16 * h + 4 * d4);
    c += du[4 * d4] * x.x + du[4 * d4 + 1] * x.y + du[4 * d4 + 2] * x.z + du[4 * d4 + 3] * x.w;
  }
  return c;
}

// this lane's share (its neighbour slot) of sum_j dpre_ij^h over the non-zeros [e0, e1) of row i
__device__ __forceinline__ float gat_bwd_row_range(const GatBwdRowsArgs& a, const Segment& s, const int32_t* col,
                                                   int64_t base, const float* du, float c, float sd, float lse,
                                                   int64_t e0, int64_t e1, int lane) {
  const int slot = lane >> 3, h = lane & 7;
  float dsd = 0.f;
  for (int64_t eb = e0; eb < e1; eb += 64) {
    const int cnt = (int)min((int64_t)64, e1 - eb);
    const int32_t jl = lane < cnt ? col[eb + lane] : 0;
    for (int q0 = 0; q0 < cnt; q0 += 8) {
      const int32_t j = __shfl(jl, q0 + slot);
      if (q0 + slot < cnt) {
        const bool in = j >= s.v_lo && j < s.v_hi;
        float z[16];
        const uint16_t* zp = (in ? a.zX : a.zC) + (base + j) * kS + 16 * h;   // half precision
        unpackh8(reinterpret_cast<const uint4*>(zp)[0], z);
        unpackh8(reinterpret_cast<const uint4*>(zp)[1], z + 8);
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
  return dsd;
}

__global__ __launch_bounds__(256) void k_gat_bwd_rows(GatBwdRowsArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_work) return;
  const int32_t si = a.work[3 * item], r0 = a.work[3 * item + 1], nr = a.work[3 * item + 2];
  const Segment s = a.segs[si];
  const int64_t* rowptr = a.g.rowptr[s.t];
  const int32_t* col = a.g.colidx[s.t];
  const int64_t base = (int64_t)s.t * a.g.N;
  const int slot = lane >> 3, h = lane & 7;
  for (int rr = 0; rr < nr; ++rr) {
    const int64_t i = s.v_lo + r0 + rr;
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    if (e1 - e0 > a.long_nnz) continue;
    float du[16];
    const float c = load_du_c(a, base + i, h, du);
    const float sd = a.sX[(base + i) * 16 + 8 + h], lse = a.lse[(base + i) * 8 + h];
    const float dsd = gat_bwd_row_range(a, s, col, base, du, c, sd, lse, e0, e1, lane);
    if (slot == 0) a.st2[(base + i) * 8 + h] = make_float4(sd, lse, c, dsd);
  }
}

__global__ __launch_bounds__(256) void k_gat_bwd_rows_long(GatBwdRowsArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_long) return;
  const int32_t* w = a.work_long + 4 * item;
  const Segment s = a.segs[w[0]];
  const int64_t i = s.v_lo + w[1];
  const int64_t* rowptr = a.g.rowptr[s.t];
  const int64_t base = (int64_t)s.t * a.g.N;
  const int slot = lane >> 3, h = lane & 7;
  const int64_t e0 = rowptr[i] + (int64_t)w[2] * a.part_nnz, e1 = min(rowptr[i + 1], e0 + a.part_nnz);
  float du[16];
  const float c = load_du_c(a, base + i, h, du);
  const float dsd = gat_bwd_row_range(a, s, a.g.colidx[s.t], base, du, c, a.sX[(base + i) * 16 + 8 + h],
                                      a.lse[(base + i) * 8 + h], e0, e1, lane);
  if (slot == 0) {
    a.long_partial[item * kLongRec + h] = dsd;
    a.long_partial[item * kLongRec + 8 + h] = c;
  }
}

__global__ void k_gat_bwd_rows_merge(GatBwdRowsArgs a) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t item = idx >> 3;
  const int h = (int)(idx & 7);
  if (item >= a.n_long) return;
  const int32_t* w = a.work_long + 4 * item;
  if (w[2] != 0) return;
  const Segment s = a.segs[w[0]];
  float dsd = 0.f;
  for (int p = 0; p < w[3]; ++p) dsd += a.long_partial[(item + p) * kLongRec + h];
  const int64_t row = (int64_t)s.t * a.g.N + s.v_lo + w[1];
  a.st2[row * 8 + h] = make_float4(a.sX[row * 16 + 8 + h], a.lse[row * 8 + h], a.long_partial[item * kLongRec + 8 + h], dsd);
}

// Graph attention backward, reverse-edge pass: for every vertex j of every snapshot in use, the
// gradients of its two projections (z_j as seen from inside its own chunk: zX; as an
// out-of-chunk neighbour: zC) are gathered over the rows i that list j, i.e. over j's own stored
// row (the adjacency is symmetric):
//   dz_j += alpha_ij du_i,   d s_src_j^h += dpre_ij^h,
// then  dzX_j += d s_dst_j a_dst + d s_srcX_j a_src,  dzC_j += d s_srcC_j a_src, and the gradients
// of a_src, a_dst are accumulated per wave.  Lanes span the 128 features (two per lane).  Long
// rows are split as in the other passes (list of (snapshot, vertex, part, parts)).
struct GatBwdColsArgs {
  GraphDev g;
  const int32_t* used_t; int32_t n_used;
  const int32_t* owner;
  const uint8_t* ecode;          // per stored non-zero (j, i) of the snapshots in use: 0 = row i is not covered,
  const int64_t* ecode_off;      //   1 = i and j are rows of the same chunk, 2 = of different chunks; [T] first entry
  const int32_t* cols_long; int64_t n_cols_long;
  int32_t long_nnz, part_nnz;
  float* long_partial;
  const uint16_t* zX; const uint16_t* zC;
  const float* sX; const float* sC;
  const uint16_t* dU;
  const float4* st2;
  const float* a_src; const float* a_dst;
  uint16_t* dzX; uint16_t* dzC;
  uint16_t* dzXlo;      // nullptr, or: what dzX loses to rounding (for the input gradient)
  float* dss;           // [T*N][16]: d s_src of the row as an in-chunk neighbour [8], as a cache row [8]
};

constexpr int kSlotRow = 16;     // rows of at most this many non-zeros are taken one per slot (k_gat_bwd_cols_slot)
constexpr int kSlotU = 2;        // neighbours in flight per slot there (4 or 8, with fewer waves per SIMD, measured slower)
constexpr int kSlotWaves = 4;    // waves per SIMD of that kernel
constexpr int kColsRec = 272;    // floats per scratch record of a part of a split row: dzX[128], dzC[128], dsx[8], dsc[8]

// Lane layout of the reverse-edge pass: lane = 16 * slot + sub.  The four slots work on four
// neighbours at a time; the 16 sub-lanes of a slot span the 128 features (8 per lane, one
// 16-byte load), two sub-lanes per head.
struct ColOwn {      // what a lane keeps about the wave's own vertex j
  int32_t oj;
  float zx[8], zc[8], ssx, ssc;
};
struct ColAcc { float ax[8], ac[8], dsx, dsc; };

__device__ __forceinline__ float quad_xor1(float x) {   // value of lane l^1
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true));
}
// sum over the four slots (lanes l, l^16, l^32, l^48), same result in all of them
__device__ __forceinline__ float slot_sum(float x) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float y = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

__device__ __forceinline__ ColOwn col_own(const GatBwdColsArgs& a, int64_t row, int sub) {
  ColOwn o;
  const int head = sub >> 1;
  // zX / sX of a vertex no chunk covers hold stale values: they are never used (no neighbour
  // can be "of the same chunk"), and loading them unconditionally keeps the loads independent
  o.oj = a.owner[row];
  unpackh8(*reinterpret_cast<const uint4*>(a.zC + row * kS + 8 * sub), o.zc);
  unpackh8(*reinterpret_cast<const uint4*>(a.zX + row * kS + 8 * sub), o.zx);
  o.ssx = a.sX[row * 16 + head];
  o.ssc = a.sC[row * 8 + head];
  return o;
}

// contributions of the stored non-zeros [e0, e1) of row j; the four slots are already summed.
// il / cl: column id and code of non-zero e0 + lane (the first 64), loaded by the caller so that
// they are in flight while the previous row is being processed.
__device__ __forceinline__ ColAcc gat_bwd_col_range(const GatBwdColsArgs& a, const int32_t* col, const uint8_t* code,
                                                    int64_t base, const ColOwn& o, int64_t e0, int64_t e1,
                                                    int32_t il, int32_t cl, int lane) {
  const int slot = lane >> 4, sub = lane & 15, head = sub >> 1;
  ColAcc r;
#pragma unroll
  for (int d = 0; d < 8; ++d) { r.ax[d] = 0.f; r.ac[d] = 0.f; }
  r.dsx = 0.f; r.dsc = 0.f;
  for (int64_t eb = e0; eb < e1; eb += 64) {
    const int cnt = (int)min((int64_t)64, e1 - eb);
    if (eb != e0) {
      il = lane < cnt ? col[eb + lane] : 0;
      cl = lane < cnt ? code[eb + lane] : 0;
    }
    for (int q0 = 0; q0 < cnt; q0 += 8) {
      uint4 dv[2];
      float4 st[2];
      int32_t cc[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int idx = q0 + 4 * u + slot;
        const int32_t ii = __shfl(il, idx);
        const int32_t cs = __shfl(cl, idx);   // outside the select: every lane has to take part
        cc[u] = idx < cnt ? cs : 0;
        dv[u] = make_uint4(0, 0, 0, 0);
        st[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (cc[u] != 0) {
          dv[u] = *reinterpret_cast<const uint4*>(a.dU + (base + ii) * kS + 8 * sub);
          st[u] = a.st2[(base + ii) * 8 + head];
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float du[8];
        unpack8(dv[u], du);
        const bool sm = cc[u] == 1;
        const float e = st[u].x + (sm ? o.ssx : o.ssc);
        float al = __expf(lrelu(e) - st[u].y);
        float da = 0.f;
#pragma unroll
        for (int d = 0; d < 8; ++d) da += du[d] * (sm ? o.zx[d] : o.zc[d]);
        da += quad_xor1(da);
        al = cc[u] != 0 ? al : 0.f;
        const float dpre = al * (da - st[u].z) * (e > 0.f ? 1.f : kSlope);
        const float alx = sm ? al : 0.f, alc = sm ? 0.f : al;
#pragma unroll
        for (int d = 0; d < 8; ++d) {
          r.ax[d] += alx * du[d];
          r.ac[d] += alc * du[d];
        }
        r.dsx += sm ? dpre : 0.f;
        r.dsc += sm ? 0.f : dpre;
      }
    }
  }
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    r.ax[d] = slot_sum(r.ax[d]);
    r.ac[d] = slot_sum(r.ac[d]);
  }
  r.dsx = slot_sum(r.dsx);
  r.dsc = slot_sum(r.dsc);
  return r;
}

struct AttVec { float as[8], ad[8]; };

__device__ __forceinline__ AttVec att_init(const GatBwdColsArgs& a, int sub) {
  AttVec v;
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    v.as[d] = a.a_src[8 * sub + d];
    v.ad[d] = a.a_dst[8 * sub + d];
  }
  return v;
}

template <bool LO, bool EVERY_SLOT = false>   // LO: also keep what dzX loses to rounding (asked for with the input gradient)
__device__ __forceinline__ void gat_bwd_col_finish(const GatBwdColsArgs& a, int64_t row, const ColOwn& o,
                                                   const ColAcc& r, const AttVec& v, int lane) {
  const int slot = lane >> 4, sub = lane & 15, head = sub >> 1;
  if (!EVERY_SLOT && slot != 0) return;      // EVERY_SLOT: each slot holds a row of its own
  float out[8];
  if (o.oj >= 0) {
    const float dsd = a.st2[row * 8 + head].w;
#pragma unroll
    for (int d = 0; d < 8; ++d) out[d] = r.ax[d] + dsd * v.ad[d] + r.dsx * v.as[d];
    const bf16x8 hi = pack8(out);
    *reinterpret_cast<uint4*>(a.dzX + row * kS + 8 * sub) = __builtin_bit_cast(uint4, hi);
    if constexpr (LO) {
      float rest[8];
#pragma unroll
      for (int d = 0; d < 8; ++d) rest[d] = out[d] - (float)hi[d];
      *reinterpret_cast<uint4*>(a.dzXlo + row * kS + 8 * sub) = __builtin_bit_cast(uint4, pack8(rest));
    }
  }
#pragma unroll
  for (int d = 0; d < 8; ++d) out[d] = r.ac[d] + r.dsc * v.as[d];
  *reinterpret_cast<uint4*>(a.dzC + row * kS + 8 * sub) = __builtin_bit_cast(uint4, pack8(out));
  if ((sub & 1) == 0) {
    a.dss[row * 16 + head] = r.dsx;
    a.dss[row * 16 + 8 + head] = r.dsc;
  }
}

// Rows of at most kSlotRow non-zeros (nine vertices in ten of a power-law graph, a third of the
// non-zeros): ONE ROW PER SLOT, four rows per wave side by side.  What a row costs apart from its
// non-zeros (its own projections and scalars, the final combination and stores) is then paid once
// per four rows, and nothing has to be summed across the slots.  The 16 lanes of a slot first
// fetch the row's column ids and codes, one neighbour per lane, and hand them round with a
// shuffle inside the slot; two neighbours per slot are in flight (eight gathered rows per wave).
template <bool LO>
__global__ __launch_bounds__(256, kSlotWaves) void k_gat_bwd_cols_slot(GatBwdColsArgs a) {
  const int lane = threadIdx.x & 63, slot = lane >> 4, sub = lane & 15, head = sub >> 1;
  const int64_t N = a.g.N;
  const int64_t quads_per_t = (N + 3) / 4, n_items = quads_per_t * a.n_used;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= n_items) return;
  const int32_t t = a.used_t[item / quads_per_t];
  const int64_t j = (item % quads_per_t) * 4 + slot;
  const bool live = j < N;
  const int64_t base = (int64_t)t * N, row = base + (live ? j : N - 1);
  const int64_t* rp = a.g.rowptr[t] + (live ? j : N - 1);
  const int64_t e0 = rp[0], len = rp[1] - e0;
  const int n = (live && len <= kSlotRow && len <= a.long_nnz) ? (int)len : 0;     // 0: not this kernel's row
  const int32_t* col = a.g.colidx[t];
  const uint8_t* code = a.ecode + a.ecode_off[t];
  const int32_t il = sub < n ? col[e0 + sub] : 0;
  const int32_t cl = sub < n ? code[e0 + sub] : 0;
  const ColOwn o = col_own(a, row, sub);
  const AttVec v = att_init(a, sub);
  int nmax = __builtin_amdgcn_readlane(n, 0);
  nmax = max(nmax, __builtin_amdgcn_readlane(n, 16));
  nmax = max(nmax, __builtin_amdgcn_readlane(n, 32));
  nmax = max(nmax, __builtin_amdgcn_readlane(n, 48));
  ColAcc r;
#pragma unroll
  for (int d = 0; d < 8; ++d) { r.ax[d] = 0.f; r.ac[d] = 0.f; }
  r.dsx = 0.f; r.dsc = 0.f;
  for (int k0 = 0; k0 < nmax; k0 += kSlotU) {
    uint4 dv[kSlotU];
    float4 st[kSlotU];
    int32_t cc[kSlotU];
#pragma unroll
    for (int u = 0; u < kSlotU; ++u) {
      const int k = k0 + u;                              // < 16 + 1: the shuffle wraps inside the slot, the code is masked
      const int32_t ii = __shfl(il, (lane & 48) | (k & 15));
      const int32_t cs = __shfl(cl, (lane & 48) | (k & 15));
      cc[u] = k < n ? cs : 0;
      dv[u] = make_uint4(0, 0, 0, 0);
      st[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (cc[u] != 0) {
        dv[u] = *reinterpret_cast<const uint4*>(a.dU + (base + ii) * kS + 8 * sub);
        st[u] = a.st2[(base + ii) * 8 + head];
      }
    }
#pragma unroll
    for (int u = 0; u < kSlotU; ++u) {
      float du[8];
      unpack8(dv[u], du);
      const bool sm = cc[u] == 1;
      const float e = st[u].x + (sm ? o.ssx : o.ssc);
      float al = __expf(lrelu(e) - st[u].y);
      float da = 0.f;
#pragma unroll
      for (int d = 0; d < 8; ++d) da += du[d] * (sm ? o.zx[d] : o.zc[d]);
      da += quad_xor1(da);
      al = cc[u] != 0 ? al : 0.f;
      const float dpre = al * (da - st[u].z) * (e > 0.f ? 1.f : kSlope);
      const float alx = sm ? al : 0.f, alc = sm ? 0.f : al;
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        r.ax[d] += alx * du[d];
        r.ac[d] += alc * du[d];
      }
      r.dsx += sm ? dpre : 0.f;
      r.dsc += sm ? 0.f : dpre;
    }
  }
  if (n > 0) gat_bwd_col_finish<LO, true>(a, row, o, r, v, lane);
}

template <bool LO>
__global__ __launch_bounds__(256, 4) void k_gat_bwd_cols(GatBwdColsArgs a) {   // 4 waves per SIMD: 128 registers
  const int lane = threadIdx.x & 63;
  const int64_t N = a.g.N;
  const int64_t groups_per_t = (N + 15) / 16, n_items = groups_per_t * a.n_used;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= n_items) return;
  const int sub = lane & 15;
  const AttVec v = att_init(a, sub);
  const int32_t t = a.used_t[item / groups_per_t];
  const int64_t j0 = (item % groups_per_t) * 16;
  const int32_t* col = a.g.colidx[t];
  const uint8_t* code = a.ecode + a.ecode_off[t];
  const int64_t base = (int64_t)t * N;
  const int nr = (int)min((int64_t)16, N - j0);
  // row pointers of the whole group at once; the next row's column ids and codes are requested
  // before the current row is processed
  const int64_t rp = a.g.rowptr[t][j0 + min(lane, nr)];
  const int32_t rlo = (int32_t)(rp & 0xffffffff), rhi = (int32_t)(rp >> 32);
  auto row_ptr = [&](int r) {
    return ((int64_t)__builtin_amdgcn_readlane(rhi, r) << 32) | (uint32_t)__builtin_amdgcn_readlane(rlo, r);
  };
  int64_t e0 = row_ptr(0), e1 = row_ptr(1);
  int32_t il = e0 + lane < e1 ? col[e0 + lane] : 0;
  int32_t cl = e0 + lane < e1 ? code[e0 + lane] : 0;
  for (int rr = 0; rr < nr; ++rr) {
    int64_t ne0 = e1, ne1 = e1;
    int32_t nil = 0, ncl = 0;
    if (rr + 1 < nr) {
      ne1 = row_ptr(rr + 2);
      nil = ne0 + lane < ne1 ? col[ne0 + lane] : 0;
      ncl = ne0 + lane < ne1 ? code[ne0 + lane] : 0;
    }
    if (e1 - e0 <= a.long_nnz && e1 - e0 > kSlotRow) {     // shorter rows: k_gat_bwd_cols_slot
      const ColOwn o = col_own(a, base + j0 + rr, sub);
      const ColAcc r = gat_bwd_col_range(a, col, code, base, o, e0, e1, il, cl, lane);
      gat_bwd_col_finish<LO>(a, base + j0 + rr, o, r, v, lane);
    }
    e0 = ne0; e1 = ne1; il = nil; cl = ncl;
  }
}

__global__ __launch_bounds__(256) void k_gat_bwd_cols_long(GatBwdColsArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_cols_long) return;
  const int32_t* w = a.cols_long + 4 * item;   // snapshot, vertex, part, parts
  const int64_t base = (int64_t)w[0] * a.g.N, j = w[1];
  const int sub = lane & 15;
  const int64_t* rowptr = a.g.rowptr[w[0]];
  const int64_t e0 = rowptr[j] + (int64_t)w[2] * a.part_nnz, e1 = min(rowptr[j + 1], e0 + a.part_nnz);
  const ColOwn o = col_own(a, base + j, sub);
  const int32_t* col = a.g.colidx[w[0]];
  const uint8_t* code = a.ecode + a.ecode_off[w[0]];
  const int32_t il = e0 + lane < e1 ? col[e0 + lane] : 0;
  const int32_t cl = e0 + lane < e1 ? code[e0 + lane] : 0;
  const ColAcc r = gat_bwd_col_range(a, col, code, base, o, e0, e1, il, cl, lane);
  if ((lane >> 4) == 0) {
    float* rec = a.long_partial + item * kColsRec;
    float4* x = reinterpret_cast<float4*>(rec + 8 * sub);
    x[0] = make_float4(r.ax[0], r.ax[1], r.ax[2], r.ax[3]);
    x[1] = make_float4(r.ax[4], r.ax[5], r.ax[6], r.ax[7]);
    float4* c = reinterpret_cast<float4*>(rec + kS + 8 * sub);
    c[0] = make_float4(r.ac[0], r.ac[1], r.ac[2], r.ac[3]);
    c[1] = make_float4(r.ac[4], r.ac[5], r.ac[6], r.ac[7]);
    if ((sub & 1) == 0) {
      rec[256 + (sub >> 1)] = r.dsx;
      rec[264 + (sub >> 1)] = r.dsc;
    }
  }
}

template <bool LO>
__global__ __launch_bounds__(256) void k_gat_bwd_cols_merge(GatBwdColsArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_cols_long) return;
  const int32_t* w = a.cols_long + 4 * item;
  if (w[2] != 0) return;
  const int sub = lane & 15;
  const AttVec v = att_init(a, sub);
  const int64_t row = (int64_t)w[0] * a.g.N + w[1];
  ColAcc r;
#pragma unroll
  for (int d = 0; d < 8; ++d) { r.ax[d] = 0.f; r.ac[d] = 0.f; }
  r.dsx = 0.f; r.dsc = 0.f;
  for (int p = 0; p < w[3]; ++p) {
    const float* rec = a.long_partial + (item + p) * kColsRec;
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      r.ax[d] += rec[8 * sub + d];
      r.ac[d] += rec[kS + 8 * sub + d];
    }
    r.dsx += rec[256 + (sub >> 1)];
    r.dsc += rec[264 + (sub >> 1)];
  }
  const ColOwn o = col_own(a, row, sub);
  gat_bwd_col_finish<LO>(a, row, o, r, v, lane);
}

// Gradients of the attention vectors, a streaming pass over every vertex of the snapshots in use:
//   d a_dst^h += d s_dst_i^h z_i^h (covered rows, own projection),
//   d a_src^h += d s_srcX_i^h zX_i^h (covered rows) + d s_srcC_i^h zC_i^h (all rows).
// Lanes span the 128 features; each wave walks rows with a grid stride and leaves its sums in its
// own slot.
struct AttGradArgs {
  const int32_t* used_t; int32_t n_used; int64_t N;
  const int32_t* owner;
  const uint16_t* zX; const uint16_t* zC;
  const float4* st2; const float* dss;
  float* da_partial;    // [waves][2][128]: d a_src, d a_dst
};

__global__ __launch_bounds__(256) void k_att_grad(AttGradArgs a) {
  const int lane = threadIdx.x & 63, head = lane >> 3;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
  const int64_t n_rows = a.N * a.n_used;
  float gs0 = 0.f, gs1 = 0.f, gd0 = 0.f, gd1 = 0.f;
  for (int64_t r0 = wave * 8; r0 < n_rows; r0 += n_waves * 8) {
    // eight rows in flight: all loads first (rows past the end and the input-side data of rows no
    // chunk covers are read from a valid row and weighted by zero)
    uint32_t zc[8], zx[8];
    float dsc[8], dsx[8], dsd[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int64_t idx = min(r0 + k, n_rows - 1);
      const int64_t row = (int64_t)a.used_t[idx / a.N] * a.N + idx % a.N;
      const float live = r0 + k < n_rows ? 1.f : 0.f;
      const float cov = a.owner[row] >= 0 ? live : 0.f;
      zc[k] = *reinterpret_cast<const uint32_t*>(a.zC + row * kS + 2 * lane);
      zx[k] = *reinterpret_cast<const uint32_t*>(a.zX + row * kS + 2 * lane);
      dsc[k] = live * a.dss[row * 16 + 8 + head];
      dsx[k] = cov * a.dss[row * 16 + head];
      dsd[k] = cov * a.st2[row * 8 + head].w;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      // 0 * (stale value) must stay 0: the input-side buffers of uncovered rows are never written
      const float x0 = dsx[k] != 0.f || dsd[k] != 0.f ? h_lo(zx[k]) : 0.f;
      const float x1 = dsx[k] != 0.f || dsd[k] != 0.f ? h_hi(zx[k]) : 0.f;
      gs0 += dsc[k] * h_lo(zc[k]) + dsx[k] * x0;
      gs1 += dsc[k] * h_hi(zc[k]) + dsx[k] * x1;
      gd0 += dsd[k] * x0;
      gd1 += dsd[k] * x1;
    }
  }
  float* o = a.da_partial + wave * 2 * kS;
  o[2 * lane] = gs0; o[2 * lane + 1] = gs1;
  o[kS + 2 * lane] = gd0; o[kS + 2 * lane + 1] = gd1;
}

// code of every stored non-zero (j, i) of snapshot t: see GatBwdColsArgs
__global__ void k_edge_code(GraphDev g, const int32_t* used_t, int32_t n_used, const int32_t* owner,
                            const int64_t* ecode_off, uint8_t* ecode) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= g.N * n_used) return;
  const int32_t t = used_t[idx / g.N];
  const int64_t j = idx % g.N, base = (int64_t)t * g.N;
  const int32_t oj = owner[base + j];
  const int32_t* col = g.colidx[t];
  uint8_t* out = ecode + ecode_off[t];
  for (int64_t e = g.rowptr[t][j]; e < g.rowptr[t][j + 1]; ++e) {
    const int32_t oi = owner[base + col[e]];
    out[e] = oi < 0 ? 0 : (oi == oj ? 1 : 2);
  }
}

// list of the split rows of the reverse-edge pass: count, then fill (the order of the rows in
// the list is arbitrary; the parts of a row are consecutive)
__global__ void k_cols_long(GraphDev g, const int32_t* used_t, int32_t n_used, int32_t long_nnz, int32_t part_nnz,
                            int32_t* counter, int32_t* list) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= g.N * n_used) return;
  const int32_t t = used_t[idx / g.N];
  const int64_t v = idx % g.N;
  const int64_t deg = g.rowptr[t][v + 1] - g.rowptr[t][v];
  if (deg <= long_nnz) return;
  const int32_t parts = (int32_t)((deg + part_nnz - 1) / part_nnz);
  const int32_t at = atomicAdd(counter, parts);
  if (!list) return;
  for (int32_t p = 0; p < parts; ++p) {
    list[4 * (at + p)] = t; list[4 * (at + p) + 1] = (int32_t)v;
    list[4 * (at + p) + 2] = p; list[4 * (at + p) + 3] = parts;
  }
}

}  // namespace

namespace {
constexpr int kDwGroups = 256;     // workgroups (slots) of the weight-gradient kernel
constexpr int kTbwdWaves = 2048;   // waves (slots) of the temporal backward kernel
constexpr int kColsBlocks = 1024;  // workgroups of the reverse-edge pass (4 slots each)

// Gradient of the input rows: the projection is z = W x, so dx = W^T dz, i.e. dX[row] = dzX[row] W for
// every covered row (a row no chunk covers is never an input row; it is not written).  Same
// tiling as the projection: one wave per 32 vertices of a snapshot, dzX rows as the second operand
// straight from memory, fragments of W^T as the first.
struct GatDxArgs {
  const uint16_t* dzX; const uint16_t* dzXlo;
  const uint4* WT; const uint4* WTlo;
  const int32_t* owner; const int32_t* used_t; int32_t n_used; int64_t N;
  uint16_t* dX; int64_t lddx;
};

__global__ __launch_bounds__(256) void k_gat_dx(GatDxArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hh = lane >> 5;
  const int64_t tiles_per_t = (a.N + 31) / 32;
  const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
  if (tile >= tiles_per_t * a.n_used) return;
  const int32_t t = a.used_t[tile / tiles_per_t];
  const int64_t v = (tile % tiles_per_t) * 32 + n;
  const bool valid = v < a.N;
  const int64_t row = (int64_t)t * a.N + (valid ? v : a.N - 1);
  const bool covered = valid && a.owner[row] >= 0;
  if (__ballot(covered) == 0ull) return;
  // both operands as a bf16 value plus what it lost to rounding: a row's gradient is one sum of
  // 128 terms, nothing averages the roundings out as the sums over rows of the weight gradients do
  bf16x8 gf[8], gl[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    // rows no chunk covers hold no gradient (their dzX was never written): zeros
    uint4 raw = make_uint4(0, 0, 0, 0), rawl = raw;
    if (covered) {
      raw = *reinterpret_cast<const uint4*>(a.dzX + row * kS + ks * 16 + 8 * hh);
      rawl = *reinterpret_cast<const uint4*>(a.dzXlo + row * kS + ks * 16 + 8 * hh);
    }
    gf[ks] = as_frag(raw);
    gl[ks] = as_frag(rawl);
  }
#pragma unroll
  for (int ib = 0; ib < 4; ++ib) {
    floatx16 acc = {};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 wh = as_frag(a.WT[(ib * 8 + ks) * 64 + lane]), wl = as_frag(a.WTlo[(ib * 8 + ks) * 64 + lane]);
      acc = mfma(wl, gf[ks], acc);
      acc = mfma(wh, gl[ks], acc);
      acc = mfma(wh, gf[ks], acc);
    }
    if (covered) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<uint2*>(a.dX + row * a.lddx + ib * 32 + 8 * g + 4 * hh) =
            pack4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
    }
  }
}

}  // namespace

// scratch layout: [weight-gradient slots | position-gradient slots | attention-vector slots]
int64_t dysat_partial_elems(const DysatWs& ws) {
  return (int64_t)kDwGroups * 3 * kS * kS + (int64_t)kTbwdWaves * ws.T * kS +
         (int64_t)kColsBlocks * 4 * 2 * kS;
}
int64_t dysat_long_partial_elems(const DysatWs& ws) {
  return std::max<int64_t>(ws.n_long * kLongRec, ws.n_cols_long * kColsRec);
}
void dysat_edge_code(const GraphDev& g, const int32_t* used_t, int32_t n_used, const int32_t* owner,
                     const int64_t* ecode_off, uint8_t* ecode, hipStream_t st) {
  hipLaunchKernelGGL(k_edge_code, blocks_for(g.N * n_used, 256), 256, 0, st, g, used_t, n_used, owner, ecode_off, ecode);
}
void dysat_cols_long(const GraphDev& g, const int32_t* used_t, int32_t n_used, int32_t long_nnz, int32_t part_nnz,
                     int32_t* counter, int32_t* list, hipStream_t st) {
  hipLaunchKernelGGL(k_cols_long, blocks_for(g.N * n_used, 256), 256, 0, st, g, used_t, n_used, long_nnz, part_nnz,
                     counter, list);
}
int64_t dysat_loss_partial_elems(const DysatWs&) { return kTbwdWaves; }

void dysat_backward(const DysatWs& ws, const void* Y, int64_t ldy, const void* dY, int64_t lddy, const void* target,
                    int64_t ldt, float* loss_out, void* dX, int64_t lddx, hipEvent_t* ev, hipStream_t st) {
  float* dw_slots = ws.partial;
  float* dpos_slots = dw_slots + (int64_t)kDwGroups * 3 * kS * kS;
  float* da_slots = dpos_slots + (int64_t)kTbwdWaves * ws.T * kS;
  const int64_t count = ws.total_rows * kS;
  const int64_t tiles32 = (ws.N + 31) / 32 * ws.n_used;
  const int groups = (int)std::min<int64_t>(kDwGroups, tiles32);

  // (1) temporal attention: dQ, dK, dV (+ loss), then dP -> dU and the position-table gradient
  const size_t lds = sizeof(uint4) * 3 * kFragsPerW;
  {
    static bool attr_set = false;   // dynamic LDS above 64 KB has to be allowed once per kernel
    if (!attr_set) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_temporal_bwd<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_temporal_bwd<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_temporal_bwd2),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      attr_set = true;
    }
  }
  const int grid_a = (int)std::min<int64_t>(256, (ws.n_tiles + 3) / 4);
  const int grid_b = (int)std::min<int64_t>(kTbwdWaves / 8, (tiles32 + 7) / 8);
  const int n_tw = grid_b * 8;
  hipLaunchKernelGGL(k_fill_f32, blocks_for((int64_t)n_tw * ws.T * kS, 256), 256, 0, st, dpos_slots, 0.f,
                     (int64_t)n_tw * ws.T * kS);
  if (ev) (void)hipEventRecord(ev[0], st);
  TemporalBwdArgs ta{};
  ta.chunks = ws.chunks; ta.n_chunks = ws.n_chunks; ta.tile_ptr = ws.tile_ptr; ta.n_tiles = ws.n_tiles;
  ta.N = ws.N; ta.T = ws.T; ta.U = ws.U; ta.pos = ws.P[DY_POS];
  ta.Wq = ws.Wqp; ta.Wk = ws.Wkp; ta.Wv = ws.Wvp;
  ta.Y = static_cast<const uint16_t*>(Y); ta.ldy = ldy;
  ta.dY = static_cast<const uint16_t*>(dY); ta.lddy = lddy;
  ta.target = static_cast<const uint16_t*>(target); ta.ldt = ldt;
  ta.scale = 2.0f / (float)count;
  ta.dQ = ws.dQ; ta.dK = ws.dK; ta.dV = ws.dV;
  ta.loss_partial = ws.loss_partial;
  if (ws.wide) hipLaunchKernelGGL(k_temporal_bwd<true>, grid_a, 256, lds, st, ta);
  else hipLaunchKernelGGL(k_temporal_bwd<false>, grid_a, 256, lds, st, ta);
  if (target && loss_out)
    hipLaunchKernelGGL(k_reduce_slots, 1, 1024, 0, st, ws.loss_partial, (int64_t)grid_a * 4, (int64_t)1, (int64_t)1,
                       1.0f / (float)count, loss_out);
  TemporalBwd2Args tb{};
  tb.used_t = ws.used_t; tb.n_used = ws.n_used; tb.N = ws.N; tb.T = ws.T; tb.owner = ws.owner; tb.U = ws.U;
  tb.WqT = ws.WqT; tb.WkT = ws.WkT; tb.WvT = ws.WvT; tb.dQ = ws.dQ; tb.dK = ws.dK; tb.dV = ws.dV;
  tb.dU = ws.dU; tb.dpos_partial = dpos_slots;
  hipLaunchKernelGGL(k_temporal_bwd2, grid_b, 512, lds, st, tb);
  hipLaunchKernelGGL(k_reduce_slots, blocks_for((int64_t)ws.T * kS, 64), 1024, 0, st, dpos_slots, (int64_t)n_tw,
                     (int64_t)ws.T * kS, (int64_t)ws.T * kS, 1.f, ws.G[DY_POS]);
  // (2) dW_q, dW_k, dW_v = sum over rows of d{q,k,v}^T P
  DwBf16Args da{};
  da.used_t = ws.used_t; da.n_used = ws.n_used; da.N = ws.N; da.owner = ws.owner; da.covered_only = 1;
  da.A = nullptr; da.lda = 0; da.Uf = ws.U; da.pos = ws.P[DY_POS];
  da.G[0] = ws.dQ; da.G[1] = ws.dK; da.G[2] = ws.dV;
  da.partial = dw_slots; da.n_groups = groups;
  {  // LDS: the position rows of the snapshots one workgroup's tile range can touch
    const int64_t tiles_per_t = (ws.N + 31) / 32, n_tiles = tiles_per_t * ws.n_used;
    const int64_t per = (n_tiles + groups - 1) / groups;
    const size_t pos_lds = sizeof(float) * kS * (size_t)((per + tiles_per_t - 1) / tiles_per_t + 1);
    hipLaunchKernelGGL((k_dw_bf16<3, true>), groups, 512, pos_lds, st, da);
  }
  for (int gi = 0; gi < 3; ++gi)
    hipLaunchKernelGGL(k_reduce_slots, blocks_for(kS * kS, 64), 1024, 0, st, dw_slots + (int64_t)gi * kS * kS,
                       (int64_t)groups, (int64_t)3 * kS * kS, (int64_t)kS * kS, 1.f, ws.G[DY_WQ + gi]);
  if (ev) (void)hipEventRecord(ev[1], st);
  // (3) graph attention, row pass
  GatBwdRowsArgs ra{};
  ra.g = ws.g; ra.segs = ws.segs; ra.work = ws.work_short; ra.n_work = ws.n_short;
  ra.zX = ws.zX; ra.zC = ws.zC; ra.sX = ws.sX; ra.sC = ws.sC; ra.U = ws.U; ra.dU = ws.dU; ra.lse = ws.lse;
  ra.st2 = reinterpret_cast<float4*>(ws.st2);
  ra.work_long = ws.work_long; ra.n_long = ws.n_long; ra.long_nnz = ws.long_nnz; ra.part_nnz = ws.part_nnz;
  ra.long_partial = ws.long_partial;
  hipLaunchKernelGGL(k_gat_bwd_rows, blocks_for(ws.n_short, 4), 256, 0, st, ra);
  if (ws.n_long > 0) {
    hipLaunchKernelGGL(k_gat_bwd_rows_long, blocks_for(ws.n_long, 4), 256, 0, st, ra);
    hipLaunchKernelGGL(k_gat_bwd_rows_merge, blocks_for(ws.n_long * 8, 256), 256, 0, st, ra);
  }
  if (ev) (void)hipEventRecord(ev[2], st);
  // (4) reverse-edge pass, then the gradients of the attention vectors
  const int64_t items = (ws.N + 15) / 16 * ws.n_used;
  GatBwdColsArgs ca{};
  ca.g = ws.g; ca.used_t = ws.used_t; ca.n_used = ws.n_used; ca.owner = ws.owner;
  ca.ecode = ws.ecode; ca.ecode_off = ws.ecode_off;
  ca.zX = ws.zX; ca.zC = ws.zC; ca.sX = ws.sX; ca.sC = ws.sC; ca.dU = ws.dU;
  ca.st2 = reinterpret_cast<const float4*>(ws.st2);
  ca.a_src = ws.P[DY_ASRC]; ca.a_dst = ws.P[DY_ADST];
  ca.dzX = ws.dzX; ca.dzC = ws.dzC; ca.dss = ws.dss;
  ca.dzXlo = dX ? ws.dzXlo : nullptr;
  ca.cols_long = ws.cols_long; ca.n_cols_long = ws.n_cols_long; ca.long_nnz = ws.long_nnz; ca.part_nnz = ws.part_nnz;
  ca.long_partial = ws.long_partial;
  const int64_t quads = (ws.N + 3) / 4 * ws.n_used;
  if (dX) hipLaunchKernelGGL(k_gat_bwd_cols_slot<true>, blocks_for(quads, 4), 256, 0, st, ca);
  else hipLaunchKernelGGL(k_gat_bwd_cols_slot<false>, blocks_for(quads, 4), 256, 0, st, ca);
  if (dX) hipLaunchKernelGGL(k_gat_bwd_cols<true>, blocks_for(items, 4), 256, 0, st, ca);
  else hipLaunchKernelGGL(k_gat_bwd_cols<false>, blocks_for(items, 4), 256, 0, st, ca);
  if (ws.n_cols_long > 0) {
    hipLaunchKernelGGL(k_gat_bwd_cols_long, blocks_for(ws.n_cols_long, 4), 256, 0, st, ca);
    if (dX) hipLaunchKernelGGL(k_gat_bwd_cols_merge<true>, blocks_for(ws.n_cols_long, 4), 256, 0, st, ca);
    else hipLaunchKernelGGL(k_gat_bwd_cols_merge<false>, blocks_for(ws.n_cols_long, 4), 256, 0, st, ca);
  }
  AttGradArgs ag{};
  ag.used_t = ws.used_t; ag.n_used = ws.n_used; ag.N = ws.N; ag.owner = ws.owner; ag.zX = ws.zX; ag.zC = ws.zC;
  ag.st2 = reinterpret_cast<const float4*>(ws.st2); ag.dss = ws.dss; ag.da_partial = da_slots;
  const int ablocks = (int)std::min<int64_t>(kColsBlocks, (ws.N * ws.n_used + 31) / 32);
  hipLaunchKernelGGL(k_att_grad, ablocks, 256, 0, st, ag);
  const int64_t da_n = (int64_t)ablocks * 4;
  hipLaunchKernelGGL(k_reduce_slots, 2, 1024, 0, st, da_slots, da_n, (int64_t)2 * kS, (int64_t)kS, 1.f, ws.G[DY_ASRC]);
  hipLaunchKernelGGL(k_reduce_slots, 2, 1024, 0, st, da_slots + kS, da_n, (int64_t)2 * kS, (int64_t)kS, 1.f,
                     ws.G[DY_ADST]);
  // (5) dW = sum over covered rows of dzX^T x  +  sum over all rows of dzC^T c
  DwBf16Args dx = da;
  dx.A = static_cast<const uint16_t*>(ws.X); dx.lda = ws.ldx; dx.Uf = nullptr; dx.covered_only = 1;
  dx.G[0] = ws.dzX; dx.partial = dw_slots;
  hipLaunchKernelGGL((k_dw_bf16<1, false>), groups, 512, 0, st, dx);
  DwBf16Args dc = dx;
  dc.A = static_cast<const uint16_t*>(ws.C); dc.lda = ws.ldc; dc.covered_only = 0;
  dc.G[0] = ws.dzC; dc.partial = dw_slots + (int64_t)groups * kS * kS;
  hipLaunchKernelGGL((k_dw_bf16<1, false>), groups, 512, 0, st, dc);
  hipLaunchKernelGGL(k_reduce_slots, blocks_for(kS * kS, 64), 1024, 0, st, dw_slots, (int64_t)2 * groups,
                     (int64_t)kS * kS, (int64_t)kS * kS, 1.f, ws.G[DY_W]);
  // (6) optional: the gradient of the input rows, dX = dzX W (covered rows only)
  if (dX) {
    GatDxArgs xa{};
    xa.dzX = ws.dzX; xa.dzXlo = ws.dzXlo; xa.WT = ws.WT; xa.WTlo = ws.WTlo; xa.owner = ws.owner; xa.used_t = ws.used_t; xa.n_used = ws.n_used; xa.N = ws.N;
    xa.dX = static_cast<uint16_t*>(dX); xa.lddx = lddx;
    hipLaunchKernelGGL(k_gat_dx, blocks_for((ws.N + 31) / 32 * ws.n_used, 4), 256, 0, st, xa);
  }
  if (ev) (void)hipEventRecord(ev[3], st);
}

}  // namespace dgc
