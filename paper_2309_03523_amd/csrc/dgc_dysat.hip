// Graph-attention structure encoder + causal temporal self-attention time encoder (the
// DySAT-style DGNN of the paper's Sections 2.1 and 6) over a fused batch of chunks, bf16 storage
// with fp32 accumulation: forward pass.  S = F = 128, 8 heads of 16 dims, windows of up to 32
// snapshots.
//
//   z = W x (own rows) / W c (cache rows, Section 5.2);  e_ij^h = LeakyReLU_0.2(a_dst^h.z_i^h + a_src^h.z_j^h)
//   alpha = softmax over the stored row;  u_i = sum_j alpha_ij z_j;  g = ELU(u)
//   p_s = g_s + pos[s];  q, k, v = W_q p, W_k p, W_v p;  y_s^h = sum_{r<=s} softmax_r(q_s^h.k_r^h / 4) v_r^h
#include "dgc_dysat_dev.h"

namespace dgc {
using namespace dysat;
namespace {

// ---------------------------------------------------------------------------------------------
// Weights [n_out = 128][n_in = 128] fp32 -> bf16 operand fragments, 16 bytes per lane.
//  mode 0: fragment (jb, kb) of W as the 32-row operand: lane l holds W[32 jb + l%32][16 kb + 8 (l/32) + 0..7].
//  mode 1: fragment (ib, ks) of W^T, for products whose contraction index is W's row index:
//          lane l holds W[16 ks + 8 (l/32) + 0..7][32 ib + l%32].
//  mode 2: as mode 1, of what W loses when it is rounded to bf16 (the low part).
__global__ void k_pack_w_bf16(const float* W, uint4* packed, int mode) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;   // (blk * 8 + k) * 64 + lane
  if (idx >= 4 * 8 * 64) return;
  const int lane = idx & 63, k = (idx >> 6) & 7, blk = idx >> 9;
  const int r32 = lane & 31, hh = lane >> 5;
  float x[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    if (mode == 0) x[p] = W[(blk * 32 + r32) * kS + k * 16 + 8 * hh + p];
    else x[p] = W[(k * 16 + 8 * hh + p) * kS + blk * 32 + r32];
  }
  if (mode == 2) {
    bf16x8 hi, lo;
    split8(x, hi, lo);
    packed[idx] = __builtin_bit_cast(uint4, lo);
  } else {
    packed[idx] = __builtin_bit_cast(uint4, pack8(x));
  }
}

__global__ void k_fill_i32(int32_t* p, int32_t v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// owner[t*N + v] = chunk that covers (t, v); one block per segment
__global__ void k_owner(const Segment* segs, int64_t N, int32_t* owner) {
  const Segment s = segs[blockIdx.x];
  for (int64_t v = s.v_lo + threadIdx.x; v < s.v_hi; v += blockDim.x) owner[(int64_t)s.t * N + v] = s.chunk;
}

// ---------------------------------------------------------------------------------------------
// Projection z = W x for every vertex of every snapshot in use: zC from the cache rows (any
// vertex can be somebody's out-of-chunk neighbour), zX from the input rows of covered vertices,
// plus the attention scalars s_src[h] = a_src^h . z^h, s_dst[h] = a_dst^h . z^h (from the fp32
// accumulators).  One wavefront per 32 vertices.
struct ProjArgs {
  const uint16_t* X; int64_t ldx;
  const uint16_t* C; int64_t ldc;
  const uint4* Wp;
  const float* a_src; const float* a_dst;
  const int32_t* owner; const int32_t* used_t; int32_t n_used; int64_t N;
  uint16_t* zX; uint16_t* zC;   // half precision
  float* sX;   // [T*N][16]: s_src[8], s_dst[8]
  float* sC;   // [T*N][8]:  s_src
};

__global__ __launch_bounds__(256) void k_gat_project(ProjArgs a) {
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
  const bool any_cov = __ballot(covered) != 0ull;
  for (int side = 0; side < 2; ++side) {          // 0: cache rows, 1: input rows
    if (side == 1 && !any_cov) break;
    const uint16_t* src = side ? a.X + row * a.ldx : a.C + row * a.ldc;
    const bool wr = side ? covered : valid;
    bf16x8 xf[8];
#pragma unroll
    for (int kb = 0; kb < 8; ++kb) xf[kb] = as_frag(*reinterpret_cast<const uint4*>(src + kb * 16 + 8 * hh));
    uint16_t* z = (side ? a.zX : a.zC) + row * kS;
    float ssrc[kHeads], sdst[kHeads];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      floatx16 acc = {};
#pragma unroll
      for (int kb = 0; kb < 8; ++kb) acc = mfma(as_frag(a.Wp[(jb * 8 + kb) * 64 + lane]), xf[kb], acc);
      if (wr) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<uint2*>(z + jb * 32 + 8 * g + 4 * hh) = packh4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
      }
#pragma unroll
      for (int hd = 0; hd < 2; ++hd) {
        const int h = 2 * jb + hd;
        float ps = 0.f, pd = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const float4 as = *reinterpret_cast<const float4*>(a.a_src + h * kD + 8 * c + 4 * hh);
          const float4 ad = *reinterpret_cast<const float4*>(a.a_dst + h * kD + 8 * c + 4 * hh);
          const int r = 8 * hd + 4 * c;
          ps += as.x * acc[r] + as.y * acc[r + 1] + as.z * acc[r + 2] + as.w * acc[r + 3];
          pd += ad.x * acc[r] + ad.y * acc[r + 1] + ad.z * acc[r + 2] + ad.w * acc[r + 3];
        }
        ssrc[h] = ps + __shfl_xor(ps, 32);
        sdst[h] = pd + __shfl_xor(pd, 32);
      }
    }
    if (wr) {
      if (side == 0) {
        if (hh == 0) {
          float4* o = reinterpret_cast<float4*>(a.sC + row * 8);
          o[0] = make_float4(ssrc[0], ssrc[1], ssrc[2], ssrc[3]);
          o[1] = make_float4(ssrc[4], ssrc[5], ssrc[6], ssrc[7]);
        }
      } else {
        float4* o = reinterpret_cast<float4*>(a.sX + row * 16 + 8 * hh);
        const float* s = hh ? sdst : ssrc;
        o[0] = make_float4(s[0], s[1], s[2], s[3]);
        o[1] = make_float4(s[4], s[5], s[6], s[7]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Edge softmax + aggregation.  One wavefront per group of rows of one segment; the 64 lanes span
// the 128 features (two per lane, head = lane / 8), so a neighbour's z row is one coalesced
// 256-byte load.  Column ids are loaded 64 at a time and broadcast lane by lane (row addresses
// stay wave-uniform); eight neighbour rows are in flight; the softmax is accumulated online
// (running maximum, rescale once per batch of eight).  Rows longer than long_nnz (hubs of the
// power-law graphs) are cut into parts of part_nnz non-zeros, one wavefront each; a part leaves
// its (maximum, sum, weighted sum) in a scratch record and a second kernel merges the records of
// a row in part order.
struct GatArgs {
  GraphDev g;
  const Segment* segs;
  const int32_t* work; int64_t n_work;     // [n][3]: segment, first local row, rows
  const int32_t* work_long; int64_t n_long;   // [n][4]: segment, local row, part, parts
  int32_t long_nnz, part_nnz;
  float* long_partial;                     // [n_long][kLongRec]
  const uint16_t* zX; const uint16_t* zC;
  const float* sX; const float* sC;
  float* U;        // [T*N][128] pre-ELU output (fp32: every later stage is sensitive to it)
  float* lse;      // [T*N][8] log-sum-exp of the logits of every (row, head)
};

struct SoftAcc { float m, l, a0, a1; };

// online softmax-weighted sum over the stored non-zeros [e0, e1) of row i of segment s
__device__ __forceinline__ SoftAcc gat_row_range(const GatArgs& a, const Segment& s, const int32_t* col, int64_t base,
                                                 float sd, int64_t e0, int64_t e1, int lane, int head) {
  SoftAcc r{-INFINITY, 0.f, 0.f, 0.f};
  for (int64_t eb = e0; eb < e1; eb += 64) {
    const int cnt = (int)min((int64_t)64, e1 - eb);
    const int32_t j = lane < cnt ? col[eb + lane] : 0;
    const int inside = (j >= s.v_lo && j < s.v_hi) ? 1 : 0;
    for (int q0 = 0; q0 < cnt; q0 += 8) {
      uint32_t zz[8];
      float ev[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        ev[q] = -INFINITY;
        zz[q] = 0u;
        if (q0 + q < cnt) {
          const int64_t jq = base + __builtin_amdgcn_readlane(j, q0 + q);
          const bool in = __builtin_amdgcn_readlane(inside, q0 + q) != 0;
          zz[q] = *reinterpret_cast<const uint32_t*>((in ? a.zX : a.zC) + jq * kS + 2 * lane);
          ev[q] = in ? a.sX[jq * 16 + head] : a.sC[jq * 8 + head];
        }
      }
      float bm = -INFINITY;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        ev[q] = lrelu(sd + ev[q]);       // -inf stays -inf
        bm = fmaxf(bm, ev[q]);
      }
      const float mn = fmaxf(r.m, bm);
      const float sc = __expf(r.m - mn);
      r.l *= sc; r.a0 *= sc; r.a1 *= sc;
      r.m = mn;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float p = __expf(ev[q] - mn);
        r.l += p;
        r.a0 += p * h_lo(zz[q]);
        r.a1 += p * h_hi(zz[q]);
      }
    }
  }
  return r;
}

__device__ __forceinline__ void gat_row_store(const GatArgs& a, int64_t row, const SoftAcc& r, int lane, int head) {
  const float inv = r.l > 0.f ? 1.f / r.l : 0.f;
  *reinterpret_cast<float2*>(a.U + row * kS + 2 * lane) = make_float2(r.a0 * inv, r.a1 * inv);
  if ((lane & 7) == 0) a.lse[row * 8 + head] = r.m + __logf(r.l);
}

__global__ __launch_bounds__(256) void k_gat_aggregate(GatArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_work) return;
  const int32_t si = a.work[3 * item], r0 = a.work[3 * item + 1], nr = a.work[3 * item + 2];
  const Segment s = a.segs[si];
  const int64_t* rowptr = a.g.rowptr[s.t];
  const int32_t* col = a.g.colidx[s.t];
  const int64_t base = (int64_t)s.t * a.g.N;
  const int head = lane >> 3;
  for (int rr = 0; rr < nr; ++rr) {
    const int64_t i = s.v_lo + r0 + rr;
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    if (e1 - e0 > a.long_nnz) continue;    // split rows: k_gat_aggregate_long
    const float sd = a.sX[(base + i) * 16 + 8 + head];
    const SoftAcc r = gat_row_range(a, s, col, base, sd, e0, e1, lane, head);
    gat_row_store(a, base + i, r, lane, head);
  }
}

// record of one part of a split row: weighted sum [128], maximum [8], sum [8]
constexpr int kLongRec = 144;

__global__ __launch_bounds__(256) void k_gat_aggregate_long(GatArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_long) return;
  const int32_t* w = a.work_long + 4 * item;
  const Segment s = a.segs[w[0]];
  const int64_t i = s.v_lo + w[1];
  const int64_t* rowptr = a.g.rowptr[s.t];
  const int64_t base = (int64_t)s.t * a.g.N;
  const int head = lane >> 3;
  const int64_t e0 = rowptr[i] + (int64_t)w[2] * a.part_nnz, e1 = min(rowptr[i + 1], e0 + a.part_nnz);
  const float sd = a.sX[(base + i) * 16 + 8 + head];
  const SoftAcc r = gat_row_range(a, s, a.g.colidx[s.t], base, sd, e0, e1, lane, head);
  float* rec = a.long_partial + item * kLongRec;
  *reinterpret_cast<float2*>(rec + 2 * lane) = make_float2(r.a0, r.a1);
  if ((lane & 7) == 0) {
    rec[128 + head] = r.m;
    rec[136 + head] = r.l;
  }
}

// one wavefront per split row (the item of its part 0) merges the parts in order
__global__ __launch_bounds__(256) void k_gat_aggregate_merge(GatArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= a.n_long) return;
  const int32_t* w = a.work_long + 4 * item;
  if (w[2] != 0) return;
  const Segment s = a.segs[w[0]];
  const int head = lane >> 3;
  const int parts = w[3];
  float mx = -INFINITY;
  for (int p = 0; p < parts; ++p) mx = fmaxf(mx, a.long_partial[(item + p) * kLongRec + 128 + head]);
  SoftAcc r{mx, 0.f, 0.f, 0.f};
  for (int p = 0; p < parts; ++p) {
    const float* rec = a.long_partial + (item + p) * kLongRec;
    const float sc = __expf(rec[128 + head] - mx);
    const float2 v = *reinterpret_cast<const float2*>(rec + 2 * lane);
    r.l += sc * rec[136 + head];
    r.a0 += sc * v.x;
    r.a1 += sc * v.y;
  }
  gat_row_store(a, (int64_t)s.t * a.g.N + s.v_lo + w[1], r, lane, head);
}

// ---------------------------------------------------------------------------------------------
// Temporal self-attention, forward.  One wavefront per two vertices of a chunk: 32 rows
// n = 16 a + s (a = vertex 0/1, s = step in the window).  Per block jb of 32 output features
// (two heads): Q and K in row layout, V in column layout; per head one product K Q^T gives the
// transposed score block of both vertices (lane (n_s, hh) holds the scores of its own query row
// against key rows 8g + 4hh + e; those of its own vertex are registers 8a .. 8a+7), the softmax
// is lane-local plus one exchange with lane l^32, and the probabilities are directly the B
// operand of the product with V (A operand = V in column layout, masked to the head; B masked
// to the vertex), which lands in row layout, ready to be stored.
// Every in-register operand (P, Q, K, V, the probabilities) is carried as a hi + lo pair of bf16
// values, so that the only roundings to bf16 are those of the stored tensors (z, U, Y).
struct TemporalArgs {
  const ChunkInfo* chunks; int32_t n_chunks;
  const int64_t* tile_ptr;   // [n_chunks+1] first tile of every chunk (2 vertices per tile; WIDE: 1)
  int64_t n_tiles;
  int64_t N; int32_t T;
  const float* U;
  const float* pos;          // [T][128]
  const uint4* Wq; const uint4* Wk; const uint4* Wv;   // mode-0 fragments
  uint16_t* Y; int64_t ldy;
};

// softmax over the key steps r <= s of the lane's own vertex; x[p] is the raw score against key
// step r = 8 (p/4) + 4 hh + p%4 (NP = 8: windows up to 16; NP = 16: up to 32); returns
// probabilities (0 for masked positions)
template <int NP>
__device__ __forceinline__ void causal_softmax(float* x, int s, int hh) {
  float mx = -INFINITY;
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const int r = 8 * (p >> 2) + 4 * hh + (p & 3);
    x[p] = r <= s ? 0.25f * x[p] : -INFINITY;
    mx = fmaxf(mx, x[p]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  float sum = 0.f;
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    x[p] = __expf(x[p] - mx);
    sum += x[p];
  }
  sum += __shfl_xor(sum, 32);
  const float inv = 1.f / sum;
#pragma unroll
  for (int p = 0; p < NP; ++p) x[p] *= inv;
}

// The three weight matrices (96 KB of fragments) are staged in LDS once per workgroup; the
// workgroup's waves then walk the tiles with a grid stride and never synchronise again.
constexpr int kFragsPerW = 4 * 8 * 64;   // uint4 fragments of one 128 x 128 weight

__device__ __forceinline__ void stage_weights(uint4* lds, const uint4* w0, const uint4* w1, const uint4* w2) {
  for (int i = threadIdx.x; i < kFragsPerW; i += blockDim.x) {
    lds[i] = w0[i];
    lds[kFragsPerW + i] = w1[i];
    lds[2 * kFragsPerW + i] = w2[i];
  }
  __syncthreads();
}

// WIDE: one vertex per tile, windows of up to 32 snapshots: the score block of a head is the whole
// 32 x 32 product (all 16 registers of a lane are keys of its own vertex), and the product with V
// contracts over the two halves of the keys (registers 0..7 and 8..15) instead of over two vertices.
template <bool WIDE>
__global__ __launch_bounds__(512) void k_temporal_fwd(TemporalArgs a) {
  extern __shared__ uint4 wlds[];
  stage_weights(wlds, a.Wq, a.Wk, a.Wv);
  const int lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  const int hh = lane >> 5, f = lane & 31;
  const uint32_t m_head[2] = {(f >> 4) == 0 ? 0xffffffffu : 0u, (f >> 4) == 1 ? 0xffffffffu : 0u};
  for (int64_t tile = (int64_t)blockIdx.x * nw + (threadIdx.x >> 6); tile < a.n_tiles; tile += (int64_t)gridDim.x * nw) {
  const TileRow r = tile_row<WIDE>(a.chunks, a.n_chunks, a.tile_ptr, tile, a.N, lane);
  const uint32_t m_vert[2] = {r.a == 0 ? 0xffffffffu : 0u, r.a == 1 ? 0xffffffffu : 0u};
  bf16x8 pf[8], pl[8];
  load_p_frags<true>(a.U, a.pos, r, hh, pf, pl);
#pragma unroll 1
  for (int jb = 0; jb < 4; ++jb) {
    floatx16 q = {}, k = {}, vt = {};
#pragma unroll
    for (int kb = 0; kb < 8; ++kb) {
      const int fi = (jb * 8 + kb) * 64 + lane;
      const bf16x8 wq = as_frag(wlds[fi]), wk = as_frag(wlds[kFragsPerW + fi]), wv = as_frag(wlds[2 * kFragsPerW + fi]);
      q = mfma(wq, pf[kb], q);
      q = mfma(wq, pl[kb], q);
      k = mfma(wk, pf[kb], k);
      k = mfma(wk, pl[kb], k);
      vt = mfma(pf[kb], wv, vt);
      vt = mfma(pl[kb], wv, vt);
    }
    floatx16 y = {};
#pragma unroll
    for (int hd = 0; hd < 2; ++hd) {
      float tmp[8];
      bf16x8 kh, kl, qh, ql;
#pragma unroll
      for (int p = 0; p < 8; ++p) tmp[p] = k[8 * hd + p];
      split8(tmp, kh, kl);
#pragma unroll
      for (int p = 0; p < 8; ++p) tmp[p] = q[8 * hd + p];
      split8(tmp, qh, ql);
      floatx16 st = {};
      st = mfma(kl, qh, st);                 // st[i = key row][j = query row]
      st = mfma(kh, ql, st);
      st = mfma(kh, qh, st);
      constexpr int NP = WIDE ? 16 : 8;
      float pr[NP];
#pragma unroll
      for (int p = 0; p < NP; ++p) pr[p] = WIDE ? st[p] : pick_half(st, p, m_vert[0], m_vert[1]);
      causal_softmax<NP>(pr, r.s, hh);
      bf16x8 ph[NP / 8], plo[NP / 8];
#pragma unroll
      for (int c = 0; c < NP / 8; ++c) split8(pr + 8 * c, ph[c], plo[c]);
#pragma unroll
      for (int av = 0; av < 2; ++av) {      // the two vertices, or (WIDE) the two halves of the keys
        bf16x8 vh, vl;
#pragma unroll
        for (int p = 0; p < 8; ++p) tmp[p] = vt[8 * av + p];
        split8(tmp, vh, vl);
        vh = and_mask(vh, m_head[hd]);
        vl = and_mask(vl, m_head[hd]);
        const bf16x8 pa = WIDE ? ph[WIDE ? av : 0] : and_mask(ph[0], m_vert[av]);
        const bf16x8 pb = WIDE ? plo[WIDE ? av : 0] : and_mask(plo[0], m_vert[av]);
        y = mfma(vl, pa, y);
        y = mfma(vh, pb, y);
        y = mfma(vh, pa, y);
      }
    }
    if (r.valid) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<uint2*>(a.Y + r.row * a.ldy + jb * 32 + 8 * g + 4 * hh) =
            pack4(y[4 * g], y[4 * g + 1], y[4 * g + 2], y[4 * g + 3]);
    }
  }
  }
}

}  // namespace

void dysat_build_owner(const Segment* segs, int64_t nseg, int32_t T, int64_t N, int32_t* owner, hipStream_t st) {
  hipLaunchKernelGGL(k_fill_i32, blocks_for((int64_t)T * N, 256), 256, 0, st, owner, -1, (int64_t)T * N);
  hipLaunchKernelGGL(k_owner, (unsigned)nseg, 256, 0, st, segs, N, owner);
}

void dysat_pack_params(const DysatWs& ws, hipStream_t st) {
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_W], ws.Wp, 0);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_WQ], ws.Wqp, 0);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_WK], ws.Wkp, 0);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_WV], ws.Wvp, 0);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_WQ], ws.WqT, 1);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_WK], ws.WkT, 1);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_WV], ws.WvT, 1);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_W], ws.WT, 1);
  hipLaunchKernelGGL(k_pack_w_bf16, 8, 256, 0, st, ws.P[DY_W], ws.WTlo, 2);
}

void dysat_forward(const DysatWs& ws, const void* X, int64_t ldx, const void* C, int64_t ldc, void* Y, int64_t ldy,
                   hipEvent_t* ev, hipStream_t st) {
  ProjArgs pa{};
  pa.X = static_cast<const uint16_t*>(X); pa.ldx = ldx;
  pa.C = static_cast<const uint16_t*>(C); pa.ldc = ldc;
  pa.Wp = ws.Wp; pa.a_src = ws.P[DY_ASRC]; pa.a_dst = ws.P[DY_ADST];
  pa.owner = ws.owner; pa.used_t = ws.used_t; pa.n_used = ws.n_used; pa.N = ws.N;
  pa.zX = ws.zX; pa.zC = ws.zC; pa.sX = ws.sX; pa.sC = ws.sC;
  const int64_t ptiles = (ws.N + 31) / 32 * ws.n_used;
  if (ev) (void)hipEventRecord(ev[0], st);
  hipLaunchKernelGGL(k_gat_project, blocks_for(ptiles, 4), 256, 0, st, pa);
  if (ev) (void)hipEventRecord(ev[1], st);
  GatArgs ga{};
  ga.g = ws.g; ga.segs = ws.segs; ga.work = ws.work_short; ga.n_work = ws.n_short;
  ga.work_long = ws.work_long; ga.n_long = ws.n_long; ga.long_nnz = ws.long_nnz; ga.part_nnz = ws.part_nnz;
  ga.long_partial = ws.long_partial;
  ga.zX = ws.zX; ga.zC = ws.zC; ga.sX = ws.sX; ga.sC = ws.sC; ga.U = ws.U; ga.lse = ws.lse;
  hipLaunchKernelGGL(k_gat_aggregate, blocks_for(ws.n_short, 4), 256, 0, st, ga);
  if (ws.n_long > 0) {
    hipLaunchKernelGGL(k_gat_aggregate_long, blocks_for(ws.n_long, 4), 256, 0, st, ga);
    hipLaunchKernelGGL(k_gat_aggregate_merge, blocks_for(ws.n_long, 4), 256, 0, st, ga);
  }
  if (ev) (void)hipEventRecord(ev[2], st);
  TemporalArgs ta{};
  ta.chunks = ws.chunks; ta.n_chunks = ws.n_chunks; ta.tile_ptr = ws.tile_ptr; ta.n_tiles = ws.n_tiles;
  ta.N = ws.N; ta.T = ws.T; ta.U = ws.U; ta.pos = ws.P[DY_POS];
  ta.Wq = ws.Wqp; ta.Wk = ws.Wkp; ta.Wv = ws.Wvp;
  ta.Y = static_cast<uint16_t*>(Y); ta.ldy = ldy;
  {
    static bool attr_set = false;   // dynamic LDS above 64 KB has to be allowed once per kernel
    const size_t lds = sizeof(uint4) * 3 * kFragsPerW;
    if (!attr_set) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_temporal_fwd<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_temporal_fwd<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds);
      attr_set = true;
    }
    const unsigned grid = (unsigned)std::min<int64_t>(256, (ws.n_tiles + 7) / 8);
    if (ws.wide) hipLaunchKernelGGL(k_temporal_fwd<true>, grid, 512, lds, st, ta);
    else hipLaunchKernelGGL(k_temporal_fwd<false>, grid, 512, lds, st, ta);
  }
  if (ev) (void)hipEventRecord(ev[3], st);
}

}  // namespace dgc
