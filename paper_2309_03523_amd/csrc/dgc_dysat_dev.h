// Device helpers shared by the forward and backward kernels of the graph-attention +
// temporal self-attention layer (bf16 storage, fp32 accumulation).
//
// All dense products run on v_mfma_f32_32x32x16_bf16: lane l supplies A[l%32][8*(l/32) .. +7] and
// B[8*(l/32) .. +7][l%32] and receives D[8*(v/4) + 4*(l/32) + v%4][l%32] in register v.  With the
// weights as A operand and 32 activation rows as B operand, lane (n = l%32, hh = l/32) ends up with
// features 8g + 4hh + e (g = v/4, e = v%4) of its own row n: "row layout".  With the activations as
// A operand and the weights as B operand, lane (f = l%32, hh) ends up with feature f of rows
// 8g + 4hh + e: "column layout".  Eight consecutive accumulator registers (g = 2c, 2c+1) of a lane
// are one k-half of a 16-wide contraction index in either layout, which is what lets every
// attention product take its operands straight from accumulators, without moving data between
// lanes.
#pragma once

#include "dgc_internal.h"

namespace dgc {
namespace dysat {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kS = 128;      // feature width (input, structure output, attention width)
constexpr int kHeads = 8;
constexpr int kD = 16;       // dims per head
constexpr float kSlope = 0.2f;

__device__ __forceinline__ bf16x8 as_frag(uint4 u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) { return make_uint2(pack2(a, b), pack2(c, d)); }
__device__ __forceinline__ bf16x8 pack8(const float* x) {
  bf16x8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (__bf16)x[i];
  return v;
}
__device__ __forceinline__ bf16x8 pack8v(const floatx16& v, int off) {
  bf16x8 r;
#pragma unroll
  for (int p = 0; p < 8; ++p) r[p] = (__bf16)v[off + p];
  return r;
}
__device__ __forceinline__ void unpack8(uint4 u, float* x) {
  x[0] = bf_lo(u.x); x[1] = bf_hi(u.x); x[2] = bf_lo(u.y); x[3] = bf_hi(u.y);
  x[4] = bf_lo(u.z); x[5] = bf_hi(u.z); x[6] = bf_lo(u.w); x[7] = bf_hi(u.w);
}
// The projections z are kept in IEEE half precision: they are O(1) values that only the vector
// units read (the neighbour gathers), so the format is free, and at the same 2 bytes per element
// half precision rounds four times finer than bf16; the rounding of z is what dominates the error
// of the whole layer.
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float h_lo(uint32_t u) { return (float)__builtin_bit_cast(halfx2, u)[0]; }
__device__ __forceinline__ float h_hi(uint32_t u) { return (float)__builtin_bit_cast(halfx2, u)[1]; }
__device__ __forceinline__ uint32_t packh2(float a, float b) {
  halfx2 v = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint2 packh4(float a, float b, float c, float d) { return make_uint2(packh2(a, b), packh2(c, d)); }
__device__ __forceinline__ void unpackh8(uint4 u, float* x) {
  x[0] = h_lo(u.x); x[1] = h_hi(u.x); x[2] = h_lo(u.y); x[3] = h_hi(u.y);
  x[4] = h_lo(u.z); x[5] = h_hi(u.z); x[6] = h_lo(u.w); x[7] = h_hi(u.w);
}

__device__ __forceinline__ floatx16 mfma(bf16x8 a, bf16x8 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float lrelu(float x) { return x > 0.f ? x : kSlope * x; }
__device__ __forceinline__ float elu(float x) { return x > 0.f ? x : __expf(x) - 1.f; }
__device__ __forceinline__ float delu(float u) { return u > 0.f ? 1.f : __expf(u); }   // ELU'(u)

// x -> hi + lo with hi = bf16(x), lo = bf16(x - hi): two bf16 operands that together carry 16
// mantissa bits, so a product taken as hi*hi + hi*lo + lo*hi is accurate to ~2^-16
__device__ __forceinline__ void split8(const float* x, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16 h = (__bf16)x[i];
    hi[i] = h;
    lo[i] = (__bf16)(x[i] - (float)h);
  }
}

// Element p of v for a lane whose mask m0 is all ones, element 8 + p where m1 is (exactly one of the
// two is): a bitwise blend.  Written as a select between two elements of one vector it is turned
// into a lane-dependent index, which costs a compare and a select per element of the vector.
__device__ __forceinline__ float pick_half(const floatx16& v, int p, uint32_t m0, uint32_t m1) {
  return __uint_as_float((__float_as_uint(v[p]) & m0) | (__float_as_uint(v[8 + p]) & m1));
}

// x where m is all ones, zero where m is zero (a select on the packed dwords: selecting on a
// vector of eight 16-bit elements would be unpacked element by element)
__device__ __forceinline__ bf16x8 and_mask(bf16x8 x, uint32_t m) {
  uint4 u = __builtin_bit_cast(uint4, x);
  u.x &= m; u.y &= m; u.z &= m; u.w &= m;
  return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ void split8v(const floatx16& v, int off, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const __bf16 h = (__bf16)v[off + p];
    hi[p] = h;
    lo[p] = (__bf16)(v[off + p] - (float)h);
  }
}
// products of split operands: (ah + al)(bh + bl) without the al*bl term; a exact: a (bh + bl)
__device__ __forceinline__ floatx16 mfma3(bf16x8 ah, bf16x8 al, bf16x8 bh, bf16x8 bl, floatx16 c) {
  c = mfma(al, bh, c);
  c = mfma(ah, bl, c);
  return mfma(ah, bh, c);
}
__device__ __forceinline__ floatx16 mfma2b(bf16x8 a, bf16x8 bh, bf16x8 bl, floatx16 c) {
  c = mfma(a, bl, c);
  return mfma(a, bh, c);
}
__device__ __forceinline__ floatx16 mfma2a(bf16x8 ah, bf16x8 al, bf16x8 b, floatx16 c) {
  c = mfma(al, b, c);
  return mfma(ah, b, c);
}

// Selection operand that transposes a 32 x 16 piece of a row-major tile on the matrix core:
// as B operand, element p of lane (j = l%32, hh) is 1 where j == 16 c + 8 hh + p.  With a natural
// 16-byte row fragment X[n][16 kb + 8 hh + 0..7] as A operand, kb = 2 jb + c, the two products
// c = 0, 1 leave X[8g + 4hh + e][32 jb + f] in lane (f, hh): column layout, exact.
__device__ __forceinline__ bf16x8 sel_frag(int c, int lane) {
  const int j = lane & 31, hh = lane >> 5;
  bf16x8 s;
#pragma unroll
  for (int p = 0; p < 8; ++p) s[p] = (j == 16 * c + 8 * hh + p) ? (__bf16)1.0f : (__bf16)0.0f;
  return s;
}

// A tile of the temporal kernels, 32 rows.  Windows of at most 16 snapshots: two vertices of one
// chunk over the chunk's window, n = 16 a + s (a = vertex 0/1, s = step).  WIDE (some window of the
// layer is longer, up to 32): one vertex, n = s.  What a lane needs to know about its row
// n = lane % 32:
struct TileRow {
  int64_t row;     // t*N + v (clamped to a valid row when !valid)
  int32_t t, s, a, t_lo;
  bool valid;
};

template <bool WIDE>
__device__ __forceinline__ TileRow tile_row(const ChunkInfo* chunks, int32_t n_chunks, const int64_t* tile_ptr,
                                            int64_t tile, int64_t N, int lane) {
  int lo = 0, hi = n_chunks;   // largest k with tile_ptr[k] <= tile
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tile_ptr[mid] <= tile) lo = mid; else hi = mid;
  }
  const ChunkInfo c = chunks[lo];
  const int n = lane & 31;
  TileRow r;
  r.a = WIDE ? 0 : n >> 4; r.s = WIDE ? n : n & 15; r.t_lo = c.t_lo;
  const int64_t vl = WIDE ? tile - tile_ptr[lo] : 2 * (tile - tile_ptr[lo]) + r.a;
  r.valid = vl < c.nv && r.s < c.w;
  r.t = c.t_lo + (r.s < c.w ? r.s : 0);
  r.row = (int64_t)r.t * N + c.v_lo + (vl < c.nv ? vl : 0);
  return r;
}

// P = ELU(U) + pos for the lane's row, as eight B/A-operand fragments (hi part, and lo part if
// LO); rows that are not valid read as zero
template <bool LO>
__device__ __forceinline__ void load_p_frags(const float* U, const float* pos, const TileRow& r, int hh, bf16x8* pf,
                                             bf16x8* pl) {
#pragma unroll
  for (int kb = 0; kb < 8; ++kb) {
    float x[8];
    if (r.valid) {
      const float4 u0 = *reinterpret_cast<const float4*>(U + r.row * kS + kb * 16 + 8 * hh);
      const float4 u1 = *reinterpret_cast<const float4*>(U + r.row * kS + kb * 16 + 8 * hh + 4);
      x[0] = u0.x; x[1] = u0.y; x[2] = u0.z; x[3] = u0.w; x[4] = u1.x; x[5] = u1.y; x[6] = u1.z; x[7] = u1.w;
      const float4 p0 = *reinterpret_cast<const float4*>(pos + r.t * kS + kb * 16 + 8 * hh);
      const float4 p1 = *reinterpret_cast<const float4*>(pos + r.t * kS + kb * 16 + 8 * hh + 4);
      x[0] = elu(x[0]) + p0.x; x[1] = elu(x[1]) + p0.y; x[2] = elu(x[2]) + p0.z; x[3] = elu(x[3]) + p0.w;
      x[4] = elu(x[4]) + p1.x; x[5] = elu(x[5]) + p1.y; x[6] = elu(x[6]) + p1.z; x[7] = elu(x[7]) + p1.w;
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = 0.f;
    }
    if (LO) split8(x, pf[kb], pl[kb]);
    else pf[kb] = pack8(x);
  }
}

inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

}  // namespace dysat
}  // namespace dgc
