// Adaptive stale-embedding filter (Section 5.2 of the paper) on the device: the L2 distance of
// every candidate row to the copy transmitted last, the largest distance D, the threshold, the
// ascending list of the rows that exceed it, their values packed as the message, and the update
// of the stored copies.  An HBM-bound scan: every candidate row of E and L is read once.
//
// Launch sequence (nothing synchronises, no float atomics, the result is the same run to run):
//   k_stale_init      result = {0, 0, 0}
//   k_stale_dist      dist[c], block maxima folded into D with an integer max on the float's bits
//                     (distances are >= 0, so the bit patterns order like the values)
//   k_stale_count     candidates above the threshold per block of kSelTile
//   exclusive scan    of the block counts
//   k_stale_compact   send_idx in ascending order, copies of the selected rows
#include <cmath>

#include <mutex>

#include "dgc_internal.h"

// Scratch of dgc_stale_filter_static: the block counts, their scan's temporaries and the total, for
// up to kStaticMaxCandidates candidates.  Every GPU the library runs on holds its own copy until the
// process ends.  Host code never uses this name as an address: the per-device address comes from
// hipGetSymbolAddress (static_scratch_ptr below).
constexpr int64_t kStaticMaxCandidates = int64_t(1) << 26;
constexpr int64_t kStaticScratchBytes = 272 * 1024;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace dgc {
namespace {

constexpr int kSelBlock = 256;
constexpr int kSelPer = 8;
constexpr int kSelTile = kSelBlock * kSelPer;  // candidates per block of the two selection kernels
constexpr int kDistUnroll = 4;                  // row groups a wave keeps in flight

struct StaleArgs {
  const void* E; int64_t lde;   // rows of float or bfloat16 (the kernels' element type), pitches in elements
  void* L; int64_t ldl;
  const int64_t* rows;  // nullptr: candidate c is row c
  int64_t R;            // rows of E and L
  int64_t n;            // candidates
  int32_t F;
  double factor;        // >= 0: threshold = factor * D; < 0: threshold = theta
  double theta;
  float* dist;
  int64_t* send_idx;
  void* send_buf; int64_t lds;
  dgc_stale_result_t* result;
  int64_t* counts;      // [blocks of kSelTile]
  const int64_t* total;
};

__global__ void k_stale_init(dgc_stale_result_t* r) {
  r->n_send = 0; r->D = 0.f; r->theta = 0.f; r->n_invalid = 0;
}

// Element types: float, or bfloat16 carried as uint16_t (its bits are the top half of a float's).
template <class T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerVec = 4;   // elements in a 16-byte vector
  static __device__ __forceinline__ float get(float v) { return v; }
  static __device__ __forceinline__ float sqdiff(const uint4 a, const uint4 b) {
    const float x = __uint_as_float(a.x) - __uint_as_float(b.x), y = __uint_as_float(a.y) - __uint_as_float(b.y);
    const float z = __uint_as_float(a.z) - __uint_as_float(b.z), w = __uint_as_float(a.w) - __uint_as_float(b.w);
    return x * x + y * y + z * z + w * w;
  }
};
template <> struct Elem<uint16_t> {
  static constexpr int kPerVec = 8;
  static __device__ __forceinline__ float get(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
  static __device__ __forceinline__ float sq2(uint32_t a, uint32_t b) {
    const float x = __uint_as_float(a << 16) - __uint_as_float(b << 16);
    const float y = __uint_as_float(a & 0xffff0000u) - __uint_as_float(b & 0xffff0000u);
    return x * x + y * y;
  }
  static __device__ __forceinline__ float sqdiff(const uint4 a, const uint4 b) {
    return sq2(a.x, b.x) + sq2(a.y, b.y) + sq2(a.z, b.z) + sq2(a.w, b.w);
  }
};

// LPR lanes share a row (a 16-byte vector each per sweep of LPR vectors), 64/LPR rows per wave
// and sweep, kDistUnroll sweeps in flight.
template <int LPR, class T>
__global__ __launch_bounds__(256) void k_stale_dist(StaleArgs a) {
  constexpr int EPV = Elem<T>::kPerVec;
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR, grp = lane / LPR;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  float dmax = 0.f;
  for (int64_t base = wave * (RPW * kDistUnroll); base < a.n; base += n_waves * (RPW * kDistUnroll)) {
    float acc[kDistUnroll];
#pragma unroll
    for (int u = 0; u < kDistUnroll; ++u) {
      const int64_t c = base + u * RPW + grp;
      acc[u] = 0.f;
      const int64_t r = c < a.n ? (a.rows ? a.rows[c] : c) : -1;
      if (c < a.n && (r < 0 || r >= a.R)) {  // a listed row outside the tensors: distance 0, counted
        if (sub == 0) atomicAdd(reinterpret_cast<unsigned long long*>(&a.result->n_invalid), 1ull);
      } else if (c < a.n) {
        const T* e = static_cast<const T*>(a.E) + r * a.lde;
        const T* l = static_cast<const T*>(a.L) + r * a.ldl;
        for (int col = sub * EPV; col < a.F; col += LPR * EPV) {
          if (col + EPV <= a.F) {
            acc[u] += Elem<T>::sqdiff(*reinterpret_cast<const uint4*>(e + col), *reinterpret_cast<const uint4*>(l + col));
          } else {
            for (int k = col; k < a.F; ++k) { const float d = Elem<T>::get(e[k]) - Elem<T>::get(l[k]); acc[u] += d * d; }
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kDistUnroll; ++u) {
      float s = acc[u];
#pragma unroll
      for (int m = LPR / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
      const int64_t c = base + u * RPW + grp;
      if (sub == 0 && c < a.n) {
        const float d = sqrtf(s);
        a.dist[c] = d;
        dmax = fmaxf(dmax, d);
      }
    }
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) dmax = fmaxf(dmax, __shfl_xor(dmax, m));
  __shared__ float wmax[4];
  if (lane == 0) wmax[threadIdx.x >> 6] = dmax;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    atomicMax(reinterpret_cast<unsigned int*>(&a.result->D), __float_as_uint(m));
  }
}

__device__ __forceinline__ float threshold_of(const StaleArgs& a) {
  return a.factor >= 0.0 ? (float)(a.factor * (double)a.result->D) : (float)a.theta;
}

// bit k of the result: candidate first + k exists and is above the threshold
__device__ __forceinline__ unsigned flags_of(const StaleArgs& a, int64_t first, float th) {
  unsigned f = 0;
  if (first + kSelPer <= a.n) {
    const float4 d0 = *reinterpret_cast<const float4*>(a.dist + first);
    const float4 d1 = *reinterpret_cast<const float4*>(a.dist + first + 4);
    f = (d0.x > th) | (d0.y > th) << 1 | (d0.z > th) << 2 | (d0.w > th) << 3 | (d1.x > th) << 4 | (d1.y > th) << 5 |
        (d1.z > th) << 6 | (d1.w > th) << 7;
  } else {
    for (int k = 0; k < kSelPer; ++k)
      if (first + k < a.n && a.dist[first + k] > th) f |= 1u << k;
  }
  return f;
}

__global__ __launch_bounds__(kSelBlock) void k_stale_count(StaleArgs a) {
  const float th = threshold_of(a);
  const int64_t first = (int64_t)blockIdx.x * kSelTile + threadIdx.x * kSelPer;
  int cnt = __popc(flags_of(a, first, th));
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) cnt += __shfl_xor(cnt, m);
  __shared__ int wsum[kSelBlock / 64];
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int s = 0;
    for (int w = 0; w < kSelBlock / 64; ++w) s += wsum[w];
    a.counts[blockIdx.x] = s;
  }
}

// counts now holds the exclusive scan.  Thread order = candidate order, so the block's selected
// rows land in ascending order; they are then copied LPR lanes to a row.
template <int LPR, class T>
__global__ __launch_bounds__(kSelBlock) void k_stale_compact(StaleArgs a) {
  constexpr int EPV = Elem<T>::kPerVec;
  __shared__ int64_t sel_row[kSelTile];
  __shared__ int wbase[kSelBlock / 64 + 1];
  const float th = threshold_of(a);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t first = (int64_t)blockIdx.x * kSelTile + threadIdx.x * kSelPer;
  const unsigned f = flags_of(a, first, th);
  const int cnt = __popc(f);
  int incl = cnt;  // inclusive scan over the wave
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const int v = __shfl_up(incl, m);
    if (lane >= m) incl += v;
  }
  if (lane == 63) wbase[w + 1] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    wbase[0] = 0;
    for (int i = 1; i <= kSelBlock / 64; ++i) wbase[i] += wbase[i - 1];
  }
  __syncthreads();
  const int64_t off = a.counts[blockIdx.x];
  int pos = wbase[w] + incl - cnt;
  for (int k = 0; k < kSelPer; ++k)
    if (f >> k & 1) {
      const int64_t r = a.rows ? a.rows[first + k] : first + k;
      sel_row[pos] = r;
      a.send_idx[off + pos] = r;
      ++pos;
    }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.result->n_send = *a.total;
    a.result->theta = th;
  }
  __syncthreads();
  const int n_sel = wbase[kSelBlock / 64];
  constexpr int RPB = kSelBlock / LPR;
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  for (int i = grp; i < n_sel; i += RPB) {
    const int64_t r = sel_row[i];
    const T* e = static_cast<const T*>(a.E) + r * a.lde;
    T* l = static_cast<T*>(a.L) + r * a.ldl;
    T* s = a.send_buf ? static_cast<T*>(a.send_buf) + (off + i) * a.lds : nullptr;
    for (int col = sub * EPV; col < a.F; col += LPR * EPV) {
      if (col + EPV <= a.F) {
        const uint4 v = *reinterpret_cast<const uint4*>(e + col);
        *reinterpret_cast<uint4*>(l + col) = v;
        if (s) *reinterpret_cast<uint4*>(s + col) = v;
      } else {
        for (int k = col; k < a.F; ++k) { l[k] = e[k]; if (s) s[k] = e[k]; }
      }
    }
  }
}

int64_t sel_blocks(int64_t n) { return (n + kSelTile - 1) / kSelTile; }

template <int LPR, class T>
void launch_all(const StaleArgs& a, int64_t* scan_tmp, int64_t* total, hipStream_t st) {
  constexpr int RPW = 64 / LPR;
  const int64_t per_block = 4 * RPW * kDistUnroll;
  const unsigned grid = (unsigned)std::min<int64_t>((a.n + per_block - 1) / per_block, 256 * 32);
  hipLaunchKernelGGL((k_stale_dist<LPR, T>), grid, 256, 0, st, a);
  const unsigned nb = (unsigned)sel_blocks(a.n);
  hipLaunchKernelGGL(k_stale_count, nb, kSelBlock, 0, st, a);
  launch_exclusive_scan(a.counts, nb, scan_tmp, total, st);
  hipLaunchKernelGGL((k_stale_compact<LPR, T>), nb, kSelBlock, 0, st, a);
}

template <class T>
void launch_for_width(const StaleArgs& a, int64_t* scan_tmp, int64_t* total, hipStream_t st) {
  const int vecs = (a.F + Elem<T>::kPerVec - 1) / Elem<T>::kPerVec;   // 16-byte vectors per row
  if (vecs <= 4) launch_all<4, T>(a, scan_tmp, total, st);
  else if (vecs <= 8) launch_all<8, T>(a, scan_tmp, total, st);
  else if (vecs <= 16) launch_all<16, T>(a, scan_tmp, total, st);
  else if (vecs <= 32) launch_all<32, T>(a, scan_tmp, total, st);
  else launch_all<64, T>(a, scan_tmp, total, st);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace
}  // namespace dgc

using namespace dgc;

extern "C" {

double dgc_stale_theta_factor(double l1, double l_prev, int32_t variant) {
  if (!(l1 > 0.0) || !std::isfinite(l_prev) || (variant != DGC_THETA_PRINTED && variant != DGC_THETA_SIGMOID)) return -1.0;
  const double norm = (l1 - l_prev) / l1;
  return 1.0 / (1.0 + std::exp(variant == DGC_THETA_PRINTED ? norm : -norm));
}

int64_t dgc_stale_workspace_bytes(int64_t n_candidates) {
  if (n_candidates < 0) return -1;
  const int64_t nb = sel_blocks(n_candidates);
  return 8 * (nb + 1 + scan_tmp_elems(nb) + 1);
}

static dgc_status_t stale_filter_impl(const void* E, int64_t lde, void* L, int64_t ldl, int64_t R, int32_t F, int32_t dtype,
                                      const int64_t* rows, int64_t n_rows, double factor, double theta, float* dist,
                                      int64_t* send_idx, void* send_buf, int64_t lds, dgc_stale_result_t* result,
                                      void* workspace, int64_t workspace_bytes, void* stream) {
  auto bad = [](dgc_status_t code, const char* msg) { set_thread_error(msg); return code; };
  if (!E || !L || !result || !workspace) return bad(DGC_ERR_INVALID_ARG, "stale filter: NULL argument");
  if (R < 0 || F < 1 || F > 4096) return bad(DGC_ERR_INVALID_ARG, "stale filter: R must be >= 0 and F in [1, 4096]");
  if (dtype != DGC_DTYPE_F32 && dtype != DGC_DTYPE_BF16) return bad(DGC_ERR_INVALID_ARG, "stale filter: unknown dtype");
  const int epv = dtype == DGC_DTYPE_F32 ? 4 : 8, esz = 16 / epv;   // elements per 16 bytes, bytes per element
  if (lde < F || ldl < F || lde % epv || ldl % epv || !aligned16(E) || !aligned16(L))
    return bad(DGC_ERR_INVALID_ARG, "stale filter: E, L need a pitch >= F that is a multiple of 16 bytes and 16-byte alignment");
  if (send_buf && (lds < F || lds % epv || !aligned16(send_buf)))
    return bad(DGC_ERR_INVALID_ARG, "stale filter: send_buf needs a pitch >= F that is a multiple of 16 bytes and 16-byte alignment");
  if (rows ? n_rows < 0 || n_rows > R : n_rows != 0)
    return bad(DGC_ERR_INVALID_ARG, "stale filter: n_rows must be in [0, R] with a row list and 0 without");
  const int64_t n = rows ? n_rows : R;
  if (n > 0 && (!dist || !send_idx || !aligned16(dist)))
    return bad(DGC_ERR_INVALID_ARG, "stale filter: dist (16-byte aligned) and send_idx must hold one entry per candidate");
  if (!(factor >= 0.0) && !(theta >= 0.0))
    return bad(DGC_ERR_INVALID_ARG, "stale filter: give factor >= 0, or factor < 0 and theta >= 0");
  if (factor >= 0.0 && !std::isfinite(factor)) return bad(DGC_ERR_INVALID_ARG, "stale filter: factor is not finite");
  if (workspace_bytes < dgc_stale_workspace_bytes(n) || (reinterpret_cast<uintptr_t>(workspace) & 7))
    return bad(DGC_ERR_INVALID_ARG, "stale filter: workspace too small (dgc_stale_workspace_bytes) or not 8-byte aligned");
  {  // E and L are read and written by different blocks of one launch: they must not overlap
    const char* e0 = reinterpret_cast<const char*>(E); const char* e1 = e0 + esz * (R * lde);
    const char* l0 = reinterpret_cast<const char*>(L); const char* l1 = l0 + esz * (R * ldl);
    if (R > 0 && e0 < l1 && l0 < e1) return bad(DGC_ERR_INVALID_ARG, "stale filter: E and L overlap");
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(k_stale_init, 1, 1, 0, st, result);
  if (n > 0) {
    const int64_t nb = sel_blocks(n);
    int64_t* ws = static_cast<int64_t*>(workspace);
    StaleArgs a{};
    a.E = E; a.lde = lde; a.L = L; a.ldl = ldl; a.rows = rows; a.R = R; a.n = n; a.F = F;
    a.factor = factor >= 0.0 ? factor : -1.0; a.theta = theta;
    a.dist = dist; a.send_idx = send_idx; a.send_buf = send_buf; a.lds = lds; a.result = result;
    a.counts = ws; a.total = ws + nb + 1;
    int64_t* scan_tmp = ws + nb + 2;
    int64_t* total = ws + nb + 1;
    if (dtype == DGC_DTYPE_F32) launch_for_width<float>(a, scan_tmp, total, st);
    else launch_for_width<uint16_t>(a, scan_tmp, total, st);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return bad(DGC_ERR_DEVICE, hipGetErrorString(e));
  return DGC_OK;
}

dgc_status_t dgc_stale_filter(const void* E, int64_t lde, void* L, int64_t ldl, int64_t R, int32_t F, int32_t dtype,
                              const int64_t* rows, int64_t n_rows, double factor, double theta, float* dist,
                              int64_t* send_idx, void* send_buf, int64_t lds, dgc_stale_result_t* result,
                              void* workspace, int64_t workspace_bytes, void* stream) {
  return stale_filter_impl(E, lde, L, ldl, R, F, dtype, rows, n_rows, factor, theta, dist, send_idx, send_buf, lds,
                           result, workspace, workspace_bytes, stream);
}

int64_t dgc_stale_static_max_candidates(void) { return kStaticMaxCandidates; }

// Address of this device's copy of `scratch`, looked up once per device with that device current.
static void* static_scratch_ptr(std::string* err) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *err = std::string("stale filter (static): hipGetDevice: ") + (e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      *err = std::string("stale filter (static): hipGetSymbolAddress: ") + hipGetErrorString(e);
      return nullptr;
    }
    ptr[dev] = p;
  }
  return ptr[dev];
}

dgc_status_t dgc_stale_filter_static(const void* E, int64_t lde, void* L, int64_t ldl, int64_t R, int32_t F,
                                     int32_t dtype, const int64_t* rows, int64_t n_rows, double factor, double theta,
                                     float* dist, int64_t* send_idx, void* send_buf, int64_t lds,
                                     dgc_stale_result_t* result, void* stream) {
  const int64_t n = rows ? n_rows : R;
  if (n > kStaticMaxCandidates || dgc_stale_workspace_bytes(n > 0 ? n : 0) > kStaticScratchBytes) {
    set_thread_error("stale filter (static): more than dgc_stale_static_max_candidates() candidates");
    return DGC_ERR_UNSUPPORTED;
  }
  std::string err;
  void* ws = static_scratch_ptr(&err);
  if (!ws) { set_thread_error(err); return DGC_ERR_DEVICE; }
  // Nothing in the scratch has to start at zero: the count kernel writes every block count of this
  // call, the scan writes its temporaries and the total before anything reads them.
  return stale_filter_impl(E, lde, L, ldl, R, F, dtype, rows, n_rows, factor, theta, dist, send_idx, send_buf, lds,
                           result, ws, kStaticScratchBytes, stream);
}

}  // extern "C"
