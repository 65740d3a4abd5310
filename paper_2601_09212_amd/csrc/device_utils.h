// Device-side building blocks of the Cool-SD verify kernels (gfx950, wave64).
//
// Layout of a row chunk on chip.  A workgroup of 256 threads holds one chunk of NT tiles of a
// row in registers.  A tile is 256 x 16 bytes; in tile k thread t owns the 16-byte vector
// number k*256 + t of the chunk, i.e. the kE = 8 (bf16) or 4 (fp32) consecutive elements
// starting at (k*256 + t)*kE.  Every global load instruction therefore reads 1 KiB of
// consecutive memory per wave.  The sampling kernel uses chunks of kChunk = 16384 logits
// (NT = Vec::kT); the statistics kernel uses smaller ones to keep many workgroups in flight.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace csd {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kChunk = 16384;
constexpr int kDtF32 = 0;
constexpr int kDtBF16 = 1;
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kRefFloor = -1.5e30f;  // "no finite logit seen yet" reference exponent
// how a kernel may load a row: element-wise, 16-byte vectors, or 16-byte vectors with the
// nontemporal hint (large read-once inputs)
enum { kUnaligned = 0, kAligned = 1, kAlignedStream = 2, kAlignedFull = 3 };

template <int DT> struct Vec {
  static constexpr int kE = (DT == kDtBF16) ? 8 : 4;       // elements per 16-byte vector
  static constexpr int kES = (DT == kDtBF16) ? 2 : 4;      // bytes per element
  static constexpr int kT = kChunk / (kThreads * kE);      // tiles per chunk: 8 / 16
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---------------------------------------------------------------- fp64 exponential
// (for the few scalar decisions and rare re-draws that are made in fp64)
constexpr double kLog2eD = 1.44269504088896340736;

// 2^y for y <= ~1: split into integer and fraction, e^(f ln 2) by its Taylor polynomial of degree
// 12 on |f ln 2| <= 0.347 (remainder below 4e-17), scaled by the integer part.  -inf and anything
// below the normal range give 0.
__device__ __forceinline__ double exp2_d(double y) {
  if (!(y > -1021.0)) return 0.0;
  const double n = rint(y);
  const double t = (y - n) * 0.693147180559945309417;
  double p = 1.0 / 479001600.0;
  p = fma(p, t, 1.0 / 39916800.0);
  p = fma(p, t, 1.0 / 3628800.0);
  p = fma(p, t, 1.0 / 362880.0);
  p = fma(p, t, 1.0 / 40320.0);
  p = fma(p, t, 1.0 / 5040.0);
  p = fma(p, t, 1.0 / 720.0);
  p = fma(p, t, 1.0 / 120.0);
  p = fma(p, t, 1.0 / 24.0);
  p = fma(p, t, 1.0 / 6.0);
  p = fma(p, t, 0.5);
  p = fma(p, t, 1.0);
  p = fma(p, t, 1.0);
  return ldexp(p, (int)n);
}

// ---------------------------------------------------------------- wave / block primitives
// Wave-wide reductions.  Within each row of 16 lanes a DPP butterfly (swap neighbours, swap
// pairs, mirror the half row, mirror the row) leaves the row's result in all 16 lanes; the four
// row results are then read with v_readlane and combined in a fixed order, so the result is
// wave-uniform and independent of which lanes are "first".
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppSwap1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppSwap2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // row_half_mirror
constexpr int kDppMirror = 0x140;      // row_mirror
__device__ __forceinline__ float lane_f(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<kDppSwap1>(v));
  v = fmaxf(v, dpp_f<kDppSwap2>(v));
  v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f<kDppMirror>(v));
  return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
  v = __fadd_rn(v, dpp_f<kDppSwap1>(v));
  v = __fadd_rn(v, dpp_f<kDppSwap2>(v));
  v = __fadd_rn(v, dpp_f<kDppHalfMirror>(v));
  v = __fadd_rn(v, dpp_f<kDppMirror>(v));
  return __fadd_rn(__fadd_rn(lane_f(v, 0), lane_f(v, 16)), __fadd_rn(lane_f(v, 32), lane_f(v, 48)));
}
template <int CTRL> __device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ int wave_min_i(int v) {
  v = min(v, dpp_i<kDppSwap1>(v));
  v = min(v, dpp_i<kDppSwap2>(v));
  v = min(v, dpp_i<kDppHalfMirror>(v));
  v = min(v, dpp_i<kDppMirror>(v));
  return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
// Inclusive prefix sum over the 64 lanes of a wave, ascending lane order, without LDS traffic:
// four DPP row shifts (1, 2, 4, 8; lanes without a source read 0) scan each row of 16 lanes,
// then the totals of rows 0..2 (lanes 15, 31, 47) are added to the rows after them in a fixed
// order.
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppWaveShr1 = 0x138;    // whole-wave shift by one lane
__device__ __forceinline__ float wave_scan_incl(float v) {
  v = __fadd_rn(v, dpp_f<kDppRowShr1>(v));
  v = __fadd_rn(v, dpp_f<kDppRowShr2>(v));
  v = __fadd_rn(v, dpp_f<kDppRowShr4>(v));
  v = __fadd_rn(v, dpp_f<kDppRowShr8>(v));
  const float t0 = lane_f(v, 15), t1 = lane_f(v, 31), t2 = lane_f(v, 47);
  const float t01 = __fadd_rn(t0, t1);
  const int row = (threadIdx.x & 63) >> 4;
  const float off = row == 0 ? 0.f : (row == 1 ? t0 : (row == 2 ? t01 : __fadd_rn(t01, t2)));
  return __fadd_rn(v, off);
}
// value of the previous lane (0 in lane 0)
__device__ __forceinline__ float wave_prev_lane(float v) { return dpp_f<kDppWaveShr1>(v); }
__device__ __forceinline__ uint32_t wave_scan_incl_u32(uint32_t v) {
  auto sh = [](uint32_t x, auto ctrl) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, decltype(ctrl)::value, 0xf, 0xf, true);
  };
  v += sh(v, std::integral_constant<int, kDppRowShr1>{});
  v += sh(v, std::integral_constant<int, kDppRowShr2>{});
  v += sh(v, std::integral_constant<int, kDppRowShr4>{});
  v += sh(v, std::integral_constant<int, kDppRowShr8>{});
  const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
  const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
  const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row == 0 ? 0u : (row == 1 ? t0 : (row == 2 ? t0 + t1 : t0 + t1 + t2)));
}

// ---------------------------------------------------------------- loads
template <int DT> __device__ __forceinline__ uint4 neg_inf_vec() {
  const uint32_t f = (DT == kDtBF16) ? 0xFF80FF80u : 0xFF800000u;
  return make_uint4(f, f, f, f);
}

// One 16-byte vector of a row starting at element e (e is a multiple of kE).  Elements at or
// beyond V read as -inf.  AL promises that the row base is 16-byte aligned and V is a positive
// multiple of kE; otherwise elements are fetched one by one.  Both paths are branch-free (the
// address is clamped into the row and the value replaced afterwards), so that all loads of a
// chunk can be in flight together.
template <int DT, int AL>
__device__ __forceinline__ uint4 load_vec(const char* __restrict__ row, int64_t e, int V) {
  constexpr int kE = Vec<DT>::kE;
  if (AL == kAlignedFull)       // the caller knows that every vector it asks for lies inside the row
    return *reinterpret_cast<const uint4*>(row + e * Vec<DT>::kES);
  if (AL) {
    const bool in = e < V;
    const int64_t ec = in ? e : int64_t(V - kE);
    uint4 v;
    if (AL == kAlignedStream) {   // read-once data: do not keep it in the caches
      typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
      const u32x4_t nv = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(row + ec * Vec<DT>::kES));
      v = make_uint4(nv.x, nv.y, nv.z, nv.w);
    } else {
      v = *reinterpret_cast<const uint4*>(row + ec * Vec<DT>::kES);
    }
    const uint4 ninf = neg_inf_vec<DT>();
    v.x = in ? v.x : ninf.x; v.y = in ? v.y : ninf.y; v.z = in ? v.z : ninf.z; v.w = in ? v.w : ninf.w;
    return v;
  }
  uint32_t w[4];
  if (DT == kDtBF16) {
    const uint16_t* r = reinterpret_cast<const uint16_t*>(row);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t i0 = e + 2 * j, i1 = e + 2 * j + 1;
      uint32_t lo = r[i0 < V ? i0 : V - 1], hi = r[i1 < V ? i1 : V - 1];
      lo = i0 < V ? lo : 0xFF80u;
      hi = i1 < V ? hi : 0xFF80u;
      w[j] = lo | (hi << 16);
    }
  } else {
    const uint32_t* r = reinterpret_cast<const uint32_t*>(row);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t i0 = e + j;
      const uint32_t x = r[i0 < V ? i0 : V - 1];
      w[j] = i0 < V ? x : 0xFF800000u;
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

template <int DT> __device__ __forceinline__ float vec_elem(const uint4& v, int j) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if (DT == kDtBF16) return (j & 1) ? bf16_hi(w[j >> 1]) : bf16_lo(w[j >> 1]);
  return __uint_as_float(w[j]);
}

// Scalar read of one logit (any alignment).
template <int DT> __device__ __forceinline__ float load_elem(const char* __restrict__ row, int64_t e) {
  if (DT == kDtBF16) return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(row)[e]) << 16);
  return reinterpret_cast<const float*>(row)[e];
}

// Logit transform, evaluated in fp32 with exactly these roundings: the difference is rounded,
// then one fused multiply-add, then one multiply by fl32(1/T).
// Guidance l_u + s (l_c - l_u).  Where both logits are -inf (a token excluded on both sides, or
// an element beyond the end of the row) the difference is NaN; fmaxf returns its other operand
// then, so such an entry stays excluded (-inf).
__device__ __forceinline__ float guide_logit(float lc, float lu, float s) {
  return fmaxf(__fmaf_rn(s, __fsub_rn(lc, lu), lu), -INFINITY);
}
__device__ __forceinline__ float transform_logit(float lc, float lu, bool guided, float s, float inv_T) {
  float l = lc;
  if (guided) l = guide_logit(lc, lu, s);
  return __fmul_rn(l, inv_T);
}

// ---------------------------------------------------------------- a row chunk in registers
// NT tiles per thread.  bf16 input without a logit transform stays packed (4 words per tile);
// otherwise kE fp32 values per tile.
template <int DT, bool XF, int NT> struct RowRegs {
  static constexpr bool kRaw = (DT == kDtBF16) && !XF;
  static constexpr int kE = Vec<DT>::kE;
  static constexpr int kWords = NT * (kRaw ? 4 : kE);
  uint32_t w[kWords];

  __device__ __forceinline__ float get(int k, int j) const {
    if (kRaw) {
      uint32_t v = w[k * 4 + (j >> 1)];
      return (j & 1) ? bf16_hi(v) : bf16_lo(v);
    }
    return __uint_as_float(w[k * kE + j]);
  }
  __device__ __forceinline__ void set(int k, int j, float v) { w[k * kE + j] = __float_as_uint(v); }
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int n = 0; n < kWords; ++n) w[n] = 0u;
  }
};

// Load the chunk of NT tiles that starts at element `base` of a row (and of its unconditional
// twin when guided) and apply the logit transform when XF: guidance, temperature, then the
// top-k mask "keep l >= thr" (thr = -inf: no mask).  Out-of-range elements become -inf.
// Vector k of thread t is vector number k*KS + t*TS of the chunk: (KS, TS) = (256, 1) is the
// tile layout described at the top; (1, NT) gives every thread NT consecutive vectors.  With a
// logit transform, KG tiles (of both tensors) are in flight at a time.
template <int DT, bool XF, int AL, int NT, int KS = kThreads, int TS = 1, int KG = 4, int GD = -1>
__device__ __forceinline__ void load_chunk(RowRegs<DT, XF, NT>& r, const char* __restrict__ cond,
                                           const char* __restrict__ uncond, int64_t base, int V,
                                           float s, float inv_T, float thr) {
  constexpr int kE = Vec<DT>::kE;
  const int tid = threadIdx.x;
  if constexpr (!XF) {
    uint4 raw[NT];
#pragma unroll
    for (int k = 0; k < NT; ++k) raw[k] = load_vec<DT, AL>(cond, base + int64_t(k * KS + tid * TS) * kE, V);
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      if (RowRegs<DT, XF, NT>::kRaw) {
        r.w[k * 4 + 0] = raw[k].x; r.w[k * 4 + 1] = raw[k].y;
        r.w[k * 4 + 2] = raw[k].z; r.w[k * 4 + 3] = raw[k].w;
      } else {
#pragma unroll
        for (int j = 0; j < kE; ++j) r.set(k, j, vec_elem<DT>(raw[k], j));
      }
    }
  } else {
    // Groups of kG tiles: the raw vectors of a group are in flight together and are consumed
    // before the next group is fetched, which bounds the registers held by raw data.  The
    // options (guided, temperature, mask) are the same for every thread, so each is one branch
    // around a loop, not a select per element.
    constexpr int kG = NT < KG ? NT : KG;
    // GD: guidance known at compile time (1 on, 0 off) or decided by the pointer (-1)
    const bool guided = GD < 0 ? (uncond != nullptr) : (GD == 1);
#pragma unroll
    for (int g = 0; g < NT; g += kG) {
      uint4 rc[kG], ru[kG];
#pragma unroll
      for (int k = 0; k < kG; ++k) rc[k] = load_vec<DT, AL>(cond, base + int64_t((g + k) * KS + tid * TS) * kE, V);
      if (guided) {
#pragma unroll
        for (int k = 0; k < kG; ++k) ru[k] = load_vec<DT, AL>(uncond, base + int64_t((g + k) * KS + tid * TS) * kE, V);
#pragma unroll
        for (int k = 0; k < kG; ++k) {
#pragma unroll
          for (int j = 0; j < kE; ++j) r.set(g + k, j, guide_logit(vec_elem<DT>(rc[k], j), vec_elem<DT>(ru[k], j), s));
        }
      } else {
#pragma unroll
        for (int k = 0; k < kG; ++k) {
#pragma unroll
          for (int j = 0; j < kE; ++j) r.set(g + k, j, vec_elem<DT>(rc[k], j));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (inv_T != 1.0f) {               // multiplying by 1 would change nothing
#pragma unroll
      for (int n = 0; n < NT * kE; ++n) r.w[n] = __float_as_uint(__fmul_rn(__uint_as_float(r.w[n]), inv_T));
    }
    if (thr > -INFINITY) {             // top-k mask: keep l >= thr
#pragma unroll
      for (int n = 0; n < NT * kE; ++n) r.w[n] = (__uint_as_float(r.w[n]) >= thr) ? r.w[n] : 0xFF800000u;
    }
  }
}

// Split form of load_chunk for code that issues loads well ahead of their use: fetch_vec only
// issues the 16-byte load (address clamped into the row, nothing depends on the result yet);
// finish_chunk later turns NT fetched vectors -- vector k of this thread starts at element
// first[k] -- into a RowRegs exactly as load_chunk would (range mask, logit transform, top-k
// mask).  Aligned rows only (see load_vec).
template <int DT>
__device__ __forceinline__ uint4 fetch_vec(const char* __restrict__ row, int64_t e, int V) {
  constexpr int kE = Vec<DT>::kE;
  const int64_t ec = e < V ? e : int64_t(V - kE);
  return *reinterpret_cast<const uint4*>(row + ec * Vec<DT>::kES);
}

template <int DT, bool XF, int NT>
__device__ __forceinline__ void finish_chunk(RowRegs<DT, XF, NT>& r, const uint4 (&rc)[NT], const uint4 (&ru)[NT],
                                             const int64_t (&first)[NT], int V, bool guided, float s, float inv_T,
                                             float thr) {
  constexpr int kE = Vec<DT>::kE;
#pragma unroll
  for (int k = 0; k < NT; ++k) {
    if constexpr (!XF) {
      const bool in = first[k] < V;
      const uint4 ninf = neg_inf_vec<DT>();
      uint4 v = rc[k];
      v.x = in ? v.x : ninf.x; v.y = in ? v.y : ninf.y; v.z = in ? v.z : ninf.z; v.w = in ? v.w : ninf.w;
      if (RowRegs<DT, XF, NT>::kRaw) {
        r.w[k * 4 + 0] = v.x; r.w[k * 4 + 1] = v.y; r.w[k * 4 + 2] = v.z; r.w[k * 4 + 3] = v.w;
      } else {
#pragma unroll
        for (int j = 0; j < kE; ++j) r.set(k, j, vec_elem<DT>(v, j));
      }
    } else {
#pragma unroll
      for (int j = 0; j < kE; ++j) {
        const float l = transform_logit(vec_elem<DT>(rc[k], j), vec_elem<DT>(ru[k], j), guided, s, inv_T);
        r.set(k, j, (first[k] + j < V && l >= thr) ? l : -INFINITY);
      }
    }
  }
}

// Per-thread softmax statistics in base-2 units with an INTEGER reference exponent:
// c = ceil(max*log2e) over the thread's logits (at least kRefFloor) and s = sum 2^(l*log2e - c).
// Because c is an integer, every later change of reference is an exact power-of-two scaling.
template <int DT, bool XF, int NT>
__device__ __forceinline__ void thread_stats(const RowRegs<DT, XF, NT>& r, float& c, float& s) {
  constexpr int kE = Vec<DT>::kE;
  float tm = r.get(0, 0);
#pragma unroll
  for (int k = 0; k < NT; ++k) {
#pragma unroll
    for (int j = 0; j < kE; ++j) tm = fmaxf(tm, r.get(k, j));
  }
  c = fmaxf(ceilf(tm * kLog2e), kRefFloor);
  s = 0.f;
#pragma unroll
  for (int k = 0; k < NT; ++k) {
#pragma unroll
    for (int j = 0; j < kE; ++j) s += exp2_fast(__fmaf_rn(r.get(k, j), kLog2e, -c));
  }
}

}  // namespace csd
