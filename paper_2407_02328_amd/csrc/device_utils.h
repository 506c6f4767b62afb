// Device helpers: 16-byte storage loads, bf16 conversion, the ranking key.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "adore_internal.h"

namespace adore {

// ---- storage access: one 16-byte vector -> EPL floats ----------------------
template <typename T>
struct Vec16;

template <>
struct Vec16<float> {
  static constexpr int EPL = 4;  // elements per 16-byte load
  __device__ static inline void load(const float *p, float (&f)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  __device__ static inline void copy(float *dst, const float *src) {
    *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
  }
  // the same in two steps: the 16 bytes as they are, and their values
  typedef float4 Raw;
  __device__ static inline Raw load_raw(const float *p) { return *reinterpret_cast<const float4 *>(p); }
  __device__ static inline void store_raw(float *p, const Raw &v) { *reinterpret_cast<float4 *>(p) = v; }
  __device__ static inline void values(const Raw &v, float (&f)[4]) {
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
};

template <>
struct Vec16<bf16_t> {
  static constexpr int EPL = 8;
  __device__ static inline void load(const bf16_t *p, float (&f)[8]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  __device__ static inline void copy(bf16_t *dst, const bf16_t *src) {
    *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
  }
  typedef uint4 Raw;
  __device__ static inline Raw load_raw(const bf16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
  __device__ static inline void store_raw(bf16_t *p, const Raw &v) { *reinterpret_cast<uint4 *>(p) = v; }
  __device__ static inline void values(const Raw &v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
};

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(bf16_t v) { return __uint_as_float(uint32_t(v.bits) << 16); }

// fp32 -> bf16, round to nearest, ties to even.  NaN stays NaN.
__device__ inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// Rotary embedding of one plane: (lo, hi) = elements j and j + d/2 of a head, cs = (cos, sin) of the angle.
// fp64 for fp32 storage.  For bf16 storage fp32 is enough (its error is a thousandth of the spacing of the storage
// values); written with explicit fused operations so that every kernel that turns a row gets the same bits.
__device__ inline double rope_lo(double lo, double hi, double2 cs) { return lo * cs.x - hi * cs.y; }
__device__ inline double rope_hi(double lo, double hi, double2 cs) { return lo * cs.y + hi * cs.x; }
__device__ inline float rope_lo(float lo, float hi, float2 cs) { return fmaf(lo, cs.x, -(hi * cs.y)); }
__device__ inline float rope_hi(float lo, float hi, float2 cs) { return fmaf(lo, cs.y, hi * cs.x); }
__device__ inline void store_elem(float *p, float v) { *p = v; }
__device__ inline void store_elem(bf16_t *p, float v) { p->bits = f32_to_bf16_rne(v); }

// ---- ranking key ------------------------------------------------------------
// Tokens of one sequence are ranked by sigma (higher is better) and, between
// equal sigma, by position (lower is better).  The 64-bit key is monotone in
// that order: larger key = better token.  Keys of distinct positions differ.
// -0 is folded into +0, NaN is treated as 0.  A valid key is never 0.
__device__ inline uint64_t rank_key(float sigma, int pos) {
  sigma = (sigma != sigma) ? 0.0f : sigma + 0.0f;
  uint32_t u = __float_as_uint(sigma);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (uint64_t(u) << 32) | uint64_t(0xffffffffu - uint32_t(pos));
}
__device__ inline int key_pos(uint64_t key) { return int(0xffffffffu - uint32_t(key & 0xffffffffu)); }

// ---- wave helpers (64 lanes) ------------------------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Scan of a 256-bin histogram from the top bin down: the bin in which the rank `need` (1 = the largest) falls, the
// rank left inside it, and how many entries it holds.  Lane l owns bins 255 - 4l .. 252 - 4l.  Wave-uniform results.
__device__ inline void pick_bin(const uint32_t *hist, int lane, int need, int &bin, int &rest, int &inbin) {
  const uint4 hq = *reinterpret_cast<const uint4 *>(hist + 252 - 4 * lane);
  const int c0 = int(hq.w), c1 = int(hq.z), c2 = int(hq.y), c3 = int(hq.x);
  const int own = c0 + c1 + c2 + c3;
  int incl = own;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int other = __shfl_up(incl, off, 64);
    if (lane >= off) incl += other;
  }
  const int excl = incl - own;
  const bool mine = excl < need && need <= incl;   // exactly one lane: need <= the number of candidates
  int b = 252 - 4 * lane, r = need - excl - c0 - c1 - c2, n = c3;
  if (need <= excl + c0) {
    b = 255 - 4 * lane; r = need - excl; n = c0;
  } else if (need <= excl + c0 + c1) {
    b = 254 - 4 * lane; r = need - excl - c0; n = c1;
  } else if (need <= excl + c0 + c1 + c2) {
    b = 253 - 4 * lane; r = need - excl - c0 - c1; n = c2;
  }
  const int src = __builtin_ctzll(__builtin_amdgcn_ballot_w64(mine));
  bin = __shfl(b, src, 64);
  rest = __shfl(r, src, 64);
  inbin = __shfl(n, src, 64);
}

// One wave's LDS operations run in order; this keeps the compiler from moving them across the point.
__device__ inline void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

}  // namespace adore
