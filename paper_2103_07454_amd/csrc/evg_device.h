// Device-side helpers for the gfx950 kernels: fixed-order reductions and scans
// over 64-lane wavefronts, and the counter-based gradient generator.
#pragma once
#include "evg_internal.h"

namespace evg {

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }
__device__ __forceinline__ uint32_t wave_id() { return threadIdx.x >> 6; }

// The iteration number and decay^k of the step in flight (uniform loads).
__device__ __forceinline__ uint32_t step_k(const Tables& T, const StepArgs& A) {
  return A.from_device ? T.it->k : A.k;
}
__device__ __forceinline__ double step_decay(const Tables& T, const StepArgs& A) {
  return A.from_device ? T.it->decay_pow : A.decay_pow;
}

// Streaming (non-temporal) 16-byte accesses: every arena is far larger than the
// caches and is touched once per pass, so lines are not worth keeping.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4s(const float* p) {
  const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4s(float* p, float4 a) {
  f32x4 v;
  v.x = a.x; v.y = a.y; v.z = a.z; v.w = a.w;
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}

// Sum over the 64 lanes by xor butterflies: every lane ends with the same value,
// and the association order is fixed, so results repeat bit for bit.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Sum over a 256-thread workgroup; valid in every thread.  `ws` is 4 doubles of LDS.
__device__ __forceinline__ double block_sum(double v, double* ws) {
  v = wave_sum(v);
  if (lane_id() == 0) ws[wave_id()] = v;
  __syncthreads();
  const double total = ((ws[0] + ws[1]) + ws[2]) + ws[3];
  __syncthreads();
  return total;
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves, no LDS traffic:
// shifted adds by 1, 2, 4, 8 inside each row of 16 lanes (lanes shifted in from outside a row
// read 0), then the last lane of rows 0 and 2 is added to rows 1 and 3, and lane 31 (by then the
// sum of rows 0-1) to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);   // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);   // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);   // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);   // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, true);   // row_bcast:15 -> rows 1, 3
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, true);   // row_bcast:31 -> rows 2, 3
  return v;
}

// Exclusive prefix sum over the threads of a workgroup of W wavefronts (thread
// order); *total receives the workgroup sum.  `ws` is W uint32 of LDS.
template <int W>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* ws, uint32_t* total) {
  const uint32_t incl = wave_incl_scan(v);
  if (lane_id() == 63) ws[wave_id()] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const uint32_t s = ws[w];
    if ((uint32_t)w < wave_id()) before += s;
    all += s;
  }
  __syncthreads();
  *total = all;
  return before + incl - v;
}

// The same over 64-bit words that pack four 16-bit counters none of which can overflow its
// field (so the two 32-bit halves scan independently), two such words at once: one barrier pair
// serves both.  `ws` is 2 * W uint64 of LDS.
template <int W>
__device__ __forceinline__ void block_excl_scan64x2(uint64_t a, uint64_t b, uint64_t* ws, uint64_t* ex_a,
                                                    uint64_t* ex_b, uint64_t* total_a, uint64_t* total_b) {
  const uint64_t ia = ((uint64_t)wave_incl_scan((uint32_t)(a >> 32)) << 32) | wave_incl_scan((uint32_t)a);
  const uint64_t ib = ((uint64_t)wave_incl_scan((uint32_t)(b >> 32)) << 32) | wave_incl_scan((uint32_t)b);
  if (lane_id() == 63) { ws[wave_id()] = ia; ws[W + wave_id()] = ib; }
  __syncthreads();
  uint64_t before_a = 0, all_a = 0, before_b = 0, all_b = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const uint64_t sa = ws[w], sb = ws[W + w];
    if ((uint32_t)w < wave_id()) { before_a += sa; before_b += sb; }
    all_a += sa;
    all_b += sb;
  }
  __syncthreads();
  *total_a = all_a;
  *total_b = all_b;
  *ex_a = before_a + ia - a;
  *ex_b = before_b + ib - b;
}

// The same accesses with the choice left to the caller: a ring whose arenas fit the
// last-level cache is better served by ordinary cached accesses (measured 10 % per step
// on an 8-worker ResNet-20-sized ring).
template <bool STREAM>
__device__ __forceinline__ float4 ld4t(const float* p) {
  if (STREAM) return ld4s(p);
  return *reinterpret_cast<const float4*>(p);
}
template <bool STREAM>
__device__ __forceinline__ void st4t(float* p, float4 a) {
  if (STREAM) st4s(p, a);
  else *reinterpret_cast<float4*>(p) = a;
}

// ----------------------------------------------------------------------------
// Synthetic gradients.  Philox4x32-10 (Salmon et al., SC'11): ten rounds, each
// two 32x32->64 multiplies by fixed odd constants followed by xors with the
// neighbouring words and the round key; the key advances by Weyl constants.
// ----------------------------------------------------------------------------
struct Rand4 { uint32_t w[4]; };

__device__ __forceinline__ Rand4 philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                        uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t y0 = hi1 ^ c1 ^ k0, y2 = hi0 ^ c3 ^ k1;
    c0 = y0; c1 = lo1; c2 = y2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Rand4 r;
  r.w[0] = c0; r.w[1] = c1; r.w[2] = c2; r.w[3] = c3;
  return r;
}

// Top 23 bits to a float in (0,1); exact.
__device__ __forceinline__ float unit_open(uint32_t w) {
  return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f;
}

// log of a normal positive float with only + * / fma, so that it rounds the same
// on any IEEE machine: split off the exponent, fold the mantissa into
// (sqrt(1/2), sqrt(2)], then the odd series of 2 atanh((m-1)/(m+1)).
__device__ __forceinline__ float ln_series(float u) {
  const uint32_t b = __float_as_uint(u);
  int e = (int)(b >> 23) - 127;
  float m = __uint_as_float((b & 0x007FFFFFu) | 0x3F800000u);
  if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
  const float t = m - 1.0f;
  const float s = t / (2.0f + t);
  const float w = s * s;
  float p = __builtin_fmaf(w, 0.111111112f, 0.142857149f);
  p = __builtin_fmaf(w, p, 0.2f);
  p = __builtin_fmaf(w, p, 0.333333343f);
  p = __builtin_fmaf(w, p, 1.0f);
  const float lm = (s + s) * p;
  return __builtin_fmaf((float)e, 0.693147182f, lm);
}

// (cos, sin)(2 pi u), u in [0,1): quarter turns split off exactly, Taylor series
// on the remaining [-pi/4, pi/4].
__device__ __forceinline__ void turn_cos_sin(float u, float& c, float& s) {
  const float a = 4.0f * u;
  const int qi = (int)(a + 0.5f);
  const float r = a - (float)qi;
  const float th = r * 1.57079637f;
  const float q = th * th;
  float sp = __builtin_fmaf(q, 2.75573192e-6f, -1.98412701e-4f);
  sp = __builtin_fmaf(q, sp, 8.33333377e-3f);
  sp = __builtin_fmaf(q, sp, -0.166666672f);
  sp = __builtin_fmaf(q, sp, 1.0f);
  const float sn = th * sp;
  float cp = __builtin_fmaf(q, -2.75573188e-7f, 2.48015876e-5f);
  cp = __builtin_fmaf(q, cp, -1.38888892e-3f);
  cp = __builtin_fmaf(q, cp, 4.16666679e-2f);
  cp = __builtin_fmaf(q, cp, -0.5f);
  const float cs = __builtin_fmaf(q, cp, 1.0f);
  // quarter turns: odd ones swap the two series; the signs follow from the quadrant
  // (cos is negated in quadrants 1 and 2, sin in 2 and 3), applied as sign-bit flips
  const uint32_t quad = (uint32_t)qi & 3u;
  const bool swap = (quad & 1u) != 0;
  const uint32_t cneg = ((quad + 1u) & 2u) << 30, sneg = (quad & 2u) << 30;
  c = __uint_as_float(__float_as_uint(swap ? sn : cs) ^ cneg);
  s = __uint_as_float(__float_as_uint(swap ? cs : sn) ^ sneg);
}

// Box-Muller on words (0,1) and (2,3): radius from the first, angle from the second.
__device__ __forceinline__ void normals4(const Rand4& r, float z[4]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const float ua = unit_open(r.w[2 * h]);
    const float ub = unit_open(r.w[2 * h + 1]);
    const float rad = __builtin_sqrtf(-2.0f * ln_series(ua));
    float c, s;
    turn_cos_sin(ub, c, s);
    z[2 * h] = rad * c;
    z[2 * h + 1] = rad * s;
  }
}

// e^y for 0 <= y < 80 with only + * fma: the nearest multiple n of ln 2 is taken out in two
// parts (high and low word of ln 2), the remainder's exponential is its Taylor polynomial of
// degree six, and 2^n is added into the exponent field.
__device__ __forceinline__ float exp_series(float y) {
  const int n = (int)(y * 1.44269502f + 0.5f);
  const float nf = (float)n;
  const float r = __builtin_fmaf(-nf, 1.42860677e-6f, __builtin_fmaf(-nf, 0.693145752f, y));
  float p = __builtin_fmaf(r, 1.38888892e-3f, 8.33333377e-3f);
  p = __builtin_fmaf(r, p, 4.16666679e-2f);
  p = __builtin_fmaf(r, p, 0.166666672f);
  p = __builtin_fmaf(r, p, 0.5f);
  p = __builtin_fmaf(r, p, 1.0f);
  p = __builtin_fmaf(r, p, 1.0f);
  return __uint_as_float(__float_as_uint(p) + ((uint32_t)n << 23));
}

// Student-t with 3 degrees of freedom from two random words by the polar method (Bailey 1994):
// a spherical bivariate t has squared radius 3 (u^(-2/3) - 1) for a uniform u, and its first
// component, radius times the cosine of a uniform angle, is Student-t(3).
__device__ __forceinline__ float student_t3(uint32_t wr, uint32_t wa) {
  const float y = 0.666666687f * -ln_series(unit_open(wr));
  const float rad = __builtin_sqrtf(3.0f * (exp_series(y) - 1.0f));
  float c, s;
  turn_cos_sin(unit_open(wa), c, s);
  return rad * c;
}

// Key that ranks elements for Top-K: the bit pattern of a non-negative float is
// monotone in its value, so unsigned compares order magnitudes.
__device__ __forceinline__ uint32_t rank_key(float xv, float hv, uint32_t by_value) {
  return __float_as_uint(__builtin_fabsf(by_value ? xv : xv - hv));
}

}  // namespace evg
