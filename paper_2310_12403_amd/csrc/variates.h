// Random variates of smoothed dependent minibatching (App. A.7), device side.
//
// r = R / 2^32.  The "PRNG initialised with (z, t, s)" is a keyed hash: four key words K0..K3 per
// (seed, group, layer, sampler) come from one Philox4x32-10 call on the host; per source vertex t (and destination
// s for NS) the uniform is
//     LABOR-0:  U = mix(t ^ K0) ^ K1
//     NS:       U = mix(mix(t ^ K0) ^ K1 ^ mix(s ^ K2)) ^ K3
// with mix a 32-bit xorshift-multiply permutation (two multiplies): a few integer instructions per examined
// neighbour, so that the neighbour scan runs at memory speed.  Inside a group of kappa iterations the variate moves
// from U(g) to U(g+1) along n(c) = cos(c pi/2) n1 + sin(c pi/2) n2 in normal space, r = Phi(n(c)).
//
// Phi and Phi^-1 are fixed sequences of binary64 add / mul / fma and bit moves (no library calls, no division,
// no square root), so that any IEEE machine produces the same bits.  This file must be compiled with
// floating-point contraction off: every fused operation below is written as __builtin_fma.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace coop {

struct LayerKeys {
  uint32_t Ka[4];  // key words of group g
  uint32_t Kb[4];  // key words of group g + 1 (blended path only)
};

struct VariateParams {
  LayerKeys K;
  double cw, sw;   // cos(c pi/2), sin(c pi/2) (blended path only)
};

__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

// the mixer is a bijection of the 32-bit integers: its inverse (0x43021123, 0x1D69E2A5: the multipliers' inverses mod 2^32)
__host__ __device__ __forceinline__ uint32_t unmix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x43021123u;
  x ^= (x >> 15) ^ (x >> 30);
  x *= 0x1D69E2A5u;
  x ^= x >> 16;
  return x;
}

// Philox4x32-10 (Salmon et al., SC'11); host side, once per layer, for the key words.
inline void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

inline void layer_keys(uint64_t seed, int sampler, int layer, uint64_t g, uint32_t K[4]) {
  const uint32_t ctr[4] = {(uint32_t)g, (uint32_t)(g >> 32), (uint32_t)layer | ((uint32_t)sampler << 8), 0x434F4F50u};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  philox4x32_10(ctr, key, K);
}

// ---- reproducible binary64 kit ------------------------------------------------------------------------------
__device__ __forceinline__ double bits_to_f64(uint64_t u) { return __longlong_as_double((long long)u); }
__device__ __forceinline__ uint64_t f64_to_bits(double x) { return (uint64_t)__double_as_longlong(x); }

// 1/x, x positive and normal: exponent-flip first guess, six Newton steps
__device__ __forceinline__ double kit_rcp(double x) {
  double y = bits_to_f64(0x7FDE623822FC16E6ull - f64_to_bits(x));
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    const double e = __builtin_fma(-x, y, 1.0);
    y = __builtin_fma(y, e, y);
  }
  return y;
}

// 1/sqrt(x), x positive and normal: shift-and-subtract first guess, five Newton steps
__device__ __forceinline__ double kit_rsqrt(double x) {
  double y = bits_to_f64(0x5FE6EB50C7B537A9ull - (f64_to_bits(x) >> 1));
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    double t = x * y;
    t = t * y;
    y = y * __builtin_fma(-0.5, t, 1.5);
  }
  return y;
}

// ln x, x positive and normal: mantissa folded into [1/sqrt2, sqrt2), atanh series in z = (m-1)/(m+1) up to z^17
__device__ __forceinline__ double kit_log(double x) {
  const uint64_t b = f64_to_bits(x);
  long long e = (long long)(b >> 52) - 1023;
  double m = bits_to_f64((b & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull);
  if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
  const double z = (m - 1.0) * kit_rcp(m + 1.0);
  const double z2 = z * z;
  double p = 1.0 / 17.0;
  p = __builtin_fma(p, z2, 1.0 / 15.0);
  p = __builtin_fma(p, z2, 1.0 / 13.0);
  p = __builtin_fma(p, z2, 1.0 / 11.0);
  p = __builtin_fma(p, z2, 1.0 / 9.0);
  p = __builtin_fma(p, z2, 1.0 / 7.0);
  p = __builtin_fma(p, z2, 1.0 / 5.0);
  p = __builtin_fma(p, z2, 1.0 / 3.0);
  p = __builtin_fma(p, z2, 1.0);
  const double lm = (2.0 * z) * p;
  return __builtin_fma((double)e, 0.6931471805599453, lm);
}

// e^y for y in [-700, 0]: y = k ln2 + r with |r| <= ln2 / 2, Taylor polynomial to r^13, scaled by 2^k
__device__ __forceinline__ double kit_exp(double y) {
  const double magic = 6755399441055744.0;  // 1.5 * 2^52
  const double kf = __builtin_fma(y, 1.4426950408889634, magic) - magic;
  double r = __builtin_fma(-kf, 0.6931471803691238, y);
  r = __builtin_fma(-kf, 1.9082149292705877e-10, r);
  double p = 1.0 / 6227020800.0;
  p = __builtin_fma(p, r, 1.0 / 479001600.0);
  p = __builtin_fma(p, r, 1.0 / 39916800.0);
  p = __builtin_fma(p, r, 1.0 / 3628800.0);
  p = __builtin_fma(p, r, 1.0 / 362880.0);
  p = __builtin_fma(p, r, 1.0 / 40320.0);
  p = __builtin_fma(p, r, 1.0 / 5040.0);
  p = __builtin_fma(p, r, 1.0 / 720.0);
  p = __builtin_fma(p, r, 1.0 / 120.0);
  p = __builtin_fma(p, r, 1.0 / 24.0);
  p = __builtin_fma(p, r, 1.0 / 6.0);
  p = __builtin_fma(p, r, 0.5);
  p = __builtin_fma(p, r, 1.0);
  p = __builtin_fma(p, r, 1.0);
  const long long k = (long long)kf;
  return p * bits_to_f64((uint64_t)(k + 1023) << 52);
}

// Phi^-1((U + 1/2) / 2^32): Acklam's rational approximation; the upper half mirrors the lower half on U.
__device__ __forceinline__ double kit_phi_inv_u32(uint32_t U) {
  const bool upper = U >= 0x80000000u;
  const uint32_t Ul = upper ? (0xFFFFFFFFu - U) : U;
  const double p = ((double)Ul + 0.5) * (1.0 / 4294967296.0);
  double x;
  if (p < 0.02425) {
    const double w = -2.0 * kit_log(p);
    const double q = w * kit_rsqrt(w);
    double num = -7.784894002430293e-03;
    num = __builtin_fma(num, q, -3.223964580411365e-01);
    num = __builtin_fma(num, q, -2.400758277161838e+00);
    num = __builtin_fma(num, q, -2.549732539343734e+00);
    num = __builtin_fma(num, q, 4.374664141464968e+00);
    num = __builtin_fma(num, q, 2.938163982698783e+00);
    double den = 7.784695709041462e-03;
    den = __builtin_fma(den, q, 3.224671290700398e-01);
    den = __builtin_fma(den, q, 2.445134137142996e+00);
    den = __builtin_fma(den, q, 3.754408661907416e+00);
    den = __builtin_fma(den, q, 1.0);
    x = num * kit_rcp(den);
  } else {
    const double q = p - 0.5;
    const double r = q * q;
    double num = -3.969683028665376e+01;
    num = __builtin_fma(num, r, 2.209460984245205e+02);
    num = __builtin_fma(num, r, -2.759285104469687e+02);
    num = __builtin_fma(num, r, 1.383577518672690e+02);
    num = __builtin_fma(num, r, -3.066479806614716e+01);
    num = __builtin_fma(num, r, 2.506628277459239e+00);
    double den = -5.447609879822406e+01;
    den = __builtin_fma(den, r, 1.615858368580409e+02);
    den = __builtin_fma(den, r, -1.556989798598866e+02);
    den = __builtin_fma(den, r, 6.680131188771972e+01);
    den = __builtin_fma(den, r, -1.328068155288572e+01);
    den = __builtin_fma(den, r, 1.0);
    x = (q * num) * kit_rcp(den);
  }
  return upper ? -x : x;
}

// The same rational form in fp32 with the hardware's logarithm, square root and reciprocal: within 4e-4 of
// kit_phi_inv_u32 for every U (kPhiInvF32Gap in blend_filters.h; coop_selftest_phi_inv_gap measures the distance over
// all 2^32 inputs; the central branch's large alternating coefficients cancel in fp32).  Used by the filters in front
// of the exact blend, which settle a candidate with it only where ten times that distance cannot change the outcome.
__device__ __forceinline__ float approx_phi_inv_f32(uint32_t U) {
  const bool upper = U >= 0x80000000u;
  const uint32_t Ul = upper ? (0xFFFFFFFFu - U) : U;
  const float p = ((float)Ul + 0.5f) * 2.3283064365386963e-10f;
  float x;
  if (p < 0.02425f) {
    const float q = __builtin_amdgcn_sqrtf(-2.0f * __logf(p));
    float num = -7.784894002430293e-03f;
    num = __builtin_fmaf(num, q, -3.223964580411365e-01f);
    num = __builtin_fmaf(num, q, -2.400758277161838e+00f);
    num = __builtin_fmaf(num, q, -2.549732539343734e+00f);
    num = __builtin_fmaf(num, q, 4.374664141464968e+00f);
    num = __builtin_fmaf(num, q, 2.938163982698783e+00f);
    float den = 7.784695709041462e-03f;
    den = __builtin_fmaf(den, q, 3.224671290700398e-01f);
    den = __builtin_fmaf(den, q, 2.445134137142996e+00f);
    den = __builtin_fmaf(den, q, 3.754408661907416e+00f);
    den = __builtin_fmaf(den, q, 1.0f);
    x = num * __builtin_amdgcn_rcpf(den);
  } else {
    const float q = p - 0.5f;
    const float r = q * q;
    float num = -3.969683028665376e+01f;
    num = __builtin_fmaf(num, r, 2.209460984245205e+02f);
    num = __builtin_fmaf(num, r, -2.759285104469687e+02f);
    num = __builtin_fmaf(num, r, 1.383577518672690e+02f);
    num = __builtin_fmaf(num, r, -3.066479806614716e+01f);
    num = __builtin_fmaf(num, r, 2.506628277459239e+00f);
    float den = -5.447609879822406e+01f;
    den = __builtin_fmaf(den, r, 1.615858368580409e+02f);
    den = __builtin_fmaf(den, r, -1.556989798598866e+02f);
    den = __builtin_fmaf(den, r, 6.680131188771972e+01f);
    den = __builtin_fmaf(den, r, -1.328068155288572e+01f);
    den = __builtin_fmaf(den, r, 1.0f);
    x = (q * num) * __builtin_amdgcn_rcpf(den);
  }
  return upper ? -x : x;
}

// 1 / (2n + 1), n = 0..28, each the correctly rounded quotient (folded by the compiler)
__constant__ const double kInvOdd[29] = {
    1.0,        1.0 / 3.0,  1.0 / 5.0,  1.0 / 7.0,  1.0 / 9.0,  1.0 / 11.0, 1.0 / 13.0, 1.0 / 15.0,
    1.0 / 17.0, 1.0 / 19.0, 1.0 / 21.0, 1.0 / 23.0, 1.0 / 25.0, 1.0 / 27.0, 1.0 / 29.0, 1.0 / 31.0,
    1.0 / 33.0, 1.0 / 35.0, 1.0 / 37.0, 1.0 / 39.0, 1.0 / 41.0, 1.0 / 43.0, 1.0 / 45.0, 1.0 / 47.0,
    1.0 / 49.0, 1.0 / 51.0, 1.0 / 53.0, 1.0 / 55.0, 1.0 / 57.0};

// upper tail 1 - Phi(a), a >= 0: power series below 3 (28 terms), Laplace continued fraction (depth 24) above
__device__ __forceinline__ double kit_qtail(double a) {
  const double a2 = a * a;
  const double pdf = kit_exp(-0.5 * a2) * 0.3989422804014327;
  if (a < 3.0) {
    double s = 1.0;
#pragma unroll
    for (int n = 28; n >= 1; --n) s = __builtin_fma(a2 * kInvOdd[n], s, 1.0);
    return __builtin_fma(-(pdf * a), s, 0.5);
  } else {
    double p = 0.0, q = 1.0;
#pragma unroll
    for (int n = 24; n >= 1; --n) {
      const double pn = (double)n * q;
      q = __builtin_fma(a, q, p);
      p = pn;
    }
    const double den = __builtin_fma(a, q, p);
    return (pdf * q) * kit_rcp(den);
  }
}

// floor(2^32 Phi(x)) clamped to 32 bits; the upper half is the integer mirror of the lower half
__device__ __forceinline__ uint32_t kit_phi_to_u32(double x) {
  const bool neg = x < 0.0;
  const double a = neg ? -x : x;
  const double s = kit_qtail(a) * 4294967296.0;
  unsigned long long f = (unsigned long long)s;
  if (f > 0xFFFFFFFFull) f = 0xFFFFFFFFull;
  const uint32_t lo = (uint32_t)f;
  return neg ? lo : (0xFFFFFFFFu - lo);
}

// sigma = mix(s ^ K2) of the destination, wave-uniform; NS only
__device__ __forceinline__ uint32_t ns_sigma(const uint32_t K[4], uint32_t s) { return mix32(s ^ K[2]); }

template <bool NS>
__device__ __forceinline__ uint32_t keyed_uniform(const uint32_t K[4], uint32_t t, uint32_t sigma) {
  const uint32_t a = mix32(t ^ K[0]) ^ K[1];
  if constexpr (!NS) return a;
  else return mix32(a ^ sigma) ^ K[3];
}

// R for source vertex t; for NS, sigma_a / sigma_b are ns_sigma(Ka, s) / ns_sigma(Kb, s) of the destination s
template <bool NS, bool BLEND>
__device__ __forceinline__ uint32_t variate(const LayerKeys& K, double cw, double sw, uint32_t t, uint32_t sigma_a,
                                            uint32_t sigma_b) {
  const uint32_t U1 = keyed_uniform<NS>(K.Ka, t, sigma_a);
  if constexpr (!BLEND) {
    return U1;
  } else {
    const uint32_t U2 = keyed_uniform<NS>(K.Kb, t, sigma_b);
    const double n1 = kit_phi_inv_u32(U1);
    const double n2 = kit_phi_inv_u32(U2);
    return kit_phi_to_u32(__builtin_fma(cw, n1, sw * n2));
  }
}

template <bool NS, bool BLEND>
__device__ __forceinline__ uint32_t variate(const VariateParams& vp, uint32_t t, uint32_t sigma_a, uint32_t sigma_b) {
  return variate<NS, BLEND>(vp.K, vp.cw, vp.sw, t, sigma_a, sigma_b);
}

}  // namespace coop
