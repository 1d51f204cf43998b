// Thresholds of the filters that stand between a blended variate (c > 0) and its exact evaluation.  For a keep test
// R <= thr with R = floor(2^32 Phi(cw n1 + sw n2)), n_i = Phi^-1((U_i + 1/2) / 2^32), they bound, per threshold thr:
// the two uniforms in integers (first filter), and the blend computed in fp32 from above and from below (second
// filter).  Used by the LABOR-0 scan (thr = the list's keep threshold) and by NS (thr = the list's candidate bound).
#pragma once
#include "variates.h"

namespace coop {

// The margins of the filters (read from this file by the tests that restate the filters on the CPU).
// kPhiInvF32Gap: the largest distance between approx_phi_inv_f32(U) and kit_phi_inv_u32(U) over all 2^32 values of U that
// the filters rely on; a GPU test evaluates both for every U and fails if the distance is ever larger.
// kPhiInvF32Allow: what the filters allow for per unit of weight: ten times that, so that the rounding of the fp32
// products and sums (below 2e-6 at |n| <= 7) and of the float weights never matters.
constexpr double kPhiInvF32Gap = 4e-4;
constexpr double kPhiInvF32Allow = 4e-3;
constexpr double kBlendRelWiden = 1e-6;   // relative widening of every bound (the kit's own error is 1.2e-9)
constexpr double kBlendAbsWiden = 1e-5;   // absolute widening of the fp32 limits
constexpr double kStripShift = 0.6;       // the strip's edge lies this many standard deviations below the L-shape's
constexpr uint32_t kThrWiden = 8u;        // thresholds are moved outwards by this many units of 2^-32 first

// Second filter of the blended path: the blend itself in fp32.  A kept edge has n = cw n1 + sw n2 below
// tau = Phi^-1 of slightly more than (thr + 1) / 2^32; the fp32 estimate of n (two approx_phi_inv_f32, each within
// kPhiInvF32Gap of the kit's value; kPhiInvF32Allow is allowed for) must therefore lie below the value returned here, rounded up to a float.
__device__ __forceinline__ float blend_second_threshold(uint32_t thr, double cs /* cw + sw */) {
  if (thr >= 0x7FFFFFF0u) return __builtin_inff();
  const double tau = kit_phi_inv_u32(thr + kThrWiden);
  const double lim = __builtin_fma(cs, kPhiInvF32Allow, tau * (1.0 - kBlendRelWiden)) + kBlendAbsWiden;
  float t = (float)lim;
  if ((double)t < lim) t = __uint_as_float(t >= 0.0f ? __float_as_uint(t) + 1u : __float_as_uint(t) - 1u);  // next float up
  return t;
}

// The other side of the second filter: an fp32 estimate at or below this value means that the exact blend keeps the
// edge (tau_lo = Phi^-1 of slightly less than thr / 2^32, less the same allowances, rounded down to a float).
__device__ __forceinline__ float blend_keep_threshold(uint32_t thr, double cs /* cw + sw */) {
  if (thr == 0xFFFFFFFFu) return __builtin_inff();  // the whole list is kept
  if (thr < 64u) return -__builtin_inff();
  const double tau_lo = kit_phi_inv_u32(thr - kThrWiden);
  const double lim = tau_lo - kBlendRelWiden * (tau_lo < 0.0 ? -tau_lo : tau_lo) - cs * kPhiInvF32Allow - kBlendAbsWiden;
  float t = (float)lim;
  if ((double)t > lim) t = __uint_as_float(t > 0.0f ? __float_as_uint(t) - 1u : __float_as_uint(t) + 1u);  // next float down
  return t;
}


// Blended variates (c > 0) cost two Phi^-1 and one Phi per neighbour, about a hundred times the integer path.  A cheap
// necessary condition in integers keeps them off almost every neighbour.  A kept edge has n = cw n1 + sw n2 below
// tau = Phi^-1 of slightly more than (thr + 1) / 2^32.  With lo = min(U1, U2), hi = max(U1, U2) and cM >= cm the two
// weights, n >= cM Phi^-1(lo) + cm Phi^-1(hi) >= (cw + sw) Phi^-1(lo).  So the edge lies in the L-shaped region
// lo <= a2 = 2^32 Phi(tau / (cw + sw)); and inside it either in the strip lo <= a1 (a1 < a2), or, with x1 = Phi^-1(a1),
// below hi <= b2 = 2^32 Phi((tau - cM x1) / cm).  The bounds are widened by 1e-6 relative and a few units so that the
// approximation errors of the kit (1.2e-9) can never matter; they are computed once per list and layer.
struct PreThr {
  uint32_t a2;  // lo <= a2 is necessary
  uint32_t a1;  // lo <= a1 is sufficient for a candidate
  uint32_t b2;  // otherwise hi <= b2 is necessary as well
  float keep2;  // second filter: an fp32 blend at or below this is kept without the exact stage
};

__device__ __forceinline__ uint32_t blend_widen(uint32_t R) {
  const double lim = (double)R * (1.0 + kBlendRelWiden) + 16.0;
  return lim >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)lim;
}

__device__ __forceinline__ PreThr blend_first_thresholds(uint32_t thr, double cw, double sw) {
  if (thr >= 0x7FFFFFF0u) return PreThr{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0.0f};  // k / d near or above 1/2: no useful bound
  const double tau_s = kit_phi_inv_u32(thr + kThrWiden) * (1.0 - kBlendRelWiden);  // < 0
  const double x2 = tau_s * kit_rcp(cw + sw);
  PreThr p;
  p.a2 = blend_widen(kit_phi_to_u32(x2));
  p.a1 = kit_phi_to_u32(x2 - kStripShift);
  const double x1 = kit_phi_inv_u32(p.a1);
  const double cM = cw > sw ? cw : sw, cm = cw > sw ? sw : cw;
  double y2 = (tau_s - cM * x1) * kit_rcp(cm);
  y2 = y2 + kBlendRelWiden * (y2 < 0.0 ? -y2 : y2) + 1e-9;
  p.b2 = y2 >= 6.0 ? 0xFFFFFFFFu : blend_widen(kit_phi_to_u32(y2));
  p.keep2 = 0.0f;
  return p;
}

}  // namespace coop
