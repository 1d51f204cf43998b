"""The GPU's blended LABOR-0 scan reaches the exact Phi / Phi^-1 evaluation through two cheap filters: integer bounds
on the two uniforms (an L-shaped region, refined to a strip and a corner rectangle) and the blend in fp32 with a
safety margin.  This checks, on the CPU and with the oracle's bit-identical arithmetic kit, that each filter is a
necessary condition: whenever the exact variate keeps an edge, the filter passes it.  (The GPU parity tests then check
the kernel that uses them.)"""
import math
import os
import re

import numpy as np

from oracle import coopref as R

M32 = 0xFFFFFFFF

# The margins are the HIP path's own: read from the header that the kernels are compiled from, so that a margin that
# drifts there is the margin that is checked here.
_HDR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2310_12403_amd", "csrc", "blend_filters.h")


def header_constants():
    text = open(_HDR).read()
    found = dict(re.findall(r"constexpr (?:double|uint32_t) (k[A-Za-z0-9]+) = ([0-9.eE+-]+)u?;", text))
    return {k: float(v) for k, v in found.items()}


_K = header_constants()
GAP = _K["kPhiInvF32Gap"]          # claimed distance between the fp32 and the binary64 Phi^-1 (measured on the GPU for every input)
REL, ABS = _K["kBlendRelWiden"], _K["kBlendAbsWiden"]
THR_WIDEN = int(_K["kThrWiden"])


def test_header_margins_are_the_ones_the_kernels_use():
    """Every margin named in the header is used by the threshold functions in it (and not replaced by a literal), and the
    allowance leaves room: ten times the claimed distance."""
    text = open(_HDR).read()
    for name in ("kPhiInvF32Allow", "kBlendRelWiden", "kBlendAbsWiden", "kStripShift", "kThrWiden"):
        assert len(re.findall(r"\b%s\b" % name, text)) >= 2, name
    body = text[text.index("blend_second_threshold"):]
    assert not re.search(r"[^0-9a-zA-Z_.](4e-3|1e-5|0\.6)[^0-9]", body)
    assert _K["kPhiInvF32Allow"] >= 10 * GAP > 0 and REL >= 1e-7 and THR_WIDEN >= 1


def pre_threshold(L, thr, cw, sw):
    """The L-shaped region alone: min(U1, U2) <= a2 of first_thresholds() below."""
    return first_thresholds(L, thr, cw, sw)[1]


def test_pre_threshold_never_rejects_a_kept_edge():
    L = R.lib()
    rng = np.random.default_rng(0)
    checked = kept = 0
    for trial in range(400):
        k = int(rng.integers(1, 60))
        d = int(k + 1 + 10 ** rng.uniform(0, 5))
        thr = (k << 32) // d
        kappa = int(rng.integers(2, 300))
        i = int(rng.integers(1, kappa))
        c = i / kappa
        cw, sw = math.cos(c * 1.5707963267948966), math.sin(c * 1.5707963267948966)
        P = pre_threshold(L, thr, cw, sw)
        # uniforms concentrated where keeps happen: around the corner of the L-shaped region and below
        base = min(P, M32 - 1)
        cands = []
        for _ in range(60):
            scale = 10 ** rng.uniform(-3, 0.3)
            U1 = min(M32, int(base * scale * rng.uniform(0.2, 1.5)))
            U2 = min(M32, int(base * scale * rng.uniform(0.2, 1.5)))
            cands.append((U1, U2))
        for dlt in range(-3, 4):      # the corner itself and its neighbours
            cands.append((max(0, min(M32, P + dlt)), max(0, min(M32, P + dlt))))
        for U1, U2 in cands:
            # the oracle's variate() evaluates exactly this blend for a (seed, t) pair; here the two uniforms are
            # fed in directly through the kit so that chosen (U1, U2) pairs can be probed
            n1, n2 = L.coopref_phi_inv_u32(U1), L.coopref_phi_inv_u32(U2)
            n = float(np.float64(cw) * np.float64(n1) + np.float64(sw) * np.float64(n2))   # within 1 ulp of the fma
            for nn in (n, np.nextafter(n, -np.inf), np.nextafter(n, np.inf)):
                Rv = L.coopref_phi_to_u32(float(nn))
                checked += 1
                if Rv <= thr:
                    kept += 1
                    assert min(U1, U2) <= P, (thr, c, U1, U2, Rv, P)
    assert kept > 2000 and checked > 50000


def test_pre_threshold_is_selective():
    """At k/d = 10/1400 the filter passes a few percent of the neighbours, not most of them."""
    L = R.lib()
    thr = (10 << 32) // 1400
    for c in (1 / 16, 0.5, 15 / 16):
        cw, sw = math.cos(c * math.pi / 2), math.sin(c * math.pi / 2)
        P = pre_threshold(L, thr, cw, sw)
        frac = 1 - (1 - P / 2**32) ** 2
        assert thr < P and frac < 0.1


# --------------------------------------------------------------------------- #
# Second filter: the blend itself in fp32 with a safety margin
# --------------------------------------------------------------------------- #
EPS2 = _K["kPhiInvF32Allow"]   # allowance for one fp32 Phi^-1 against the fp64 kit's (the distance itself stays below
                               # kPhiInvF32Gap: the central branch's large alternating coefficients cancel in fp32)


def fmaf(a, b, c):
    """Single-rounding fused multiply-add of float32 values: the product of two 24-bit significands is exact in binary64, and
    the sum is rounded to binary64 and then to float32 (a double rounding that differs from the fused result only in
    vanishingly rare ties)."""
    return np.float32(np.float64(a) * np.float64(b) + np.float64(c))


def approx_phi_inv_f32(U):
    """Restatement of approx_phi_inv_f32() in csrc/variates.h: Acklam's rational form of Phi^-1((U + 1/2) / 2^32)
    evaluated in fp32 with fused multiply-adds (the GPU uses its hardware log2 / sqrt / reciprocal, each good to about one
    ulp; numpy's are correctly rounded: the difference is far inside the margin)."""
    f = np.float32
    upper = U >= 0x80000000
    Ul = (M32 - U) if upper else U
    p = (f(Ul) + f(0.5)) * f(1.0 / 4294967296.0)
    if p < f(0.02425):
        q = np.sqrt(f(-2.0) * np.log(p, dtype=np.float32), dtype=np.float32)
        num = f(-7.784894002430293e-03)
        for c in (-3.223964580411365e-01, -2.400758277161838e+00, -2.549732539343734e+00, 4.374664141464968e+00, 2.938163982698783e+00):
            num = fmaf(num, q, f(c))
        den = f(7.784695709041462e-03)
        for c in (3.224671290700398e-01, 2.445134137142996e+00, 3.754408661907416e+00, 1.0):
            den = fmaf(den, q, f(c))
        x = f(num * (f(1.0) / den))
    else:
        q = f(p - f(0.5))
        r = f(q * q)
        num = f(-3.969683028665376e+01)
        for c in (2.209460984245205e+02, -2.759285104469687e+02, 1.383577518672690e+02, -3.066479806614716e+01, 2.506628277459239e+00):
            num = fmaf(num, r, f(c))
        den = f(-5.447609879822406e+01)
        for c in (1.615858368580409e+02, -1.556989798598866e+02, 6.680131188771972e+01, -1.328068155288572e+01, 1.0):
            den = fmaf(den, r, f(c))
        x = f(f(q * num) * (f(1.0) / den))
    return f(-x) if upper else x


def second_threshold(L, thr, cw, sw):
    """Restatement of blend_second_threshold() in csrc/blend_filters.h: keep needs n = cw n1 + sw n2 below this."""
    if thr >= 0x7FFFFFF0:
        return np.float32(np.inf)
    tau = L.coopref_phi_inv_u32(thr + THR_WIDEN)
    lim = tau * (1.0 - REL) + (cw + sw) * EPS2 + ABS
    t = np.float32(lim)
    return np.nextafter(t, np.float32(np.inf)) if float(t) < lim else t


def test_fp32_phi_inv_is_close_to_the_kit():
    L = R.lib()
    rng = np.random.default_rng(1)
    worst = 0.0
    Us = [0, 1, 2, 3, 100, M32, M32 - 1, 0x7FFFFFFF, 0x80000000, int(0.02425 * 2**32), int(0.02425 * 2**32) + 1]
    Us += [int(x) for x in rng.integers(0, 1 << 32, 20000)]
    Us += [int(10 ** rng.uniform(0, 9.6)) for _ in range(20000)]
    for U in Us:
        worst = max(worst, abs(float(approx_phi_inv_f32(U)) - L.coopref_phi_inv_u32(U)))
    assert worst < GAP, worst


def test_second_filter_never_rejects_a_kept_edge():
    from scipy.special import ndtr, ndtri
    L = R.lib()
    rng = np.random.default_rng(2)
    checked = kept = rejected = 0
    for trial in range(300):
        k = int(rng.integers(1, 60))
        d = int(k + 1 + 10 ** rng.uniform(0, 5))
        thr = (k << 32) // d
        kappa = int(rng.integers(2, 300))
        i = int(rng.integers(1, kappa))
        c = i / kappa
        cw, sw = math.cos(c * 1.5707963267948966), math.sin(c * 1.5707963267948966)
        T2 = second_threshold(L, thr, cw, sw)
        tau = float(ndtri((thr + 0.5) / 2**32))
        cands = []
        for _ in range(40):
            # pairs whose blend lands near the keep boundary: pick n1, solve n2, perturb a little
            n1 = float(rng.normal())
            n2 = (tau - cw * n1) / sw + float(rng.normal()) * 10 ** rng.uniform(-6, -1)
            U1 = int(min(M32, max(0, ndtr(n1) * 2**32)))
            U2 = int(min(M32, max(0, ndtr(n2) * 2**32)))
            cands.append((U1, U2))
            cands.append((int(rng.integers(0, 1 << 32)), int(rng.integers(0, 1 << 32))))
        for U1, U2 in cands:
            n = np.float64(cw) * np.float64(L.coopref_phi_inv_u32(U1)) + np.float64(sw) * np.float64(L.coopref_phi_inv_u32(U2))
            n_hat = np.float32(np.float32(cw) * approx_phi_inv_f32(U1)) + np.float32(np.float32(sw) * approx_phi_inv_f32(U2))
            passes = bool(n_hat <= T2)
            for nn in (float(n), float(np.nextafter(n, -np.inf)), float(np.nextafter(n, np.inf))):
                checked += 1
                if L.coopref_phi_to_u32(nn) <= thr:
                    kept += 1
                    assert passes, (thr, c, U1, U2, float(n), float(n_hat), float(T2))
                elif not passes:
                    rejected += 1
    assert kept > 3000 and rejected > 3000 and checked > 60000


def test_second_filter_is_selective():
    """At k/d = 10/1400 and c = 1/2 the second filter passes little more than the edges that are kept."""
    from scipy.special import ndtri
    L = R.lib()
    thr = (10 << 32) // 1400
    cw = sw = math.cos(math.pi / 4)
    T2 = float(second_threshold(L, thr, cw, sw))
    tau = float(ndtri(thr / 2**32))
    from scipy.special import ndtr
    assert ndtr(T2) / ndtr(tau) < 1.03       # n ~ N(0, 1): pass probability against keep probability


# --------------------------------------------------------------------------- #
# First filter, refined: a strip and a corner rectangle instead of the L-shaped region
# --------------------------------------------------------------------------- #
STRIP_SHIFT = _K["kStripShift"]     # the strip's edge lies this far (in standard deviations) below the L-shape's


def first_thresholds(L, thr, cw, sw):
    """Restatement of blend_first_thresholds() in csrc/blend_filters.h: with lo = min(U1, U2), hi = max(U1, U2), a kept edge
    has lo <= a1, or lo <= a2 and hi <= b2."""
    if thr >= 0x7FFFFFF0:
        return M32, M32, M32
    tau_s = L.coopref_phi_inv_u32(thr + THR_WIDEN) * (1.0 - REL)
    widen = lambda R: M32 if float(R) * (1.0 + REL) + 16.0 >= 4294967295.0 else int(float(R) * (1.0 + REL) + 16.0)
    x2 = tau_s * L.coopref_rcp(cw + sw)
    a2 = widen(L.coopref_phi_to_u32(x2))
    a1 = L.coopref_phi_to_u32(x2 - STRIP_SHIFT)
    x1 = L.coopref_phi_inv_u32(a1)
    cM, cm = max(cw, sw), min(cw, sw)
    y2 = (tau_s - cM * x1) * L.coopref_rcp(cm)
    y2 = y2 + REL * abs(y2) + 1e-9
    b2 = M32 if y2 >= 6.0 else widen(L.coopref_phi_to_u32(y2))
    return a1, a2, b2


def test_refined_first_filter_never_rejects_a_kept_edge():
    from scipy.special import ndtr, ndtri
    L = R.lib()
    rng = np.random.default_rng(3)
    checked = kept = rejected = 0
    for trial in range(400):
        k = int(rng.integers(1, 60))
        d = int(k + 1 + 10 ** rng.uniform(0, 5))
        thr = (k << 32) // d
        kappa = int(rng.integers(2, 300))
        i = int(rng.integers(1, kappa))
        c = i / kappa
        cw, sw = math.cos(c * 1.5707963267948966), math.sin(c * 1.5707963267948966)
        a1, a2, b2 = first_thresholds(L, thr, cw, sw)
        assert a1 <= a2
        tau = float(ndtri((thr + 0.5) / 2**32))
        cands = []
        for _ in range(40):
            n1 = float(rng.normal()) - (2.0 if rng.random() < 0.5 else 0.0)
            n2 = (tau - cw * n1) / sw + float(rng.normal()) * 10 ** rng.uniform(-6, -1)
            if rng.random() < 0.5:      # also the mirror image: the small uniform in the other seat
                n2b = float(rng.normal()) - 2.0
                n1, n2 = (tau - sw * n2b) / cw + float(rng.normal()) * 10 ** rng.uniform(-6, -1), n2b
            cands.append((int(min(M32, max(0, ndtr(n1) * 2**32))), int(min(M32, max(0, ndtr(n2) * 2**32)))))
        for base in (a1, a2, b2):       # the rectangle's corners and their neighbours
            for dl in range(-2, 3):
                v = max(0, min(M32, base + dl))
                cands += [(v, min(M32, b2 + 1)), (min(M32, b2 + 1), v), (v, v), (v, b2), (b2, v)]
        for U1, U2 in cands:
            n = np.float64(cw) * np.float64(L.coopref_phi_inv_u32(U1)) + np.float64(sw) * np.float64(L.coopref_phi_inv_u32(U2))
            lo, hi = min(U1, U2), max(U1, U2)
            passes = lo <= a1 or (lo <= a2 and hi <= b2)
            for nn in (float(n), float(np.nextafter(n, -np.inf)), float(np.nextafter(n, np.inf))):
                checked += 1
                if L.coopref_phi_to_u32(nn) <= thr:
                    kept += 1
                    assert passes, (thr, c, U1, U2, float(n), a1, a2, b2)
                elif not passes:
                    rejected += 1
    assert kept > 3000 and rejected > 3000 and checked > 60000


def test_refined_first_filter_is_more_selective():
    """At k/d = 10/1400 and c = 1/2 the strip + rectangle passes less than a third of what the L-shape passes."""
    L = R.lib()
    thr = (10 << 32) // 1400
    cw = sw = math.cos(math.pi / 4)
    a1, a2, b2 = first_thresholds(L, thr, cw, sw)
    p1, p2, q = a1 / 2**32, a2 / 2**32, b2 / 2**32
    old = 1 - (1 - p2) ** 2
    new = (1 - (1 - p1) ** 2) + 2 * (p2 - p1) * q - (p2 - p1) ** 2
    assert new < old / 3, (old, new)


# --------------------------------------------------------------------------- #
# The fp32 blend also settles most candidates the other way: safely below the threshold means kept
# --------------------------------------------------------------------------- #
def keep_threshold(L, thr, cw, sw):
    """Restatement of blend_keep_threshold() in csrc/blend_filters.h: an fp32 estimate at or below this means the exact blend
    keeps the edge."""
    if thr == M32:
        return np.float32(np.inf)           # the whole list is kept
    if thr < 64:
        return np.float32(-np.inf)
    tau_lo = L.coopref_phi_inv_u32(thr - THR_WIDEN)
    lim = tau_lo - REL * abs(tau_lo) - (cw + sw) * EPS2 - ABS
    t = np.float32(lim)
    return np.nextafter(t, np.float32(-np.inf)) if float(t) > lim else t


def test_fp32_blend_below_the_keep_threshold_means_kept():
    from scipy.special import ndtr, ndtri
    L = R.lib()
    rng = np.random.default_rng(4)
    certain = band = checked = 0
    for trial in range(400):
        k = int(rng.integers(1, 60))
        d = int(k + 1 + 10 ** rng.uniform(0, 5))
        thr = (k << 32) // d
        kappa = int(rng.integers(2, 300))
        i = int(rng.integers(1, kappa))
        c = i / kappa
        cw, sw = math.cos(c * 1.5707963267948966), math.sin(c * 1.5707963267948966)
        Tk, T2 = keep_threshold(L, thr, cw, sw), second_threshold(L, thr, cw, sw)
        assert Tk < T2
        tau = float(ndtri((thr + 0.5) / 2**32))
        for _ in range(60):
            n1 = float(rng.normal()) - (2.0 if rng.random() < 0.5 else 0.0)
            n2 = (tau - cw * n1) / sw + float(rng.normal()) * 10 ** rng.uniform(-6, -1) * (1 if rng.random() < 0.7 else -3)
            U1 = int(min(M32, max(0, ndtr(n1) * 2**32)))
            U2 = int(min(M32, max(0, ndtr(n2) * 2**32)))
            n = np.float64(cw) * np.float64(L.coopref_phi_inv_u32(U1)) + np.float64(sw) * np.float64(L.coopref_phi_inv_u32(U2))
            n_hat = np.float32(np.float32(cw) * approx_phi_inv_f32(U1)) + np.float32(np.float32(sw) * approx_phi_inv_f32(U2))
            checked += 1
            if n_hat <= Tk:
                certain += 1
                for nn in (float(n), float(np.nextafter(n, -np.inf)), float(np.nextafter(n, np.inf))):
                    assert L.coopref_phi_to_u32(nn) <= thr, (thr, c, U1, U2, float(n), float(n_hat), float(Tk))
            elif n_hat <= T2:
                band += 1
    assert certain > 3000 and band > 300 and checked > 20000
    # the band that still needs the exact blend is narrow: at k/d = 10/1400, c = 1/2, a few percent of the kept edges
    thr = (10 << 32) // 1400
    cw = sw = math.cos(math.pi / 4)
    lo, hi = float(keep_threshold(L, thr, cw, sw)), float(second_threshold(L, thr, cw, sw))
    assert (ndtr(hi) - ndtr(lo)) / ndtr(lo) < 0.06
