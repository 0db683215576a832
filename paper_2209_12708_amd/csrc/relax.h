// Device-side scalar relaxations: k_L x + c_L <= f(x) <= k_U x + c_U on [l, u].
// These are the f(l, u) of the paper's "generalized elementwise multiplication" pattern (Sec. 4.1),
// with intercepts.  ReLU: two lower-bound designs selected by the range (Sec. 2.1), slope 1 when
// l >= 0 (Sec. 4.1).  tanh: tangent / chord lines between the concretized bounds (Sec. 4.1).
// The remaining functions (exp, reciprocal, sqrt, square) are needed by softmax, LayerNorm and GELU.
//
// Precision.  This is per-neuron work (1/C of the traffic), done in double: the radius plane of an
// output state is driven by differences such as (k_U - k_L)/2 and (u - l)/2, which are far below the
// fp32 resolution of k or of l, u themselves when an interval is narrow.  Intervals therefore enter
// as (mid, half), both accurate in fp32, and the lines leave as centre/radius map coefficients that
// are rounded to fp32 only at the end; the per-coefficient streaming arithmetic stays in fp32.
#pragma once
#include <hip/hip_runtime.h>

// The scalar algebra below relies on identical inputs giving bit-identical outputs for the lower and
// the upper line (a point interval must produce exactly coinciding lines, hence an exactly zero radius).
// Fused multiply-add contraction breaks that: after inlining, one of two equal products may be fused
// into a following sum and the other not.  Every function here therefore switches contraction off.
#define TV_NO_CONTRACT _Pragma("clang fp contract(off)")

namespace tv {

struct Line2 { double kL, cL, kU, cU; };

constexpr double kTau = 1e-12;         // relative width under which an interval counts as a point
constexpr double kExpCap = 0.99;       // exp lower tangent at min(mid, l + 0.99): stays positive on [l, u]
constexpr double kRecipMin = 1e-12;    // domain guard of the reciprocal

__device__ __forceinline__ bool is_point(double l, double u) {
  TV_NO_CONTRACT
  return (u - l) <= kTau * fmax(1.0, fmax(fabs(l), fabs(u)));
}

// slope f'(m) for both lines, intercepts min / max of f(x) - k x over {l, m, u}
__device__ __forceinline__ Line2 point_rule(double k, double fl, double fm, double fu, double l, double m, double u) {
  TV_NO_CONTRACT
  const double a = fl - k * l, b = fm - k * m, c = fu - k * u;
  Line2 r;
  r.kL = r.kU = k;
  r.cL = fmin(a, fmin(b, c));
  r.cU = fmax(a, fmax(b, c));
  return r;
}

__device__ __forceinline__ Line2 relax_relu(double l, double u) {
  TV_NO_CONTRACT
  Line2 r;
  if (l >= 0.0) { r.kL = r.kU = 1.0; r.cL = r.cU = 0.0; }
  else if (u <= 0.0) { r.kL = r.kU = 0.0; r.cL = r.cU = 0.0; }
  else {
    const double inv = 1.0 / (u - l);
    r.kU = u * inv; r.cU = -l * u * inv;
    r.kL = (u >= -l) ? 1.0 : 0.0; r.cL = 0.0;
  }
  return r;
}

// Leaky ReLU x (x >= 0), a x (x < 0) with 0 <= a <= 1, convex: the design of ReLU with the line a x in place of 0
// (upper = chord through (l, a l), (u, u); lower = the steeper or the flatter branch, whichever end is farther).
__device__ __forceinline__ Line2 relax_leaky_relu(double l, double u, double a) {
  TV_NO_CONTRACT
  Line2 r;
  if (l >= 0.0) { r.kL = r.kU = 1.0; r.cL = r.cU = 0.0; }
  else if (u <= 0.0) { r.kL = r.kU = a; r.cL = r.cU = 0.0; }
  else {
    const double den = u - l;
    r.kU = (u - a * l) / den; r.cU = (a - 1.0) * l * u / den;
    r.kL = (u >= -l) ? 1.0 : a; r.cL = 0.0;
  }
  return r;
}

// tangent point d in [lo, hi] whose tangent passes through (end, tanh end): the root of
//   g(d) = tanh d + (1 - tanh^2 d)(end - d) - tanh end,      g'(d) = -2 tanh d (1 - tanh^2 d)(end - d),
// which changes sign once on the bracket.  Returned on the sound side of the root (towards lo for the lower line,
// towards hi for the upper line), as a plain bisection would return its bracket end.  Newton steps kept inside the
// bracket (a bisection step otherwise) reach the root in a handful of tanh evaluations instead of two per halving;
// the sound side is then taken as the nearest probe next to the root whose sign of g says it is on that side.
__device__ __forceinline__ double tanh_tangent_through(double end, double lo, double hi, bool sound_lo) {
  TV_NO_CONTRACT
  const double te = tanh(end);
  const double lo0 = lo, hi0 = hi;
  const double scale = fmax(hi0 - lo0, 1e-300);
  double t = tanh(lo);
  const bool neg_lo = t + (1.0 - t * t) * (end - lo) - te < 0.0;
  // to leading order g(d) = (end - d)^2 (end + 2 d) / 3: the root of a short interval is near -end / 2
  double d = 0.5 * (lo + hi);
  if (fabs(end) < 0.5 && -0.5 * end > lo && -0.5 * end < hi) d = -0.5 * end;
  for (int it = 0; it < 64; ++it) {       // far from the root the steps are bisections; near it, Newton's
    t = tanh(d);
    const double s = 1.0 - t * t;
    const double gd = t + s * (end - d) - te;
    // below the rounding noise of its own terms g says nothing more about the root (intervals under ~1e-5,
    // where the candidate lines differ by less than 1e-10 in slope)
    if (fabs(gd) <= 4.5e-16 * (fabs(t) + fabs(te) + s * fabs(end - d))) break;
    if ((gd < 0.0) == neg_lo) lo = d; else hi = d;
    const double dg = -2.0 * t * s * (end - d);
    double dn = d - gd / dg;
    if (!(dn > lo && dn < hi)) dn = 0.5 * (lo + hi);
    const bool done = fabs(dn - d) <= 1.0e-13 * scale + 4.0e-16 * fmax(1.0, fabs(d));
    d = dn;
    if (done) break;
  }
  // step off the root towards the sound side until g confirms the side
  double step = 1.5e-14 * scale;
  for (int k = 0; k < 12; ++k, step *= 16.0) {   // up to 0.26 of the bracket: past any noise band of g around the root
    const double c = sound_lo ? fmax(d - step, lo0) : fmin(d + step, hi0);
    t = tanh(c);
    const bool neg = t + (1.0 - t * t) * (end - c) - te < 0.0;
    if ((neg == neg_lo) == sound_lo) return c;
  }
  return sound_lo ? lo : hi;                // the bracket keeps g's sign at both ends: sound, if not as close
}

__device__ __forceinline__ Line2 relax_tanh(double l, double u) {
  TV_NO_CONTRACT
  const double m = 0.5 * (l + u);
  const double tl = tanh(l), tu = tanh(u), tm = tanh(m);
  if (is_point(l, u)) return point_rule(1.0 - tm * tm, tl, tm, tu, l, m, u);
  const double kap = (tu - tl) / (u - l);
  const double chord_c = tl - kap * l;
  Line2 r;
  if (l >= 0.0) {
    r.kL = kap; r.cL = chord_c; r.kU = 1.0 - tm * tm; r.cU = tm - r.kU * m;
  } else if (u <= 0.0) {
    r.kU = kap; r.cU = chord_c; r.kL = 1.0 - tm * tm; r.cL = tm - r.kL * m;
  } else {
    if (kap <= 1.0 - tl * tl) { r.kL = kap; r.cL = chord_c; }
    else {
      const double d = tanh_tangent_through(u, l, 0.0, true);
      const double td = tanh(d);
      r.kL = 1.0 - td * td; r.cL = td - r.kL * d;
    }
    if (kap <= 1.0 - tu * tu) { r.kU = kap; r.cU = chord_c; }
    else {
      const double d = tanh_tangent_through(l, 0.0, u, false);
      const double td = tanh(d);
      r.kU = 1.0 - td * td; r.cU = td - r.kU * d;
    }
  }
  return r;
}

__device__ __forceinline__ Line2 relax_exp(double l, double u) {
  TV_NO_CONTRACT
  const double m = 0.5 * (l + u);
  const double el = exp(l), eu = exp(u);
  if (is_point(l, u)) { const double em = exp(m); return point_rule(em, el, em, eu, l, m, u); }
  Line2 r;
  r.kU = (eu - el) / (u - l); r.cU = el - r.kU * l;
  const double d = fmin(m, l + kExpCap);
  r.kL = exp(d); r.cL = r.kL * (1.0 - d);
  return r;
}

__device__ __forceinline__ Line2 relax_recip(double l, double u) {   // requires l > 0
  TV_NO_CONTRACT
  const double m = 0.5 * (l + u);
  if (is_point(l, u)) return point_rule(-1.0 / (m * m), 1.0 / l, 1.0 / m, 1.0 / u, l, m, u);
  Line2 r;
  r.kL = -1.0 / (m * m); r.cL = 2.0 / m;
  r.kU = -1.0 / (l * u); r.cU = 1.0 / l + 1.0 / u;
  return r;
}

__device__ __forceinline__ Line2 relax_sqrt(double l, double u) {    // requires l > 0
  TV_NO_CONTRACT
  const double m = 0.5 * (l + u);
  const double sl = sqrt(l), su = sqrt(u), sm = sqrt(m);
  if (is_point(l, u)) return point_rule(0.5 / sm, sl, sm, su, l, m, u);
  Line2 r;
  r.kU = 0.5 / sm; r.cU = 0.5 * sm;
  r.kL = 1.0 / (sl + su); r.cL = sl * su / (sl + su);
  return r;
}

__device__ __forceinline__ Line2 relax_square(double l, double u) {
  TV_NO_CONTRACT
  const double m = 0.5 * (l + u);
  if (is_point(l, u)) return point_rule(2.0 * m, l * l, m * m, u * u, l, m, u);
  Line2 r;
  r.kL = 2.0 * m; r.cL = -m * m;
  r.kU = l + u; r.cU = -l * u;
  return r;
}

// ---- linear forms relative to a base neuron x with bound lines (x_L, x_U):
//   lower = pL * x_L + qL * x_U + cL   (pL >= 0 >= qL),   upper = pU * x_U + qU * x_L + cU   (pU >= 0 >= qU)
struct Form { double pL, qL, cL, pU, qU, cU; };

__device__ __forceinline__ Form form_identity() { return Form{1.0, 0.0, 0.0, 1.0, 0.0, 0.0}; }

// z with k_L y + c_L <= z <= k_U y + c_U: each line takes y's own side for a non-negative slope, the
// other side for a negative one (sign rule of Eq. (2) applied to a per-neuron scalar)
__device__ __forceinline__ Form form_sub(const Form &y, double kL, double cL, double kU, double cU) {
  TV_NO_CONTRACT
  Form z;
  if (kL >= 0.0) { z.pL = kL * y.pL; z.qL = kL * y.qL; z.cL = kL * y.cL + cL; }
  else           { z.pL = kL * y.qU; z.qL = kL * y.pU; z.cL = kL * y.cU + cL; }
  if (kU >= 0.0) { z.pU = kU * y.pU; z.qU = kU * y.qU; z.cU = kU * y.cU + cU; }
  else           { z.pU = kU * y.qL; z.qU = kU * y.pL; z.cU = kU * y.cL + cU; }
  return z;
}
__device__ __forceinline__ Form form_sub(const Form &y, const Line2 &ln) { return form_sub(y, ln.kL, ln.cL, ln.kU, ln.cU); }

__device__ __forceinline__ Form form_add(const Form &a, const Form &b) {
  TV_NO_CONTRACT
  return Form{a.pL + b.pL, a.qL + b.qL, a.cL + b.cL, a.pU + b.pU, a.qU + b.qU, a.cU + b.cU};
}

// z = x * y (both relative to the same base), McCormick planes
//   z >= ly x + lx y - lx ly ,   z <= uy x + lx y - lx uy
__device__ __forceinline__ Form form_mul(const Form &x, const Form &y, double lx, double ly, double uy) {
  TV_NO_CONTRACT
  const Form ax = form_sub(x, ly, 0.0, uy, 0.0);
  const Form by = form_sub(y, lx, 0.0, lx, 0.0);
  Form z = form_add(ax, by);
  z.cL -= lx * ly;
  z.cU -= lx * uy;
  return z;
}

// concretized bounds of z = relaxation of y on [ly, uy] (single-input chain: the norm of z's
// coefficients is |k| times the norm of one side of y)
__device__ __forceinline__ void line_range(const Line2 &ln, double ly, double uy, double &lz, double &uz) {
  TV_NO_CONTRACT
  lz = (ln.kL >= 0.0 ? ln.kL * ly : ln.kL * uy) + ln.cL;
  uz = (ln.kU >= 0.0 ? ln.kU * uy : ln.kU * ly) + ln.cU;
}

// SiLU x sigmoid(x) with sigmoid(x) = 0.5 (1 + tanh(x / 2)) as a chain on one neuron: x / 2 -> tanh -> 0.5 t + 0.5 ->
// product with x.  Every link is a function of x alone, so the chain is one form in x.
__device__ __forceinline__ Form silu_form(double l, double u) {
  TV_NO_CONTRACT
  const double lh = 0.5 * l, uh = 0.5 * u;
  const Line2 th = relax_tanh(lh, uh);
  double lt, ut;
  line_range(th, lh, uh, lt, ut);
  const Form half = form_sub(form_identity(), 0.5, 0.0, 0.5, 0.0);
  const Form sg = form_sub(form_sub(half, th), 0.5, 0.5, 0.5, 0.5);
  return form_mul(form_identity(), sg, l, 0.5 * lt + 0.5, 0.5 * ut + 0.5);
}

// centre/radius map of a form:  S_y = sS*S + sR*R + sC [bias row],  R_y = rS*S + rR*R + rC [bias row].
// The differences are taken in double; the fp32 copies serve the coefficient rows, the double ones the
// bias row.
struct Map2 {
  float sS, sR, rS, rR;
  double sSd, sRd, sCd, rSd, rRd, rCd;
};
__device__ __forceinline__ Map2 form_map(const Form &f) {
  TV_NO_CONTRACT
  Map2 m;
  m.sSd = 0.5 * (f.pL + f.qL + f.pU + f.qU);
  m.sRd = 0.5 * (-f.pL + f.qL + f.pU - f.qU);
  m.sCd = 0.5 * (f.cL + f.cU);
  // differences of corresponding members first: coinciding lines give exactly zero
  m.rSd = 0.5 * ((f.pU - f.pL) + (f.qU - f.qL));
  m.rRd = 0.5 * ((f.pU + f.pL) - (f.qU + f.qL));
  m.rCd = 0.5 * (f.cU - f.cL);
  m.sS = (float)m.sSd; m.sR = (float)m.sRd; m.rS = (float)m.rSd; m.rR = (float)m.rRd;
  return m;
}

// product z = x * y with x a state (S_x, R_x) and y a state (S_y, R_y), in centre/radius form:
//   S_z = a1 S_x + a2 R_x + b S_y - b a1 [bias],   R_z = a3 S_x + a4 R_x + |b| R_y - b a3 [bias]
// with the multiplier range [ly, uy] of y and b = lx.  On the bias row a3 S_x - b a3 = a3 (S_x - lx) is
// formed from the slack S_x - lx = R_x + eps N(lower line of x), which has no cancellation.
struct Mul2 {
  float a1, a2, a3, a4;
  double a1d, a2d, a3d, a4d;
};
__device__ __forceinline__ Mul2 mul_coeffs(double ly, double uy) {
  TV_NO_CONTRACT
  Mul2 m;
  m.a1d = 0.5 * (ly + uy);
  m.a2d = 0.5 * (fabs(uy) - fabs(ly));
  m.a3d = 0.5 * (uy - ly);
  m.a4d = 0.5 * (fabs(uy) + fabs(ly));
  m.a1 = (float)m.a1d; m.a2 = (float)m.a2d; m.a3 = (float)m.a3d; m.a4 = (float)m.a4d;
  return m;
}

}  // namespace tv
