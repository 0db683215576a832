// Device-side scalar relaxations: k_L x + c_L <= f(x) <= k_U x + c_U on [l, u].
// These are the f(l, u) of the paper's "generalized elementwise multiplication" pattern (Sec. 4.1),
// with intercepts.  ReLU: two lower-bound designs selected by the range (Sec. 2.1), slope 1 when
// l >= 0 (Sec. 4.1).  tanh: tangent / chord lines between the concretized bounds (Sec. 4.1).
// The remaining functions (exp, reciprocal, sqrt, square) are needed by softmax, LayerNorm and GELU.
#pragma once
#include <hip/hip_runtime.h>

namespace tv {

struct Line2 { float kL, cL, kU, cU; };

constexpr float kTau = 1e-6f;          // relative width under which an interval counts as a point
constexpr float kExpCap = 0.99f;       // exp lower tangent at min(mid, l + 0.99): stays positive on [l, u]
constexpr float kRecipMin = 1e-12f;    // domain guard of the reciprocal

__device__ __forceinline__ bool is_point(float l, float u) {
  return (u - l) <= kTau * fmaxf(1.f, fmaxf(fabsf(l), fabsf(u)));
}

// slope f'(m) for both lines, intercepts min / max of f(x) - k x over {l, m, u}
__device__ __forceinline__ Line2 point_rule(float k, float fl, float fm, float fu, float l, float m, float u) {
  const float a = fl - k * l, b = fm - k * m, c = fu - k * u;
  Line2 r;
  r.kL = r.kU = k;
  r.cL = fminf(a, fminf(b, c));
  r.cU = fmaxf(a, fmaxf(b, c));
  return r;
}

__device__ __forceinline__ Line2 relax_relu(float l, float u) {
  Line2 r;
  if (l >= 0.f) { r.kL = r.kU = 1.f; r.cL = r.cU = 0.f; }
  else if (u <= 0.f) { r.kL = r.kU = 0.f; r.cL = r.cU = 0.f; }
  else {
    const float inv = 1.f / (u - l);
    r.kU = u * inv; r.cU = -l * u * inv;
    r.kL = (u >= -l) ? 1.f : 0.f; r.cL = 0.f;
  }
  return r;
}

__device__ __forceinline__ float dtanh(float x) { const float t = tanhf(x); return 1.f - t * t; }

// tangent point d in [lo, hi] whose tangent passes through (end, tanh end); returns the bracket end on
// the sound side (lower end for the lower line, upper end for the upper line)
__device__ __forceinline__ float tanh_tangent_through(float end, float lo, float hi, bool sound_lo) {
  const float te = tanhf(end);
  auto g = [&](float d) { const float t = tanhf(d); return t + (1.f - t * t) * (end - d) - te; };
  const bool neg_lo = g(lo) < 0.f;
  for (int it = 0; it < 32; ++it) {
    const float mid = 0.5f * (lo + hi);
    if ((g(mid) < 0.f) == neg_lo) lo = mid; else hi = mid;
  }
  return sound_lo ? lo : hi;
}

__device__ __forceinline__ Line2 relax_tanh(float l, float u) {
  const float m = 0.5f * (l + u);
  const float tl = tanhf(l), tu = tanhf(u), tm = tanhf(m);
  if (is_point(l, u)) return point_rule(1.f - tm * tm, tl, tm, tu, l, m, u);
  const float kap = (tu - tl) / (u - l);
  const float chord_c = tl - kap * l;
  Line2 r;
  if (l >= 0.f) {
    r.kL = kap; r.cL = chord_c; r.kU = 1.f - tm * tm; r.cU = tm - r.kU * m;
  } else if (u <= 0.f) {
    r.kU = kap; r.cU = chord_c; r.kL = 1.f - tm * tm; r.cL = tm - r.kL * m;
  } else {
    if (kap <= 1.f - tl * tl) { r.kL = kap; r.cL = chord_c; }
    else {
      const float d = tanh_tangent_through(u, l, 0.f, true);
      const float td = tanhf(d);
      r.kL = 1.f - td * td; r.cL = td - r.kL * d;
    }
    if (kap <= 1.f - tu * tu) { r.kU = kap; r.cU = chord_c; }
    else {
      const float d = tanh_tangent_through(l, 0.f, u, false);
      const float td = tanhf(d);
      r.kU = 1.f - td * td; r.cU = td - r.kU * d;
    }
  }
  return r;
}

__device__ __forceinline__ Line2 relax_exp(float l, float u) {
  const float m = 0.5f * (l + u);
  const float el = expf(l), eu = expf(u);
  if (is_point(l, u)) { const float em = expf(m); return point_rule(em, el, em, eu, l, m, u); }
  Line2 r;
  r.kU = (eu - el) / (u - l); r.cU = el - r.kU * l;
  const float d = fminf(m, l + kExpCap);
  r.kL = expf(d); r.cL = r.kL * (1.f - d);
  return r;
}

__device__ __forceinline__ Line2 relax_recip(float l, float u) {   // requires l > 0
  const float m = 0.5f * (l + u);
  if (is_point(l, u)) return point_rule(-1.f / (m * m), 1.f / l, 1.f / m, 1.f / u, l, m, u);
  Line2 r;
  r.kL = -1.f / (m * m); r.cL = 2.f / m;
  r.kU = -1.f / (l * u); r.cU = 1.f / l + 1.f / u;
  return r;
}

__device__ __forceinline__ Line2 relax_sqrt(float l, float u) {    // requires l > 0
  const float m = 0.5f * (l + u);
  const float sl = sqrtf(l), su = sqrtf(u), sm = sqrtf(m);
  if (is_point(l, u)) return point_rule(0.5f / sm, sl, sm, su, l, m, u);
  Line2 r;
  r.kU = 0.5f / sm; r.cU = 0.5f * sm;
  r.kL = 1.f / (sl + su); r.cL = sl * su / (sl + su);
  return r;
}

__device__ __forceinline__ Line2 relax_square(float l, float u) {
  const float m = 0.5f * (l + u);
  if (is_point(l, u)) return point_rule(2.f * m, l * l, m * m, u * u, l, m, u);
  Line2 r;
  r.kL = 2.f * m; r.cL = -m * m;
  r.kU = l + u; r.cU = -l * u;
  return r;
}

// ---- linear forms relative to a base neuron x with bound lines (x_L, x_U):
//   lower = pL * x_L + qL * x_U + cL   (pL >= 0 >= qL),   upper = pU * x_U + qU * x_L + cU   (pU >= 0 >= qU)
struct Form { float pL, qL, cL, pU, qU, cU; };

__device__ __forceinline__ Form form_identity() { return Form{1.f, 0.f, 0.f, 1.f, 0.f, 0.f}; }

// z with k_L y + c_L <= z <= k_U y + c_U: each line takes y's own side for a non-negative slope, the
// other side for a negative one (sign rule of Eq. (2) applied to a per-neuron scalar)
__device__ __forceinline__ Form form_sub(const Form &y, float kL, float cL, float kU, float cU) {
  Form z;
  if (kL >= 0.f) { z.pL = kL * y.pL; z.qL = kL * y.qL; z.cL = kL * y.cL + cL; }
  else           { z.pL = kL * y.qU; z.qL = kL * y.pU; z.cL = kL * y.cU + cL; }
  if (kU >= 0.f) { z.pU = kU * y.pU; z.qU = kU * y.qU; z.cU = kU * y.cU + cU; }
  else           { z.pU = kU * y.qL; z.qU = kU * y.pL; z.cU = kU * y.cL + cU; }
  return z;
}

__device__ __forceinline__ Form form_add(const Form &a, const Form &b) {
  return Form{a.pL + b.pL, a.qL + b.qL, a.cL + b.cL, a.pU + b.pU, a.qU + b.qU, a.cU + b.cU};
}

// z = x * y (both relative to the same base), McCormick planes
//   z >= ly x + lx y - lx ly ,   z <= uy x + lx y - lx uy
__device__ __forceinline__ Form form_mul(const Form &x, const Form &y, float lx, float ly, float uy) {
  const Form ax = form_sub(x, ly, 0.f, uy, 0.f);
  const Form by = form_sub(y, lx, 0.f, lx, 0.f);
  Form z = form_add(ax, by);
  z.cL -= lx * ly;
  z.cU -= lx * uy;
  return z;
}

// concretized bounds of z = relaxation of y on [ly, uy] (single-input chain: the norm of z's
// coefficients is |k| times the norm of one side of y)
__device__ __forceinline__ void line_range(float kL, float cL, float kU, float cU, float ly, float uy, float &lz,
                                           float &uz) {
  lz = (kL >= 0.f ? kL * ly : kL * uy) + cL;
  uz = (kU >= 0.f ? kU * uy : kU * ly) + cU;
}

// centre/radius map of a form:  S_y = sS*S + sR*R + sC [bias row],  R_y = rS*S + rR*R + rC [bias row]
struct Map2 { float sS, sR, sC, rS, rR, rC; };
__device__ __forceinline__ Map2 form_map(const Form &f) {
  Map2 m;
  m.sS = 0.5f * (f.pL + f.qL + f.pU + f.qU);
  m.sR = 0.5f * (-f.pL + f.qL + f.pU - f.qU);
  m.sC = 0.5f * (f.cL + f.cU);
  m.rS = 0.5f * (f.pU + f.qU - f.pL - f.qL);
  m.rR = 0.5f * (f.pU - f.qU + f.pL - f.qL);
  m.rC = 0.5f * (f.cU - f.cL);
  return m;
}

}  // namespace tv
