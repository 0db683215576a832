// Memory-bound kernels over bound states [rows][C][n]: concretization (Eq. (1)), fused activation
// relaxation, LayerNorm and softmax bounds.
//
// Common geometry.  A workgroup (256 threads) owns one row block (one token, or one attention row)
// and a chunk of its columns.  Lanes lie along the contiguous neuron axis (each lane owns VEC float4
// column groups), G lanes cover the chunk, and the 256/G "row slots" stride over the C coefficient
// rows.  The norm of Eq. (1) is a reduction down the coefficient axis: lane-private accumulation
// over the rows of a slot, then one butterfly across the slots of a wave and one LDS exchange
// across the 4 waves - the paper's hybrid reduction (Sec. 4.2: k lane-private steps + one shuffle
// tree), turned by 90 degrees because here the reduced axis is the strided one, and widened to
// 64-lane wavefronts.  Sums along the neuron axis (softmax row sums, LayerNorm means) are butterflies
// over the G lanes of a slot.  As in the paper's sharing-oriented scheduling (Sec. 4.3) the
// concretized bounds never go to memory: the same workgroup that reduces a neuron's coefficients
// rescales them.
#include <float.h>
#include "common.h"
#include "relax.h"

namespace tv {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxVec = 4;

struct Geo {
  int G;      // lanes per row (power of two, <= 64)
  int NS;     // row slots per workgroup = 256 / G
  int slot;   // this thread's row slot
  int g;      // this thread's lane within the row
  int n4;     // float4 groups in the chunk
  __device__ Geo(int G_, int n4_) : G(G_), NS(kThreads / G_), slot(threadIdx.x / G_), g(threadIdx.x % G_), n4(n4_) {}
};

__device__ __forceinline__ float norm_acc(float a, float x, int pn) {
  return pn == TV_NORM_INF ? a + fabsf(x) : (pn == 2 ? fmaf(x, x, a) : fmaxf(a, fabsf(x)));
}
__device__ __forceinline__ float norm_comb(float a, float b, int pn) { return pn == 1 ? fmaxf(a, b) : a + b; }
__device__ __forceinline__ float norm_fin(float a, int pn) { return pn == 2 ? sqrtf(a) : a; }
__device__ __forceinline__ bool finite_f(float x) { return fabsf(x) <= FLT_MAX; }

// Combine CNT per-lane partials across the row slots; afterwards every thread holds the totals of its
// own columns.  red: LDS [4][64][CNT].  `mx`: combine with max instead of +.
template <int CNT>
__device__ __forceinline__ void slot_reduce(float (&x)[CNT], const Geo &ge, bool mx, float *red) {
  for (int off = ge.G; off < kWave; off <<= 1) {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
      const float o = __shfl_xor(x[i], off);
      x[i] = mx ? fmaxf(x[i], o) : x[i] + o;
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();   // red may still be read from a previous call
  if (lane < ge.G) {
#pragma unroll
    for (int i = 0; i < CNT; ++i) red[(wave * kWave + lane) * CNT + i] = x[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < CNT; ++i) {
    float t = red[(0 * kWave + ge.g) * CNT + i];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float o = red[(w * kWave + ge.g) * CNT + i];
      t = mx ? fmaxf(t, o) : t + o;
    }
    x[i] = t;
  }
}

// Sum (or max) of one value over the G lanes of a row slot (lanes of a slot are consecutive).
__device__ __forceinline__ float row_sum(float x, int G) {
  for (int off = 1; off < G; off <<= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ __forceinline__ float row_max(float x, int G) {
  for (int off = 1; off < G; off <<= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
// Sum over the whole workgroup of one value held per row slot (same value on the G lanes of a slot).
__device__ __forceinline__ float block_sum_slots(float x, const Geo &ge, bool mx, float *red) {
  float v[1] = {x};
  slot_reduce<1>(v, ge, mx, red);
  return v[0];
}
// Max over all columns of the chunk of a per-column value that every slot holds identically.
__device__ __forceinline__ float cols_max(float x, int G) { return row_max(x, G); }

// n here is the row stride in floats (the row length when densely packed)
__device__ __forceinline__ const float4 *row_ptr(const float *base, long row, int C, int r, int n, int c0) {
  return reinterpret_cast<const float4 *>(base + ((row * C + r) * (long)n + c0));
}
__device__ __forceinline__ float4 *row_ptr(float *base, long row, int C, int r, int n, int c0) {
  return reinterpret_cast<float4 *>(base + ((row * C + r) * (long)n + c0));
}

#define F4(v, c) (reinterpret_cast<float *>(&(v))[c])
#define CF4(v, c) (reinterpret_cast<const float *>(&(v))[c])

// ------------------------------------------------------------------------------------------------
// Norms of two linear forms of the state down the coefficient axis, for this thread's columns:
//   NL = N(pL * lo + qL * up),  NU = N(pU * up + qU * lo),   lo = S - R, up = S + R,
// N = sum over the P blocks of the dual norm.  forms == nullptr means the state itself (pL = pU = 1).
// Also returns the bias-row values of lo / up mapped the same way (without the forms' constants).
template <int VEC>
__device__ __forceinline__ void column_norms(const float *S, const float *R, long row, int P, int E, int n, int c0,
                                             const Geo &ge, int pn, const Form *forms, float *red,
                                             float (&NL)[4 * VEC], float (&NU)[4 * VEC], float (&bL)[4 * VEC],
                                             float (&bU)[4 * VEC]) {
  const int C = P * E + 1;
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) NL[i] = NU[i] = 0.f;
  for (int pb = 0; pb < P; ++pb) {
    float acc[8 * VEC];
#pragma unroll
    for (int i = 0; i < 8 * VEC; ++i) acc[i] = 0.f;
    const int r1 = (pb + 1) * E;
#pragma unroll 4
    for (int r = pb * E + ge.slot; r < r1; r += ge.NS) {
      const float4 *ps = row_ptr(S, row, C, r, n, c0), *pr = row_ptr(R, row, C, r, n, c0);
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const int f = ge.g + ge.G * v;
        if (f < ge.n4) {
          const float4 s = ps[f], rr = pr[f];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float lo = CF4(s, c) - CF4(rr, c), up = CF4(s, c) + CF4(rr, c);
            float a = lo, b = up;
            if (forms) {
              const Form &fm = forms[4 * v + c];
              a = fm.pL * lo + fm.qL * up;
              b = fm.pU * up + fm.qU * lo;
            }
            acc[8 * v + c] = norm_acc(acc[8 * v + c], a, pn);
            acc[8 * v + 4 + c] = norm_acc(acc[8 * v + 4 + c], b, pn);
          }
        }
      }
    }
    slot_reduce<8 * VEC>(acc, ge, pn == 1, red);
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        NL[4 * v + c] += norm_fin(acc[8 * v + c], pn);
        NU[4 * v + c] += norm_fin(acc[8 * v + 4 + c], pn);
      }
  }
  const float4 *ps = row_ptr(S, row, C, C - 1, n, c0), *pr = row_ptr(R, row, C, C - 1, n, c0);
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    const int f = ge.g + ge.G * v;
    float4 s = make_float4(0, 0, 0, 0), rr = s;
    if (f < ge.n4) { s = ps[f]; rr = pr[f]; }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float lo = CF4(s, c) - CF4(rr, c), up = CF4(s, c) + CF4(rr, c);
      float a = lo, b = up;
      if (forms) {
        const Form &fm = forms[4 * v + c];
        a = fm.pL * lo + fm.qL * up;
        b = fm.pU * up + fm.qU * lo;
      }
      bL[4 * v + c] = a; bU[4 * v + c] = b;
    }
  }
}

// Write y = map(x) for every row of the block (bias constants on the last row).
template <int VEC>
__device__ __forceinline__ void apply_maps(const float *S, const float *R, float *So, float *Ro, long row, int C,
                                           int n, int c0, const Geo &ge, const Map2 *maps) {
#pragma unroll 4
  for (int r = ge.slot; r < C; r += ge.NS) {
    const float4 *ps = row_ptr(S, row, C, r, n, c0), *pr = row_ptr(R, row, C, r, n, c0);
    float4 *qs = row_ptr(So, row, C, r, n, c0), *qr = row_ptr(Ro, row, C, r, n, c0);
    const bool last = r == C - 1;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      if (f < ge.n4) {
        const float4 s = ps[f], rr = pr[f];
        float4 os, orr;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const Map2 &m = maps[4 * v + c];
          float a = m.sS * CF4(s, c) + m.sR * CF4(rr, c);
          float b = m.rS * CF4(s, c) + m.rR * CF4(rr, c);
          if (last) { a += m.sC; b += m.rC; }
          F4(os, c) = a; F4(orr, c) = b;
        }
        qs[f] = os; qr[f] = orr;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Eq. (1).  grid = (rows, column chunks).
template <int VEC>
__global__ __launch_bounds__(kThreads) void concretize_kernel(const float *S, const float *R, int P, int E, int n,
                                                              int ld, int G, int rps, int pn, const float *eps,
                                                              float *l, float *u) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int chunk = 4 * G * VEC, c0 = blockIdx.y * chunk;
  const Geo ge(G, min(chunk, n - c0) / 4);
  float NL[4 * VEC], NU[4 * VEC], bL[4 * VEC], bU[4 * VEC];
  column_norms<VEC>(S, R, row, P, E, ld, c0, ge, pn, nullptr, red, NL, NU, bL, bU);
  if (ge.slot == 0) {
    const float e = eps[row / rps];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      if (f < ge.n4) {
        float4 lo, up;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          F4(lo, c) = bL[4 * v + c] - e * NL[4 * v + c];
          F4(up, c) = bU[4 * v + c] + e * NU[4 * v + c];
        }
        reinterpret_cast<float4 *>(l + row * n + c0)[f] = lo;
        reinterpret_cast<float4 *>(u + row * n + c0)[f] = up;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Activation: concretize, relax, substitute - one workgroup reads its coefficients for the norm and
// again (from cache) for the rescale.  GELU adds one mapped-norm pass for the inner product.
__device__ __forceinline__ Form gelu_inner(float lx, float ux, float &lb, float &ub) {
  // a = x^2 ; b = k (1 + c3 a) ; returns the form of b and its range
  const float k = 0.7978845608028654f, c3 = 0.044715f;
  const Line2 sq = relax_square(lx, ux);
  Form a = form_sub(form_identity(), sq.kL, sq.cL, sq.kU, sq.cU);
  float la, ua;
  line_range(sq.kL, sq.cL, sq.kU, sq.cU, lx, ux, la, ua);
  lb = k * c3 * la + k; ub = k * c3 * ua + k;
  return form_sub(a, k * c3, k, k * c3, k);
}

template <int VEC, int ACT>
__global__ __launch_bounds__(kThreads) void activation_kernel(const float *S, const float *R, int P, int E, int n,
                                                              int G, int rps, int pn, const float *eps,
                                                              float *So, float *Ro, int32_t *status) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int C = P * E + 1;
  const int chunk = 4 * G * VEC, c0 = blockIdx.y * chunk;
  const Geo ge(G, min(chunk, n - c0) / 4);
  const float e = eps[row / rps];
  float NL[4 * VEC], NU[4 * VEC], bL[4 * VEC], bU[4 * VEC];
  column_norms<VEC>(S, R, row, P, E, n, c0, ge, pn, nullptr, red, NL, NU, bL, bU);
  Map2 maps[4 * VEC];
  bool bad = false;
  if (ACT != TV_ACT_GELU) {
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      const float l = bL[i] - e * NL[i], u = bU[i] + e * NU[i];
      bad |= !(finite_f(l) && finite_f(u));
      const Line2 ln = ACT == TV_ACT_RELU ? relax_relu(l, u) : relax_tanh(l, u);
      maps[i] = form_map(form_sub(form_identity(), ln.kL, ln.cL, ln.kU, ln.cU));
    }
  } else {
    Form fg[4 * VEC];
    float lx[4 * VEC], ux[4 * VEC];
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      lx[i] = bL[i] - e * NL[i]; ux[i] = bU[i] + e * NU[i];
      bad |= !(finite_f(lx[i]) && finite_f(ux[i]));
      float lb, ub;
      const Form b = gelu_inner(lx[i], ux[i], lb, ub);
      fg[i] = form_mul(form_identity(), b, lx[i], lb, ub);     // g = x * b
    }
    column_norms<VEC>(S, R, row, P, E, n, c0, ge, pn, fg, red, NL, NU, bL, bU);
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      const float lg = bL[i] + fg[i].cL - e * NL[i], ug = bU[i] + fg[i].cU + e * NU[i];
      bad |= !(finite_f(lg) && finite_f(ug));
      const Line2 th = relax_tanh(lg, ug);
      float lt, ut;
      line_range(th.kL, th.cL, th.kU, th.cU, lg, ug, lt, ut);
      Form h = form_sub(form_sub(fg[i], th.kL, th.cL, th.kU, th.cU), 0.5f, 0.5f, 0.5f, 0.5f);
      maps[i] = form_map(form_mul(form_identity(), h, lx[i], 0.5f * lt + 0.5f, 0.5f * ut + 0.5f));
    }
  }
  if (bad) status[row / rps] = 1;
  apply_maps<VEC>(S, R, So, Ro, row, C, n, c0, ge, maps);
}

// ------------------------------------------------------------------------------------------------
// LayerNorm bound.  One workgroup per token; lanes cover all n columns (VEC float4 per lane).
//   c = x - mean(x)                 one affine map (I - 11^T/n): S_c = S - mean S, R_c = (1-2/n) R + mean R
//   q = c^2 (relaxed) ; v = mean q + ln_eps ; s = sqrt v ; rho = 1/s ; y = c * rho ; out = gamma y + beta
// Three sweeps over the block: norms of c; norm of v; output.
template <int VEC>
struct LnRow {
  float sc[4 * VEC], rc[4 * VEC];   // centred centre / radius planes of one coefficient row
};

template <int VEC>
__device__ __forceinline__ void ln_load_row(const float *S, const float *R, long row, int C, int r, int n,
                                            const Geo &ge, LnRow<VEC> &o) {
  const float4 *ps = row_ptr(S, row, C, r, n, 0), *pr = row_ptr(R, row, C, r, n, 0);
  float ss = 0.f, sr = 0.f;
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    const int f = ge.g + ge.G * v;
    float4 s = make_float4(0, 0, 0, 0), rr = s;
    if (f < ge.n4) { s = ps[f]; rr = pr[f]; }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      o.sc[4 * v + c] = CF4(s, c); o.rc[4 * v + c] = CF4(rr, c);
      ss += CF4(s, c); sr += CF4(rr, c);
    }
  }
  const float inv = 1.f / (float)n;
  const float ms = row_sum(ss, ge.G) * inv, mr = row_sum(sr, ge.G) * inv;
  const float w = 1.f - 2.f * inv;
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) {
    o.sc[i] = o.sc[i] - ms;
    o.rc[i] = w * o.rc[i] + mr;
  }
}

template <int VEC>
__global__ __launch_bounds__(kThreads) void layernorm_kernel(const float *S, const float *R, int P, int E, int n,
                                                             int G, int rps, int pn, const float *eps,
                                                             const float *gamma, const float *beta, float ln_eps,
                                                             float *So, float *Ro, int32_t *status) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int C = P * E + 1;
  const Geo ge(G, n / 4);
  const float e = eps[row / rps];
  const float inv = 1.f / (float)n;
  bool colon[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) colon[v] = ge.g + ge.G * v < ge.n4;
  bool bad = false;

  // ---- sweep 1: concretize c
  float lc[4 * VEC], uc[4 * VEC];
  {
    float NL[4 * VEC], NU[4 * VEC];
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) NL[i] = NU[i] = 0.f;
    for (int pb = 0; pb < P; ++pb) {
      float acc[8 * VEC];
#pragma unroll
      for (int i = 0; i < 8 * VEC; ++i) acc[i] = 0.f;
      for (int r = pb * E + ge.slot; r < (pb + 1) * E; r += ge.NS) {
        LnRow<VEC> x;
        ln_load_row<VEC>(S, R, row, C, r, n, ge, x);
#pragma unroll
        for (int i = 0; i < 4 * VEC; ++i) {
          acc[2 * i] = norm_acc(acc[2 * i], x.sc[i] - x.rc[i], pn);
          acc[2 * i + 1] = norm_acc(acc[2 * i + 1], x.sc[i] + x.rc[i], pn);
        }
      }
      slot_reduce<8 * VEC>(acc, ge, pn == 1, red);
#pragma unroll
      for (int i = 0; i < 4 * VEC; ++i) {
        NL[i] += norm_fin(acc[2 * i], pn);
        NU[i] += norm_fin(acc[2 * i + 1], pn);
      }
    }
    LnRow<VEC> x;
    ln_load_row<VEC>(S, R, row, C, C - 1, n, ge, x);
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      lc[i] = (x.sc[i] - x.rc[i]) - e * NL[i];
      uc[i] = (x.sc[i] + x.rc[i]) + e * NU[i];
      if (colon[i / 4]) bad |= !(finite_f(lc[i]) && finite_f(uc[i]));
    }
  }
  // square relaxation per column: q_L = kL c_(L|U) + cL etc.  (forms relative to c)
  Form fq[4 * VEC];
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) {
    const Line2 sq = relax_square(lc[i], uc[i]);
    fq[i] = form_sub(form_identity(), sq.kL, sq.cL, sq.kU, sq.cU);
    if (!colon[i / 4]) fq[i] = Form{0, 0, 0, 0, 0, 0};
  }
  // v_L[r] = mean_d (pL c_L + qL c_U)[r, d],  v_U[r] = mean_d (pU c_U + qU c_L)[r, d]
  auto v_row = [&](const LnRow<VEC> &x, float &vl, float &vu) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      const float lo = x.sc[i] - x.rc[i], up = x.sc[i] + x.rc[i];
      a += fq[i].pL * lo + fq[i].qL * up;
      b += fq[i].pU * up + fq[i].qU * lo;
    }
    vl = row_sum(a, ge.G) * inv;
    vu = row_sum(b, ge.G) * inv;
  };
  float cql = 0.f, cqu = 0.f;   // mean of the square relaxation's intercepts
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) { cql += fq[i].cL; cqu += fq[i].cU; }
  cql = row_sum(cql, ge.G) * inv; cqu = row_sum(cqu, ge.G) * inv;

  // ---- sweep 2: concretize v (one neuron per token: each slot accumulates whole rows)
  float lv, uv;
  {
    float NLv = 0.f, NUv = 0.f;
    for (int pb = 0; pb < P; ++pb) {
      float acc[2] = {0.f, 0.f};
      for (int r = pb * E + ge.slot; r < (pb + 1) * E; r += ge.NS) {
        LnRow<VEC> x;
        ln_load_row<VEC>(S, R, row, C, r, n, ge, x);
        float vl, vu;
        v_row(x, vl, vu);
        acc[0] = norm_acc(acc[0], vl, pn);
        acc[1] = norm_acc(acc[1], vu, pn);
      }
      slot_reduce<2>(acc, ge, pn == 1, red);
      NLv += norm_fin(acc[0], pn);
      NUv += norm_fin(acc[1], pn);
    }
    LnRow<VEC> x;
    ln_load_row<VEC>(S, R, row, C, C - 1, n, ge, x);
    float vl, vu;
    v_row(x, vl, vu);
    lv = vl + cql + ln_eps - e * NLv;
    uv = vu + cqu + ln_eps + e * NUv;
    bad |= !(finite_f(lv) && finite_f(uv));
  }
  // sqrt and reciprocal on the scalar v: rho_L = a_L v_U + g_L, rho_U = a_U v_L + g_U
  const float lvc = fmaxf(lv, ln_eps), uvc = fmaxf(uv, lvc);
  const Line2 sq = relax_sqrt(lvc, uvc);
  float ls, us;
  line_range(sq.kL, sq.cL, sq.kU, sq.cU, lv, uv, ls, us);       // range of the sqrt state (unclamped v state)
  ls = fmaxf(ls, sqrtf(ln_eps)); us = fmaxf(us, ls);
  const Line2 rc = relax_recip(ls, us);
  float lr, ur;
  line_range(rc.kL, rc.cL, rc.kU, rc.cU, ls, us, lr, ur);
  // (the reciprocal's range uses the clamped sqrt range; its slopes are negative, so it reads the
  //  opposite side of the sqrt state)
  {
    // range of rho from the *state* of s: s_L = kLs v_L + cLs (range [ls_state, us_state]); the state
    // range before clamping is what the norm of rho's coefficients scales with
    float ls0, us0;
    line_range(sq.kL, sq.cL, sq.kU, sq.cU, lv, uv, ls0, us0);
    lr = rc.kL * us0 + rc.cL;
    ur = rc.kU * ls0 + rc.cU;
  }
  const float aL = rc.kL * sq.kU, gL = rc.kL * (sq.cU + sq.kU * (cqu + ln_eps)) + rc.cL;   // on v_U (without intercepts)
  const float aU = rc.kU * sq.kL, gU = rc.kU * (sq.cL + sq.kL * (cql + ln_eps)) + rc.cU;   // on v_L
  if (bad) status[row / rps] = 1;

  // ---- sweep 3: y = c * rho (McCormick, x = c_d, y = rho), then gamma / beta
  float gm[4 * VEC], bt[4 * VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    const int f = ge.g + ge.G * v;
    float4 a = make_float4(0, 0, 0, 0), b = a;
    if (f < ge.n4) { a = reinterpret_cast<const float4 *>(gamma)[f]; b = reinterpret_cast<const float4 *>(beta)[f]; }
#pragma unroll
    for (int c = 0; c < 4; ++c) { gm[4 * v + c] = CF4(a, c); bt[4 * v + c] = CF4(b, c); }
  }
  for (int r = ge.slot; r < C; r += ge.NS) {
    LnRow<VEC> x;
    ln_load_row<VEC>(S, R, row, C, r, n, ge, x);
    float vl, vu;
    v_row(x, vl, vu);
    const bool last = r == C - 1;
    float rhoL = aL * vu, rhoU = aU * vl;          // rho's lower / upper linear forms at coefficient row r
    if (last) { rhoL += gL; rhoU += gU; }
    float4 *qs = row_ptr(So, row, C, r, n, 0), *qr = row_ptr(Ro, row, C, r, n, 0);
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      float4 os, orr;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int i = 4 * v + c;
        const float lo = x.sc[i] - x.rc[i], up = x.sc[i] + x.rc[i];
        // lower: lr * c + lc * rho - lc lr ; upper: ur * c + lc * rho - lc ur  (sign rule per slope)
        float yl = (lr >= 0.f ? lr * lo : lr * up) + (lc[i] >= 0.f ? lc[i] * rhoL : lc[i] * rhoU);
        float yu = (ur >= 0.f ? ur * up : ur * lo) + (lc[i] >= 0.f ? lc[i] * rhoU : lc[i] * rhoL);
        if (last) { yl -= lc[i] * lr; yu -= lc[i] * ur; }
        float ol = gm[i] >= 0.f ? gm[i] * yl : gm[i] * yu;
        float ou = gm[i] >= 0.f ? gm[i] * yu : gm[i] * yl;
        if (last) { ol += bt[i]; ou += bt[i]; }
        F4(os, c) = 0.5f * (ou + ol);
        F4(orr, c) = 0.5f * (ou - ol);
      }
      if (f < ge.n4) { qs[f] = os; qr[f] = orr; }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Softmax bound over the last axis of the score state, in place.  One workgroup per attention row.
//   shift by max_j u_j ; e = exp (relaxed) ; sigma = sum_j e ; rho = 1 / sigma ; p = e * rho.
// Sweeps: norms of s; norm of sigma; output p (and the norm of p for its concretized bounds).
template <int VEC>
__global__ __launch_bounds__(kThreads) void softmax_kernel(float *S, float *R, int P, int E, int n, int G, int rps,
                                                           int pn, const float *eps, float *lp_out,
                                                           int32_t *status) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int C = P * E + 1;
  const Geo ge(G, n / 4);
  const float e = eps[row / rps];
  bool colon[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) colon[v] = ge.g + ge.G * v < ge.n4;
  bool bad = false;

  float NL[4 * VEC], NU[4 * VEC], bL[4 * VEC], bU[4 * VEC];
  column_norms<VEC>(S, R, row, P, E, n, 0, ge, pn, nullptr, red, NL, NU, bL, bU);
  float ls[4 * VEC], us[4 * VEC];
  float mx = -FLT_MAX;
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) {
    ls[i] = bL[i] - e * NL[i]; us[i] = bU[i] + e * NU[i];
    if (colon[i / 4]) { bad |= !(finite_f(ls[i]) && finite_f(us[i])); mx = fmaxf(mx, us[i]); }
  }
  const float shift = cols_max(mx, ge.G);
  // exp relaxation per column on the shifted range; slopes are positive
  float kLe[4 * VEC], kUe[4 * VEC], cLe[4 * VEC], cUe[4 * VEC], le[4 * VEC];
  float sumcl = 0.f, sumcu = 0.f;
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) {
    const Line2 ex = relax_exp(ls[i] - shift, us[i] - shift);
    const bool on = colon[i / 4];
    kLe[i] = on ? ex.kL : 0.f; kUe[i] = on ? ex.kU : 0.f;
    // the shift moves the bias of s: fold -shift * k into the intercepts
    cLe[i] = on ? ex.cL - ex.kL * shift : 0.f; cUe[i] = on ? ex.cU - ex.kU * shift : 0.f;
    le[i] = on ? ex.kL * (ls[i] - shift) + ex.cL : 0.f;
    sumcl += cLe[i]; sumcu += cUe[i];
  }
  sumcl = row_sum(sumcl, ge.G); sumcu = row_sum(sumcu, ge.G);

  auto load_row = [&](int r, float (&lo)[4 * VEC], float (&up)[4 * VEC]) {
    const float4 *ps = row_ptr((const float *)S, row, C, r, n, 0), *pr = row_ptr((const float *)R, row, C, r, n, 0);
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      float4 s = make_float4(0, 0, 0, 0), rr = s;
      if (f < ge.n4) { s = ps[f]; rr = pr[f]; }
#pragma unroll
      for (int c = 0; c < 4; ++c) { lo[4 * v + c] = CF4(s, c) - CF4(rr, c); up[4 * v + c] = CF4(s, c) + CF4(rr, c); }
    }
  };
  auto sigma_row = [&](const float (&lo)[4 * VEC], const float (&up)[4 * VEC], float &sl, float &su) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) { a += kLe[i] * lo[i]; b += kUe[i] * up[i]; }
    sl = row_sum(a, ge.G); su = row_sum(b, ge.G);
  };

  // ---- sweep 2: concretize sigma
  float lsg, usg;
  {
    float NLs = 0.f, NUs = 0.f;
    float lo[4 * VEC], up[4 * VEC];
    for (int pb = 0; pb < P; ++pb) {
      float acc[2] = {0.f, 0.f};
      for (int r = pb * E + ge.slot; r < (pb + 1) * E; r += ge.NS) {
        load_row(r, lo, up);
        float sl, su;
        sigma_row(lo, up, sl, su);
        acc[0] = norm_acc(acc[0], sl, pn);
        acc[1] = norm_acc(acc[1], su, pn);
      }
      slot_reduce<2>(acc, ge, pn == 1, red);
      NLs += norm_fin(acc[0], pn); NUs += norm_fin(acc[1], pn);
    }
    load_row(C - 1, lo, up);
    float sl, su;
    sigma_row(lo, up, sl, su);
    lsg = sl + sumcl - e * NLs;
    usg = su + sumcu + e * NUs;
  }
  bad |= !(finite_f(lsg) && finite_f(usg)) || !(lsg >= kRecipMin);
  const Line2 rc = relax_recip(lsg, usg);
  float lr, ur;
  line_range(rc.kL, rc.cL, rc.kU, rc.cU, lsg, usg, lr, ur);
  // rho_L[r] = kLr * sigma_U[r] (+ kLr * sumcu + cLr on the bias row); rho_U[r] = kUr * sigma_L[r] (+ ...)
  const float gL = rc.kL * sumcu + rc.cL, gU = rc.kU * sumcl + rc.cU;
  if (bad) status[row / rps] = 1;

  // ---- sweep 3: p = e * rho (x = e_j, y = rho): lower lr e + le rho - le lr ; upper ur e + le rho - le ur
  float NLp[4 * VEC], NUp[4 * VEC], pbl[4 * VEC], pbu[4 * VEC];
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) NLp[i] = NUp[i] = pbl[i] = pbu[i] = 0.f;
  for (int pb = 0; pb <= P; ++pb) {          // block P is the bias row
    float acc[8 * VEC];
#pragma unroll
    for (int i = 0; i < 8 * VEC; ++i) acc[i] = 0.f;
    const int rbeg = pb < P ? pb * E : C - 1, rend = pb < P ? (pb + 1) * E : C;
    for (int r = rbeg + ge.slot; r < rend; r += ge.NS) {
      float lo[4 * VEC], up[4 * VEC];
      load_row(r, lo, up);
      float sl, su;
      sigma_row(lo, up, sl, su);
      const bool last = r == C - 1;
      float rhoL = rc.kL * su, rhoU = rc.kU * sl;
      if (last) { rhoL += gL; rhoU += gU; }
      float4 *qs = row_ptr(S, row, C, r, n, 0), *qr = row_ptr(R, row, C, r, n, 0);
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const int f = ge.g + ge.G * v;
        float4 os, orr;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int i = 4 * v + c;
          float eL = kLe[i] * lo[i], eU = kUe[i] * up[i];
          if (last) { eL += cLe[i]; eU += cUe[i]; }
          float pl = (lr >= 0.f ? lr * eL : lr * eU) + (le[i] >= 0.f ? le[i] * rhoL : le[i] * rhoU);
          float pu = (ur >= 0.f ? ur * eU : ur * eL) + (le[i] >= 0.f ? le[i] * rhoU : le[i] * rhoL);
          if (last) { pl -= le[i] * lr; pu -= le[i] * ur; pbl[i] = pl; pbu[i] = pu; }
          else { acc[2 * i] = norm_acc(acc[2 * i], pl, pn); acc[2 * i + 1] = norm_acc(acc[2 * i + 1], pu, pn); }
          F4(os, c) = 0.5f * (pu + pl);
          F4(orr, c) = 0.5f * (pu - pl);
        }
        if (f < ge.n4) { qs[f] = os; qr[f] = orr; }
      }
    }
    if (pb < P) {
      slot_reduce<8 * VEC>(acc, ge, pn == 1, red);
#pragma unroll
      for (int i = 0; i < 4 * VEC; ++i) { NLp[i] += norm_fin(acc[2 * i], pn); NUp[i] += norm_fin(acc[2 * i + 1], pn); }
    }
  }
  // concretized lower bound of p, clamped to [0, 1]; the bias row was handled by slot 0
  {
    float bb[8 * VEC];
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) { bb[2 * i] = pbl[i]; bb[2 * i + 1] = pbu[i]; }
    slot_reduce<8 * VEC>(bb, ge, false, red);      // only one slot holds non-zero values
    if (ge.slot == 0) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const int f = ge.g + ge.G * v;
        float4 o;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int i = 4 * v + c;
          const float l = bb[2 * i] - e * NLp[i];
          F4(o, c) = fminf(fmaxf(l, 0.f), 1.f);
        }
        if (f < ge.n4) reinterpret_cast<float4 *>(lp_out + row * n)[f] = o;
      }
    }
  }
}

__global__ void abs_kernel(const float *in, float *out, size_t count) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) out[i] = fabsf(in[i]);
}
__global__ void zero_kernel(float4 *p, size_t count4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < count4; i += stride) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

int pow2_le(int x) { int p = 1; while (p * 2 <= x) p *= 2; return p; }
int pow2_ge(int x) { int p = 1; while (p < x) p *= 2; return p; }
int gcd(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }

// chunked geometry for per-column kernels: G = gcd(n/4, 64) lanes, one float4 per lane
void chunk_geo(int n, int &G, int &nchunks) {
  G = gcd(n / 4, 64);
  nchunks = (n + 4 * G - 1) / (4 * G);
}
// whole-row geometry: G lanes (power of two), VEC float4 per lane
int row_geo(int n, int &G, int &VEC) {
  G = pow2_ge(n / 4); if (G > 64) G = 64;
  VEC = (n / 4 + G - 1) / G;
  return VEC <= kMaxVec;
}

int check_common(const void *S, const void *R, int rows, int P, int E, int n, int rps, int pn, const float *eps) {
  TV_REQUIRE(S && R && eps, TV_E_NULL, "null state or eps pointer");
  TV_REQUIRE(rows > 0 && P >= 0 && P <= kMaxP && E > 0 && n > 0 && n % 4 == 0 && rps > 0 && rows % rps == 0,
             TV_E_SHAPE, "bad shape rows=%d P=%d E=%d n=%d rows_per_sentence=%d", rows, P, E, n, rps);
  TV_REQUIRE(norm_ok(pn), TV_E_NORM, "p_norm must be 1, 2 or TV_NORM_INF, got %d", pn);
  return TV_OK;
}

}  // namespace

int concretize(CState x, int rows, int P, int E, int n, int ld, int rps, int pn, const float *eps, float *l,
               float *u, hipStream_t st) {
  if (int rc = check_common(x.S, x.R, rows, P, E, n, rps, pn, eps)) return rc;
  TV_REQUIRE(l && u, TV_E_NULL, "null output");
  TV_REQUIRE(ld >= n && ld % 4 == 0, TV_E_SHAPE, "concretize: row stride %d must be a multiple of 4 and >= %d", ld, n);
  int G, nch;
  chunk_geo(n, G, nch);
  hipLaunchKernelGGL((concretize_kernel<1>), dim3(rows, nch), dim3(kThreads), 0, st, x.S, x.R, P, E, n, ld, G, rps,
                     pn, eps, l, u);
  TV_HIP(hipGetLastError());
  return TV_OK;
}

int activation(int act, CState x, int rows, int P, int E, int n, int rps, int pn, const float *eps, State y,
               int32_t *status, hipStream_t st) {
  if (int rc = check_common(x.S, x.R, rows, P, E, n, rps, pn, eps)) return rc;
  TV_REQUIRE(y.S && y.R && status, TV_E_NULL, "null output");
  TV_REQUIRE(act == TV_ACT_RELU || act == TV_ACT_TANH || act == TV_ACT_GELU, TV_E_ARG, "unknown activation %d", act);
  int G, nch;
  chunk_geo(n, G, nch);
  dim3 grid(rows, nch), block(kThreads);
  if (act == TV_ACT_RELU)
    hipLaunchKernelGGL((activation_kernel<1, TV_ACT_RELU>), grid, block, 0, st, x.S, x.R, P, E, n, G, rps, pn, eps,
                       y.S, y.R, status);
  else if (act == TV_ACT_TANH)
    hipLaunchKernelGGL((activation_kernel<1, TV_ACT_TANH>), grid, block, 0, st, x.S, x.R, P, E, n, G, rps, pn, eps,
                       y.S, y.R, status);
  else
    hipLaunchKernelGGL((activation_kernel<1, TV_ACT_GELU>), grid, block, 0, st, x.S, x.R, P, E, n, G, rps, pn, eps,
                       y.S, y.R, status);
  TV_HIP(hipGetLastError());
  return TV_OK;
}

int layernorm(CState x, int rows, int P, int E, int n, int rps, int pn, const float *eps, const float *gamma,
              const float *beta, float ln_eps, State y, int32_t *status, hipStream_t st) {
  if (int rc = check_common(x.S, x.R, rows, P, E, n, rps, pn, eps)) return rc;
  TV_REQUIRE(y.S && y.R && status && gamma && beta, TV_E_NULL, "null pointer");
  TV_REQUIRE(ln_eps > 0.f, TV_E_ARG, "ln_eps must be positive");
  int G, VEC;
  TV_REQUIRE(row_geo(n, G, VEC), TV_E_SHAPE, "layernorm width %d exceeds %d", n, 4 * 64 * kMaxVec);
  dim3 grid(rows), block(kThreads);
#define LN_LAUNCH(V)                                                                                            \
  hipLaunchKernelGGL((layernorm_kernel<V>), grid, block, 0, st, x.S, x.R, P, E, n, G, rps, pn, eps, gamma, beta, \
                     ln_eps, y.S, y.R, status)
  switch (VEC) {
    case 1: LN_LAUNCH(1); break;
    case 2: LN_LAUNCH(2); break;
    case 3: LN_LAUNCH(3); break;
    default: LN_LAUNCH(4); break;
  }
#undef LN_LAUNCH
  TV_HIP(hipGetLastError());
  return TV_OK;
}

int softmax(State s, int rows, int P, int E, int L, int rps, int pn, const float *eps, float *lp, int32_t *status,
            hipStream_t st) {
  if (int rc = check_common(s.S, s.R, rows, P, E, L, rps, pn, eps)) return rc;
  TV_REQUIRE(lp && status, TV_E_NULL, "null pointer");
  int G, VEC;
  TV_REQUIRE(row_geo(L, G, VEC), TV_E_SHAPE, "softmax width %d exceeds %d", L, 4 * 64 * kMaxVec);
  dim3 grid(rows), block(kThreads);
#define SM_LAUNCH(V) \
  hipLaunchKernelGGL((softmax_kernel<V>), grid, block, 0, st, s.S, s.R, P, E, L, G, rps, pn, eps, lp, status)
  switch (VEC) {
    case 1: SM_LAUNCH(1); break;
    case 2: SM_LAUNCH(2); break;
    case 3: SM_LAUNCH(3); break;
    default: SM_LAUNCH(4); break;
  }
#undef SM_LAUNCH
  TV_HIP(hipGetLastError());
  return TV_OK;
}

int vec_abs(const float *in, float *out, size_t count, hipStream_t st) {
  TV_REQUIRE(in && out, TV_E_NULL, "null pointer");
  if (count == 0) return TV_OK;
  const unsigned blocks = (unsigned)((count + 255) / 256 > 4096 ? 4096 : (count + 255) / 256);
  hipLaunchKernelGGL(abs_kernel, dim3(blocks), dim3(256), 0, st, in, out, count);
  TV_HIP(hipGetLastError());
  return TV_OK;
}

int fill_zero(float *p, size_t count, hipStream_t st) {
  TV_REQUIRE(p && count % 4 == 0, TV_E_ARG, "fill_zero: count must be a multiple of 4");
  if (count == 0) return TV_OK;
  const size_t c4 = count / 4;
  const unsigned blocks = (unsigned)((c4 + 255) / 256 > 8192 ? 8192 : (c4 + 255) / 256);
  hipLaunchKernelGGL(zero_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<float4 *>(p), c4);
  TV_HIP(hipGetLastError());
  return TV_OK;
}

}  // namespace tv
