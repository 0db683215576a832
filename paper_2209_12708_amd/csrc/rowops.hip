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
// Norms of a lower and an upper line of the state down the coefficient axis, for this thread's columns:
//   NL = N(aS * S + aR * R),  NU = N(bS * S + bR * R),    N = sum over the P blocks of the dual norm.
// lines == nullptr means the state's own lines (S - R, S + R).  Also returns the bias-row S and R.
struct LineCoef { float aS, aR, bS, bR; };

template <int VEC>
__device__ __forceinline__ void column_norms(const float *S, const float *R, long row, int P, int E, int n, int c0,
                                             const Geo &ge, int pn, const LineCoef *lines, float *red,
                                             float (&NL)[4 * VEC], float (&NU)[4 * VEC], float (&bS)[4 * VEC],
                                             float (&bR)[4 * VEC]) {
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
            float a = CF4(s, c) - CF4(rr, c), b = CF4(s, c) + CF4(rr, c);
            if (lines) {
              const LineCoef &lc = lines[4 * v + c];
              a = lc.aS * CF4(s, c) + lc.aR * CF4(rr, c);
              b = lc.bS * CF4(s, c) + lc.bR * CF4(rr, c);
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
    for (int c = 0; c < 4; ++c) { bS[4 * v + c] = CF4(s, c); bR[4 * v + c] = CF4(rr, c); }
  }
}

// Concretized range as (mid, half) in double from centre / radius biases and the two norms:
//   l = (bS - bR) - e NL,  u = (bS + bR) + e NU   =>   mid = bS + e (NU - NL)/2,  half = bR + e (NU + NL)/2.
// Both are sums of quantities that fp32 holds accurately, so narrow intervals keep their width.
__device__ __forceinline__ void range_of(double bS, double bR, double e, double NL, double NU, double &l, double &u) {
  const double mid = bS + 0.5 * e * (NU - NL), half = bR + 0.5 * e * (NU + NL);
  l = mid - half; u = mid + half;
}
__device__ __forceinline__ bool finite_d(double x) { return fabs(x) <= 3.4028234663852886e38; }

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
// Eq. (1).  grid = (rows, column chunks).  mode 0 writes (l, u); mode 1 writes (mid, half).
template <int VEC>
__global__ __launch_bounds__(kThreads) void concretize_kernel(const float *S, const float *R, int P, int E, int n,
                                                              int ld, int G, int rps, int pn, const float *eps,
                                                              float *o0, float *o1, int mode) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int chunk = 4 * G * VEC, c0 = blockIdx.y * chunk;
  const Geo ge(G, min(chunk, n - c0) / 4);
  float NL[4 * VEC], NU[4 * VEC], bS[4 * VEC], bR[4 * VEC];
  column_norms<VEC>(S, R, row, P, E, ld, c0, ge, pn, nullptr, red, NL, NU, bS, bR);
  if (ge.slot == 0) {
    const float e = eps[row / rps];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      if (f < ge.n4) {
        float4 a, b;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int i = 4 * v + c;
          if (mode == 0) {
            F4(a, c) = (bS[i] - bR[i]) - e * NL[i];
            F4(b, c) = (bS[i] + bR[i]) + e * NU[i];
          } else {
            F4(a, c) = bS[i] + 0.5f * e * (NU[i] - NL[i]);
            F4(b, c) = bR[i] + 0.5f * e * (NU[i] + NL[i]);
          }
        }
        reinterpret_cast<float4 *>(o0 + row * n + c0)[f] = a;
        reinterpret_cast<float4 *>(o1 + row * n + c0)[f] = b;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Activation: concretize, relax, substitute - one workgroup reads its coefficients for the norm and
// again (from cache) for the rescale.  GELU adds one mapped-norm pass for the inner product.
__device__ __forceinline__ Form gelu_inner(double lx, double ux, double &lb, double &ub) {
  // a = x^2 ; b = k (1 + c3 a) ; returns the form of b and its range
  const double k = 0.7978845608028654, c3 = 0.044715;
  const Line2 sq = relax_square(lx, ux);
  const Form a = form_sub(form_identity(), sq);
  double la, ua;
  line_range(sq, lx, ux, la, ua);
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
  const double e = eps[row / rps];
  float NL[4 * VEC], NU[4 * VEC], bS[4 * VEC], bR[4 * VEC];
  column_norms<VEC>(S, R, row, P, E, n, c0, ge, pn, nullptr, red, NL, NU, bS, bR);
  Map2 maps[4 * VEC];
  bool bad = false;
  if (ACT != TV_ACT_GELU) {
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      double l, u;
      range_of(bS[i], bR[i], e, NL[i], NU[i], l, u);
      bad |= !(finite_d(l) && finite_d(u));
      const Line2 ln = ACT == TV_ACT_RELU ? relax_relu(l, u) : relax_tanh(l, u);
      maps[i] = form_map(form_sub(form_identity(), ln));
    }
  } else {
    Form fg[4 * VEC];
    LineCoef lc[4 * VEC];
    double lx[4 * VEC], ux[4 * VEC];
    float xS[4 * VEC], xR[4 * VEC];
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      range_of(bS[i], bR[i], e, NL[i], NU[i], lx[i], ux[i]);
      bad |= !(finite_d(lx[i]) && finite_d(ux[i]));
      double lb, ub;
      const Form b = gelu_inner(lx[i], ux[i], lb, ub);
      fg[i] = form_mul(form_identity(), b, lx[i], lb, ub);     // g = x * b
      lc[i] = LineCoef{(float)(fg[i].pL + fg[i].qL), (float)(fg[i].qL - fg[i].pL), (float)(fg[i].pU + fg[i].qU),
                       (float)(fg[i].pU - fg[i].qU)};
      xS[i] = bS[i]; xR[i] = bR[i];
    }
    column_norms<VEC>(S, R, row, P, E, n, c0, ge, pn, lc, red, NL, NU, bS, bR);
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      // bias values of g's two lines, as centre / radius in double
      const Form &f = fg[i];
      const double gS = 0.5 * ((f.pL + f.qL + f.pU + f.qU) * xS[i] + (-f.pL + f.qL + f.pU - f.qU) * xR[i] + f.cL + f.cU);
      const double gR = 0.5 * ((f.pU + f.qU - f.pL - f.qL) * xS[i] + (f.pU - f.qU + f.pL - f.qL) * xR[i] + f.cU - f.cL);
      double lg, ug;
      range_of(gS, gR, e, NL[i], NU[i], lg, ug);
      bad |= !(finite_d(lg) && finite_d(ug));
      const Line2 th = relax_tanh(lg, ug);
      double lt, ut;
      line_range(th, lg, ug, lt, ut);
      const Form h = form_sub(form_sub(f, th), 0.5, 0.5, 0.5, 0.5);
      maps[i] = form_map(form_mul(form_identity(), h, lx[i], 0.5 * lt + 0.5, 0.5 * ut + 0.5));
    }
  }
  if (bad) status[row / rps] = 1;
  apply_maps<VEC>(S, R, So, Ro, row, C, n, c0, ge, maps);
}

// ------------------------------------------------------------------------------------------------
// LayerNorm bound.  One workgroup per token; lanes cover all n columns (VEC float4 per lane).
//   c = x - mean(x)                 one affine map (I - 11^T/n): S_c = S - mean S, R_c = (1-2/n) R + mean R
//   q = c^2 (relaxed) ; v = mean q + ln_eps ; s = sqrt v ; rho = 1/s ; y = c * rho ; out = gamma y + beta
// Three sweeps over the block: norms of c; norm of v; output.  All streaming arithmetic is on centre
// and radius planes (never on lower / upper values, whose difference fp32 cannot hold).
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
                                                             const float *gamma, const float *beta, float ln_eps_f,
                                                             float *So, float *Ro, int32_t *status) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int C = P * E + 1;
  const Geo ge(G, n / 4);
  const double e = eps[row / rps];
  const double ln_eps = ln_eps_f;
  const float inv = 1.f / (float)n;
  bool colon[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) colon[v] = ge.g + ge.G * v < ge.n4;
  bool bad = false;

  // ---- sweep 1: concretize c
  float lc[4 * VEC];         // lower end of c's range (the McCormick multiplier on rho)
  Map2 mq[4 * VEC];          // centre / radius map of the square relaxation, relative to c
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
      double l, u;
      range_of(x.sc[i], x.rc[i], e, NL[i], NU[i], l, u);
      if (colon[i / 4]) bad |= !(finite_d(l) && finite_d(u));
      lc[i] = (float)l;
      mq[i] = form_map(form_sub(form_identity(), relax_square(l, u)));
      if (!colon[i / 4]) mq[i] = Map2{0, 0, 0, 0, 0, 0};
    }
  }
  // v = mean_d q + ln_eps, as centre / radius per coefficient row
  auto v_row = [&](const LnRow<VEC> &x, float &vS, float &vR) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      a += mq[i].sS * x.sc[i] + mq[i].sR * x.rc[i];
      b += mq[i].rS * x.sc[i] + mq[i].rR * x.rc[i];
    }
    vS = row_sum(a, ge.G) * inv;
    vR = row_sum(b, ge.G) * inv;
  };
  float cvS = 0.f, cvR = 0.f;   // constants of v on the bias row
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) { cvS += mq[i].sC; cvR += mq[i].rC; }
  cvS = row_sum(cvS, ge.G) * inv + ln_eps_f; cvR = row_sum(cvR, ge.G) * inv;

  // ---- sweep 2: concretize v (one neuron per token: each slot accumulates whole rows)
  double lv, uv;
  {
    float NLv = 0.f, NUv = 0.f;
    for (int pb = 0; pb < P; ++pb) {
      float acc[2] = {0.f, 0.f};
      for (int r = pb * E + ge.slot; r < (pb + 1) * E; r += ge.NS) {
        LnRow<VEC> x;
        ln_load_row<VEC>(S, R, row, C, r, n, ge, x);
        float vS, vR;
        v_row(x, vS, vR);
        acc[0] = norm_acc(acc[0], vS - vR, pn);
        acc[1] = norm_acc(acc[1], vS + vR, pn);
      }
      slot_reduce<2>(acc, ge, pn == 1, red);
      NLv += norm_fin(acc[0], pn);
      NUv += norm_fin(acc[1], pn);
    }
    LnRow<VEC> x;
    ln_load_row<VEC>(S, R, row, C, C - 1, n, ge, x);
    float vS, vR;
    v_row(x, vS, vR);
    range_of((double)vS + cvS, (double)vR + cvR, e, NLv, NUv, lv, uv);
    bad |= !(finite_d(lv) && finite_d(uv));
  }
  // sqrt and reciprocal on the scalar v (double): ranges from the states, clamped where the true value allows
  const double lvc = fmax(lv, ln_eps), uvc = fmax(uv, lvc);
  const Line2 sq = relax_sqrt(lvc, uvc);
  double ls0, us0;
  line_range(sq, lv, uv, ls0, us0);                 // range of the sqrt state (from the unclamped v state)
  const double ls = fmax(ls0, sqrt(ln_eps)), us = fmax(us0, ls);
  const Line2 rc = relax_recip(ls, us);
  double lr, ur;
  line_range(rc, ls0, us0, lr, ur);                 // range of rho's state
  const Map2 mr = form_map(form_sub(form_sub(form_identity(), sq), rc));   // rho relative to v
  const Mul2 mc = mul_coeffs(lr, ur);
  if (bad) status[row / rps] = 1;

  // ---- sweep 3: y = c * rho (x = c_d with multiplier range of rho; y = rho with multiplier lc_d), gamma / beta
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
    float vS, vR;
    v_row(x, vS, vR);
    const bool last = r == C - 1;
    if (last) { vS += cvS; vR += cvR; }
    float rhoS = mr.sS * vS + mr.sR * vR, rhoR = mr.rS * vS + mr.rR * vR;
    if (last) { rhoS += mr.sC; rhoR += mr.rC; }
    float4 *qs = row_ptr(So, row, C, r, n, 0), *qr = row_ptr(Ro, row, C, r, n, 0);
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      float4 os, orr;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int i = 4 * v + c;
        float yS = mc.a1 * x.sc[i] + mc.a2 * x.rc[i] + lc[i] * rhoS;
        float yR = mc.a3 * x.sc[i] + mc.a4 * x.rc[i] + fabsf(lc[i]) * rhoR;
        if (last) { yS -= lc[i] * mc.a1; yR -= lc[i] * mc.a3; }
        float oS = gm[i] * yS, oR = fabsf(gm[i]) * yR;
        if (last) oS += bt[i];
        F4(os, c) = oS;
        F4(orr, c) = oR;
      }
      if (f < ge.n4) { qs[f] = os; qr[f] = orr; }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Softmax bound over the last axis of the score state, in place.  One workgroup per attention row.
//   shift by max_j u_j ; e = exp (relaxed) ; sigma = sum_j e ; rho = 1 / sigma ; p = e * rho.
// Sweeps: norms of s; norm of sigma; output p (and the norm of p's lower line for its concretized bound).
template <int VEC>
__global__ __launch_bounds__(kThreads) void softmax_kernel(float *S, float *R, int P, int E, int n, int G, int rps,
                                                           int pn, const float *eps, float *lp_out,
                                                           int32_t *status) {
  __shared__ float red[4 * kWave * 8 * VEC];
  const long row = blockIdx.x;
  const int C = P * E + 1;
  const Geo ge(G, n / 4);
  const double e = eps[row / rps];
  bool colon[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) colon[v] = ge.g + ge.G * v < ge.n4;
  bool bad = false;

  float NL[4 * VEC], NU[4 * VEC], bS[4 * VEC], bR[4 * VEC];
  column_norms<VEC>(S, R, row, P, E, n, 0, ge, pn, nullptr, red, NL, NU, bS, bR);
  double ls[4 * VEC], us[4 * VEC];
  float mx = -FLT_MAX;
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) {
    range_of(bS[i], bR[i], e, NL[i], NU[i], ls[i], us[i]);
    if (colon[i / 4]) { bad |= !(finite_d(ls[i]) && finite_d(us[i])); mx = fmaxf(mx, (float)us[i]); }
  }
  const double shift = cols_max(mx, ge.G);
  // exp relaxation per column on the shifted range (slopes positive); the shift moves s's bias, which
  // is folded into the constants of the map
  Map2 me[4 * VEC];
  float le[4 * VEC];
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) {
    const Line2 ex = relax_exp(ls[i] - shift, us[i] - shift);
    Line2 sh = ex;
    sh.cL = ex.cL - ex.kL * shift; sh.cU = ex.cU - ex.kU * shift;
    me[i] = form_map(form_sub(form_identity(), sh));
    le[i] = (float)(ex.kL * (ls[i] - shift) + ex.cL);
    if (!colon[i / 4]) { me[i] = Map2{0, 0, 0, 0, 0, 0}; le[i] = 0.f; }
  }
  float csS = 0.f, csR = 0.f;   // constants of sigma on the bias row
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) { csS += me[i].sC; csR += me[i].rC; }
  csS = row_sum(csS, ge.G); csR = row_sum(csR, ge.G);

  auto load_row = [&](int r, float (&xs)[4 * VEC], float (&xr)[4 * VEC]) {
    const float4 *ps = row_ptr((const float *)S, row, C, r, n, 0), *pr = row_ptr((const float *)R, row, C, r, n, 0);
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int f = ge.g + ge.G * v;
      float4 s = make_float4(0, 0, 0, 0), rr = s;
      if (f < ge.n4) { s = ps[f]; rr = pr[f]; }
#pragma unroll
      for (int c = 0; c < 4; ++c) { xs[4 * v + c] = CF4(s, c); xr[4 * v + c] = CF4(rr, c); }
    }
  };
  // e's planes for one coefficient row (without bias constants) and sigma's planes
  auto e_row = [&](const float (&xs)[4 * VEC], const float (&xr)[4 * VEC], float (&eS)[4 * VEC], float (&eR)[4 * VEC],
                   float &sgS, float &sgR) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) {
      eS[i] = me[i].sS * xs[i] + me[i].sR * xr[i];
      eR[i] = me[i].rS * xs[i] + me[i].rR * xr[i];
      a += eS[i]; b += eR[i];
    }
    sgS = row_sum(a, ge.G); sgR = row_sum(b, ge.G);
  };

  // ---- sweep 2: concretize sigma
  double lsg, usg;
  {
    float NLs = 0.f, NUs = 0.f;
    float xs[4 * VEC], xr[4 * VEC], eS[4 * VEC], eR[4 * VEC];
    for (int pb = 0; pb < P; ++pb) {
      float acc[2] = {0.f, 0.f};
      for (int r = pb * E + ge.slot; r < (pb + 1) * E; r += ge.NS) {
        load_row(r, xs, xr);
        float sgS, sgR;
        e_row(xs, xr, eS, eR, sgS, sgR);
        acc[0] = norm_acc(acc[0], sgS - sgR, pn);
        acc[1] = norm_acc(acc[1], sgS + sgR, pn);
      }
      slot_reduce<2>(acc, ge, pn == 1, red);
      NLs += norm_fin(acc[0], pn); NUs += norm_fin(acc[1], pn);
    }
    load_row(C - 1, xs, xr);
    float sgS, sgR;
    e_row(xs, xr, eS, eR, sgS, sgR);
    range_of((double)sgS + csS, (double)sgR + csR, e, NLs, NUs, lsg, usg);
  }
  bad |= !(finite_d(lsg) && finite_d(usg)) || !(lsg >= kRecipMin);
  const Line2 rc = relax_recip(lsg, usg);
  double lr, ur;
  line_range(rc, lsg, usg, lr, ur);
  const Map2 mr = form_map(form_sub(form_identity(), rc));      // rho relative to sigma
  const Mul2 mc = mul_coeffs(lr, ur);
  if (bad) status[row / rps] = 1;

  // ---- sweep 3: p = e * rho (x = e_j with multiplier range of rho; y = rho with multiplier le_j)
  float NLp[4 * VEC], pbl[4 * VEC];
#pragma unroll
  for (int i = 0; i < 4 * VEC; ++i) NLp[i] = pbl[i] = 0.f;
  for (int pb = 0; pb <= P; ++pb) {          // block P is the bias row
    float acc[4 * VEC];
#pragma unroll
    for (int i = 0; i < 4 * VEC; ++i) acc[i] = 0.f;
    const int rbeg = pb < P ? pb * E : C - 1, rend = pb < P ? (pb + 1) * E : C;
    for (int r = rbeg + ge.slot; r < rend; r += ge.NS) {
      float xs[4 * VEC], xr[4 * VEC], eS[4 * VEC], eR[4 * VEC];
      load_row(r, xs, xr);
      float sgS, sgR;
      e_row(xs, xr, eS, eR, sgS, sgR);
      const bool last = r == C - 1;
      if (last) { sgS += csS; sgR += csR; }
      float rhoS = mr.sS * sgS + mr.sR * sgR, rhoR = mr.rS * sgS + mr.rR * sgR;
      if (last) { rhoS += mr.sC; rhoR += mr.rC; }
      float4 *qs = row_ptr(S, row, C, r, n, 0), *qr = row_ptr(R, row, C, r, n, 0);
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const int f = ge.g + ge.G * v;
        float4 os, orr;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int i = 4 * v + c;
          float es = eS[i], er = eR[i];
          if (last) { es += me[i].sC; er += me[i].rC; }
          float pS = mc.a1 * es + mc.a2 * er + le[i] * rhoS;
          float pR = mc.a3 * es + mc.a4 * er + fabsf(le[i]) * rhoR;
          if (last) { pS -= le[i] * mc.a1; pR -= le[i] * mc.a3; pbl[i] = pS - pR; }
          else acc[i] = norm_acc(acc[i], pS - pR, pn);
          F4(os, c) = pS;
          F4(orr, c) = pR;
        }
        if (f < ge.n4) { qs[f] = os; qr[f] = orr; }
      }
    }
    if (pb < P) {
      slot_reduce<4 * VEC>(acc, ge, pn == 1, red);
#pragma unroll
      for (int i = 0; i < 4 * VEC; ++i) NLp[i] += norm_fin(acc[i], pn);
    }
  }
  // concretized lower bound of p, clamped to [0, 1]; the bias row was handled by slot 0
  {
    slot_reduce<4 * VEC>(pbl, ge, false, red);      // only one slot holds non-zero values
    if (ge.slot == 0) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const int f = ge.g + ge.G * v;
        float4 o;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int i = 4 * v + c;
          const float l = pbl[i] - (float)e * NLp[i];
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
               float *u, int mode, hipStream_t st) {
  if (int rc = check_common(x.S, x.R, rows, P, E, n, rps, pn, eps)) return rc;
  TV_REQUIRE(l && u, TV_E_NULL, "null output");
  TV_REQUIRE(ld >= n && ld % 4 == 0, TV_E_SHAPE, "concretize: row stride %d must be a multiple of 4 and >= %d", ld, n);
  int G, nch;
  chunk_geo(n, G, nch);
  const double C = (double)P * E + 1;
  ProfScope prof(K_CONCRETIZE, st, 4.0 * rows * C * n, 8.0 * rows * C * n + 8.0 * rows * n);
  hipLaunchKernelGGL((concretize_kernel<1>), dim3(rows, nch), dim3(kThreads), 0, st, x.S, x.R, P, E, n, ld, G, rps,
                     pn, eps, l, u, mode);
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
  const double C = (double)P * E + 1;
  ProfScope prof(K_ACTIVATION, st, 12.0 * rows * C * n, 16.0 * rows * C * n);
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
  const double C = (double)P * E + 1;
  ProfScope prof(K_LAYERNORM, st, 40.0 * rows * C * n, 16.0 * rows * C * n);
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
  const double C = (double)P * E + 1;
  ProfScope prof(K_SOFTMAX, st, 40.0 * rows * C * L, 16.0 * rows * C * L);
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
