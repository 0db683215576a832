// Self-attention core on bound states: the dot-product bound with both operands perturbed (paper
// Sec. 2.3, first observation; the "generalized scalar-vector multiplication" pattern of Sec. 4.1),
// the softmax bound, and the attention x value product.
//
// z = x * y is relaxed per scalar product with the planes  z >= ly x + lx y - lx ly,
// z <= uy x + lx y - lx uy,  then both operands are substituted with the sign rule of Eq. (2).
// In centre/radius form, summed over the contracted index, this is
//   S_z = [S_x | R_x] . [(ly+uy)/2 ; (|uy|-|ly|)/2]  +  lx . S_y  - lx.(ly+uy)/2
//   R_z = [S_x | R_x] . [(uy-ly)/2 ; (|uy|+|ly|)/2]  + |lx| . R_y - lx.(uy-ly)/2
// i.e. per head two dense contractions over the state of x (K doubled, coefficients from y's
// concretized range) and two over the state of y (coefficients from x's range).  The scalars that the
// paper's kernels broadcast per vector become the small B operands of MFMA products.
//
// States are [B][C][L][*]: for one coefficient row the tokens of a sentence are contiguous, so all
// four contractions read and write dense slabs.
//
// The radius of the bias row is second order (a slack times a half-width): the MFMA products form it
// as a difference of O(1) terms, which fp32 cannot hold, so two small kernels recompute that one row
// from slacks and half-widths (no cancellation) and overwrite it.
#include "common.h"

namespace tv {
namespace {

// Ranges arrive as (mid, half) so that narrow intervals keep their width in fp32; with l = mid - half,
// u = mid + half:  (l+u)/2 = mid, (u-l)/2 = half, and (|u| -+ |l|)/2 is half / mid, -half / -mid or
// mid / half for l >= 0, u <= 0 or a crossing interval.
__device__ __forceinline__ void abs_parts(float mid, float half, float &dif, float &sum) {
  const float l = mid - half, u = mid + half;
  if (l >= 0.f) { dif = half; sum = mid; }
  else if (u <= 0.f) { dif = -half; sum = -mid; }
  else { dif = mid; sum = half; }
}

struct Ranges {   // concretized ranges of q, k, v: arrays [B][L][rld] (+ column offset already applied)
  const float *mq, *hq, *sq, *mk, *hk, *mv, *hv;
  int rld;
};

// coefficient matrices for q k^T from the concretized ranges of q and k
//   coef[b][h][plane][j][kk]   (kk < dh: on S_q ; kk >= dh: on R_q),  lqs[plane][b][i][D]
__global__ void qk_prep_kernel(Ranges rg, int B, int L, int H, int dh, float scale, float *coef, float *lqs) {
  const int D = H * dh;
  const long total = (long)B * L * D;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int dfull = (int)(i % D);
    const long bj = i / D;
    const int j = (int)(bj % L), b = (int)(bj / L);
    const int h = dfull / dh, d = dfull % dh;
    const long ri = bj * rg.rld + dfull;
    float dif, sum;
    abs_parts(rg.mk[ri], rg.hk[ri], dif, sum);
    float *c0 = coef + ((((long)b * H + h) * 2 + 0) * L + j) * (2 * dh);
    float *c1 = coef + ((((long)b * H + h) * 2 + 1) * L + j) * (2 * dh);
    c0[d] = rg.mk[ri] * scale;
    c0[dh + d] = dif * scale;
    c1[d] = rg.hk[ri] * scale;
    c1[dh + d] = sum * scale;
    const float q = rg.mq[ri] - rg.hq[ri];
    lqs[i] = q * scale;
    lqs[total + i] = fabsf(q) * scale;
  }
}

// constants of the centre plane: cst[b][h][plane][i][j] = -scale * sum_d lq[i,d] * {mid_k, half_k}[j,d]
__global__ void qk_const_kernel(Ranges rg, int B, int L, int H, int dh, float scale, float *cst) {
  const long total = (long)B * H * L * L;
  for (long t = (long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long)gridDim.x * blockDim.x) {
    const int j = (int)(t % L);
    long r = t / L;
    const int i = (int)(r % L); r /= L;
    const int h = (int)(r % H), b = (int)(r / H);
    const long oq = ((long)b * L + i) * rg.rld + h * dh, ok = ((long)b * L + j) * rg.rld + h * dh;
    float s = 0.f, rr = 0.f;
    for (int d = 0; d < dh; ++d) {
      const float q = rg.mq[oq + d] - rg.hq[oq + d];
      s = fmaf(q, rg.mk[ok + d], s);
      rr = fmaf(q, rg.hk[ok + d], rr);
    }
    float *o = cst + (((long)b * H + h) * 2) * L * L + (long)i * L + j;
    o[0] = -scale * s;
    o[(long)L * L] = -scale * rr;
  }
}

// bias row of the radius plane of the scores, from slacks and half-widths:
//   R_s_b[i,j] = scale * sum_d ( half_k[j,d] (S_q_b - l_q)[i,d] + (|u_k|+|l_k|)/2 [j,d] R_q_b[i,d] + |l_q[i,d]| R_k_b[j,d] )
__global__ void qk_fix_kernel(Ranges rg, const float *qR, const float *kR, int ld, int B, int L, int H, int dh, int C,
                              float scale, float *sR) {
  const long total = (long)B * H * L * L;
  for (long t = (long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long)gridDim.x * blockDim.x) {
    const int j = (int)(t % L);
    long r = t / L;
    const int i = (int)(r % L); r /= L;
    const int h = (int)(r % H), b = (int)(r / H);
    const long oq = ((long)b * L + i) * rg.rld + h * dh, ok = ((long)b * L + j) * rg.rld + h * dh;
    const float *qb = qR + (((long)b * C + C - 1) * L + i) * ld + h * dh;
    const float *kb = kR + (((long)b * C + C - 1) * L + j) * ld + h * dh;
    float acc = 0.f;
    for (int d = 0; d < dh; ++d) {
      float dif, sum;
      abs_parts(rg.mk[ok + d], rg.hk[ok + d], dif, sum);
      const float lq = rg.mq[oq + d] - rg.hq[oq + d];
      acc += rg.hk[ok + d] * rg.sq[oq + d] + sum * qb[d] + fabsf(lq) * kb[d];
    }
    sR[((((long)b * H + h) * C + C - 1) * L + i) * L + j] = scale * acc;
  }
}

// coefficient matrices for p v:  coef[b][h][plane][d][kk]  (kk < L: on S_p[.., j=kk] ; kk >= L: on R_p)
__global__ void pv_prep_kernel(Ranges rg, int B, int L, int H, int dh, float *coef) {
  const int D = H * dh;
  const long total = (long)B * L * D;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int dfull = (int)(i % D);
    const long bj = i / D;
    const int j = (int)(bj % L), b = (int)(bj / L);
    const int h = dfull / dh, d = dfull % dh;
    const long ri = bj * rg.rld + dfull;
    float dif, sum;
    abs_parts(rg.mv[ri], rg.hv[ri], dif, sum);
    float *c0 = coef + ((((long)b * H + h) * 2 + 0) * dh + d) * (2 * L);
    float *c1 = coef + ((((long)b * H + h) * 2 + 1) * dh + d) * (2 * L);
    c0[j] = rg.mv[ri];
    c0[L + j] = dif;
    c1[j] = rg.hv[ri];
    c1[L + j] = sum;
  }
}

// cst[plane][b][i][D] = - sum_j lp[b,h,i,j] * {mid_v, half_v}[b,j,dfull]
__global__ void pv_const_kernel(Ranges rg, const float *lp, int B, int L, int H, int dh, float *cst) {
  const int D = H * dh;
  const long total = (long)B * L * D;
  for (long t = (long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long)gridDim.x * blockDim.x) {
    const int dfull = (int)(t % D);
    const long bi = t / D;
    const int i = (int)(bi % L), b = (int)(bi / L);
    const int h = dfull / dh;
    const float *pp = lp + (((long)b * H + h) * L + i) * L;
    float s = 0.f, rr = 0.f;
    for (int j = 0; j < L; ++j) {
      const long k = ((long)b * L + j) * rg.rld + dfull;
      s = fmaf(pp[j], rg.mv[k], s);
      rr = fmaf(pp[j], rg.hv[k], rr);
    }
    cst[t] = -s;
    cst[total + t] = -rr;
  }
}

// bias row of the radius plane of the attention output:
//   R_o_b[i,d] = sum_j ( half_v[j,d] (S_p_b - l_p)[i,j] + (|u_v|+|l_v|)/2 [j,d] R_p_b[i,j] + l_p[i,j] R_v_b[j,d] )
__global__ void pv_fix_kernel(Ranges rg, const float *lp, const float *slack_p, const float *pR, const float *vR,
                              int ld, int B, int L, int H, int dh, int C, float *oR) {
  const int D = H * dh;
  const long total = (long)B * L * D;
  for (long t = (long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long)gridDim.x * blockDim.x) {
    const int dfull = (int)(t % D);
    const long bi = t / D;
    const int i = (int)(bi % L), b = (int)(bi / L);
    const int h = dfull / dh;
    const long op = (((long)b * H + h) * L + i) * L;
    const float *pb = pR + ((((long)b * H + h) * C + C - 1) * L + i) * L;
    float acc = 0.f;
    for (int j = 0; j < L; ++j) {
      const long k = ((long)b * L + j) * rg.rld + dfull;
      float dif, sum;
      abs_parts(rg.mv[k], rg.hv[k], dif, sum);
      const float vb = vR[(((long)b * C + C - 1) * L + j) * ld + dfull];
      acc += rg.hv[k] * slack_p[op + j] + sum * pb[j] + lp[op + j] * vb;
    }
    oR[(((long)b * C + C - 1) * L + i) * D + dfull] = acc;
  }
}

unsigned blocks_for(long total) {
  long b = (total + 255) / 256;
  return (unsigned)(b > 16384 ? 16384 : (b < 1 ? 1 : b));
}

size_t align_up(size_t x) { return (x + 63) & ~(size_t)63; }   // in floats: keeps 256-byte alignment

struct AttnLayout {
  size_t rmid, rhalf, rslack, coef_qk, lqs, cst_qk, sS, sR, lp, slack_p, coef_pv, cst_pv, total;
  AttnLayout(int B, int L, int H, int D, int P, bool own_scores) {
    const size_t bld = (size_t)B * L * D, C = (size_t)P * D + 1;
    size_t o = 0;
    auto take = [&](size_t n) { size_t r = o; o += align_up(n); return r; };
    rmid = take(3 * bld); rhalf = take(3 * bld); rslack = take(3 * bld);
    coef_qk = take(4 * bld); lqs = take(2 * bld); cst_qk = take((size_t)2 * B * H * L * L);
    lp = take((size_t)B * H * L * L); slack_p = take((size_t)B * H * L * L);
    coef_pv = take(4 * bld); cst_pv = take(2 * bld);
    const size_t plane = (size_t)B * H * C * L * L;
    sS = take(own_scores ? plane : 0); sR = take(own_scores ? plane : 0);
    total = o;
  }
};

}  // namespace

size_t attention_workspace_ext(int B, int L, int H, int D, int P, bool own_scores) {
  return AttnLayout(B, L, H, D, P, own_scores).total * sizeof(float);
}

int attention(CState q, CState k, CState v, int ld, int B, int L, int H, int D, int P, int pn, const float *eps, State o,
              State s, int stop_after, int32_t *status, void *ws, size_t ws_bytes, hipStream_t st) {
  TV_REQUIRE(q.S && q.R && k.S && k.R && v.S && v.R && eps && status && ws, TV_E_NULL, "attention: null pointer");
  TV_REQUIRE(B > 0 && L > 0 && H > 0 && D > 0 && P >= 0 && D % H == 0 && (D / H) % 4 == 0 && L % 4 == 0, TV_E_SHAPE,
             "attention: need D %% H == 0, head width and L multiples of 4 (B=%d L=%d H=%d D=%d)", B, L, H, D);
  TV_REQUIRE(norm_ok(pn), TV_E_NORM, "p_norm must be 1, 2 or TV_NORM_INF, got %d", pn);
  TV_REQUIRE(stop_after >= 0 && stop_after <= 2, TV_E_ARG, "stop_after must be 0, 1 or 2");
  TV_REQUIRE(stop_after == 0 ? (o.S && o.R) : (s.S && s.R), TV_E_NULL, "attention: null output state");
  TV_REQUIRE(ld >= D && ld % 4 == 0, TV_E_SHAPE, "attention: bad row stride %d", ld);
  const bool own = !(s.S && s.R);
  const AttnLayout lay(B, L, H, D, P, own);
  TV_REQUIRE(ws_bytes >= lay.total * sizeof(float), TV_E_WORKSPACE, "attention: workspace %zu < %zu bytes", ws_bytes,
             lay.total * sizeof(float));
  float *w = static_cast<float *>(ws);
  const int dh = D / H, C = P * D + 1;
  const float scale = 1.0f / sqrtf((float)dh);
  if (own) { s.S = w + lay.sS; s.R = w + lay.sR; }
  const long bld = (long)B * L * D;

  // concretized ranges of q, k, v as (mid, half) and, for q, the slack to its lower bound
  Ranges rg;
  float *rm = w + lay.rmid, *rh = w + lay.rhalf, *rs = w + lay.rslack;
  const bool fused = ld == 3 * D && k.S == q.S + D && v.S == q.S + 2 * D && k.R == q.R + D && v.R == q.R + 2 * D;
  if (fused) {
    if (int rc = concretize(q, B, P, D, L, ld, 1, pn, eps, rm, rh, rs, 1, st)) return rc;
    rg = Ranges{rm, rh, rs, rm + D, rh + D, rm + 2 * D, rh + 2 * D, ld};
  } else {
    TV_REQUIRE(ld == D, TV_E_SHAPE, "attention: separate q, k, v states must be densely packed");
    if (int rc = concretize(q, B, P, D, L, D, 1, pn, eps, rm, rh, rs, 1, st)) return rc;
    if (int rc = concretize(k, B, P, D, L, D, 1, pn, eps, rm + bld, rh + bld, nullptr, 1, st)) return rc;
    if (int rc = concretize(v, B, P, D, L, D, 1, pn, eps, rm + 2 * bld, rh + 2 * bld, nullptr, 1, st)) return rc;
    rg = Ranges{rm, rh, rs, rm + bld, rh + bld, rm + 2 * bld, rh + 2 * bld, D};
  }
  {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(qk_prep_kernel, dim3(blocks_for(bld)), dim3(256), 0, st, rg, B, L, H, dh, scale,
                       w + lay.coef_qk, w + lay.lqs);
    hipLaunchKernelGGL(qk_const_kernel, dim3(blocks_for((long)B * H * L * L)), dim3(256), 0, st, rg, B, L, H, dh, scale,
                       w + lay.cst_qk);
  }
  TV_HIP(hipGetLastError());

  const long cll = (long)C * L * L, clx = (long)C * L * ld, cld = (long)C * L * D;   // per-group plane sizes
  {  // scores, part 1: [S_q | R_q] x coefficients from k's range  -> both planes of s
    GemmArgs g;
    g.A = q.S; g.A2 = q.R; g.K1 = dh; g.lda = ld;
    g.B = w + lay.coef_qk; g.ldb = 2 * dh; g.b_mode = 0;
    g.C = s.S; g.ldc = L;
    g.bias = w + lay.cst_qk; g.bias_ld = L; g.bias_T = L; g.bias_C = C;
    g.M = C * L; g.N = L; g.K = 2 * dh;
    g.nz0 = 2; g.nz1 = H; g.nz2 = B; g.kind = K_QK_X;
    g.sA[0] = 0; g.sA[1] = dh; g.sA[2] = clx;
    g.sA2[0] = 0; g.sA2[1] = dh; g.sA2[2] = clx;
    g.sB[0] = (long)L * 2 * dh; g.sB[1] = 2L * L * 2 * dh; g.sB[2] = (long)H * 2 * L * 2 * dh;
    g.sC[0] = s.R - s.S; g.sC[1] = cll; g.sC[2] = (long)H * cll;
    g.sBias[0] = (long)L * L; g.sBias[1] = 2L * L * L; g.sBias[2] = (long)H * 2 * L * L;
    if (int rc = gemm(g, st)) return rc;
  }
  {  // scores, part 2: coefficients from q's range x the state of k, accumulated.  n = (r, j)
    GemmArgs g;
    g.A = w + lay.lqs; g.lda = D;
    g.B = k.S; g.ldb = ld; g.b_mode = 0;
    g.C = s.S; g.Cadd = s.S; g.ldc = L; g.cq = L; g.cstride = (long)L * L;
    g.M = L; g.N = C * L; g.K = dh;
    g.nz0 = 2; g.nz1 = H; g.nz2 = B; g.kind = K_QK_Y;
    g.sA[0] = bld; g.sA[1] = dh; g.sA[2] = (long)L * D;
    g.sB[0] = k.R - k.S; g.sB[1] = dh; g.sB[2] = clx;
    g.sC[0] = s.R - s.S; g.sC[1] = cll; g.sC[2] = (long)H * cll;
    g.sAdd[0] = g.sC[0]; g.sAdd[1] = g.sC[1]; g.sAdd[2] = g.sC[2];
    if (int rc = gemm(g, st)) return rc;
  }
  {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(qk_fix_kernel, dim3(blocks_for((long)B * H * L * L)), dim3(256), 0, st, rg, q.R, k.R, ld, B, L, H,
                       dh, C, scale, s.R);
  }
  TV_HIP(hipGetLastError());
  if (stop_after == 1) return TV_OK;

  float *lp = w + lay.lp, *slp = w + lay.slack_p;
  if (int rc = softmax(s, B * H, P, D, L, L, H, pn, eps, lp, slp, status, st)) return rc;
  if (stop_after == 2) return TV_OK;

  {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(pv_prep_kernel, dim3(blocks_for(bld)), dim3(256), 0, st, rg, B, L, H, dh, w + lay.coef_pv);
    hipLaunchKernelGGL(pv_const_kernel, dim3(blocks_for(bld)), dim3(256), 0, st, rg, lp, B, L, H, dh, w + lay.cst_pv);
  }
  TV_HIP(hipGetLastError());
  {  // o, part 1: [S_p | R_p] x coefficients from v's range
    GemmArgs g;
    g.A = s.S; g.A2 = s.R; g.K1 = L; g.lda = L;
    g.B = w + lay.coef_pv; g.ldb = 2 * L; g.b_mode = 0;
    g.C = o.S; g.ldc = D;
    g.bias = w + lay.cst_pv; g.bias_ld = D; g.bias_T = L; g.bias_C = C;
    g.M = C * L; g.N = dh; g.K = 2 * L;
    g.nz0 = 2; g.nz1 = H; g.nz2 = B; g.kind = K_PV_X;
    g.sA[0] = 0; g.sA[1] = cll; g.sA[2] = (long)H * cll;
    g.sA2[0] = 0; g.sA2[1] = cll; g.sA2[2] = (long)H * cll;
    g.sB[0] = (long)dh * 2 * L; g.sB[1] = 2L * dh * 2 * L; g.sB[2] = (long)H * 2 * dh * 2 * L;
    g.sC[0] = o.R - o.S; g.sC[1] = dh; g.sC[2] = cld;
    g.sBias[0] = bld; g.sBias[1] = dh; g.sBias[2] = (long)L * D;
    if (int rc = gemm(g, st)) return rc;
  }
  {  // o, part 2: lp x the state of v, accumulated (lp >= 0 after the clamp, so |lp| = lp).  n = (r, d)
    GemmArgs g;
    g.A = lp; g.lda = L;
    g.B = v.S; g.ldb = ld; g.b_mode = 1; g.cq = dh; g.b_cstride = (long)L * ld;
    g.C = o.S; g.Cadd = o.S; g.ldc = D; g.cstride = (long)L * D;
    g.M = L; g.N = C * dh; g.K = L;
    g.nz0 = 2; g.nz1 = H; g.nz2 = B; g.kind = K_PV_Y;
    g.sA[0] = 0; g.sA[1] = (long)L * L; g.sA[2] = (long)H * L * L;
    g.sB[0] = v.R - v.S; g.sB[1] = dh; g.sB[2] = clx;
    g.sC[0] = o.R - o.S; g.sC[1] = dh; g.sC[2] = cld;
    g.sAdd[0] = g.sC[0]; g.sAdd[1] = g.sC[1]; g.sAdd[2] = g.sC[2];
    if (int rc = gemm(g, st)) return rc;
  }
  {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(pv_fix_kernel, dim3(blocks_for(bld)), dim3(256), 0, st, rg, lp, slp, s.R, v.R, ld, B, L, H, dh, C,
                       o.R);
  }
  TV_HIP(hipGetLastError());
  return TV_OK;
}

}  // namespace tv
