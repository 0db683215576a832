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
// as a difference of O(1) terms, which fp32 cannot hold, so the preparation kernels also form that one
// row from slacks and half-widths (no cancellation) and a copy puts it over the products' result.
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

// ---- preparation for q k^T, one kernel.  Elementwise part (grid-stride over [B][L][D]):
//   coef[b][h][plane][j][kk]   (kk < dh: on S_q ; kk >= dh: on R_q), from k's range
//   lqs[plane][b][i][D] = scale * {l_q, |l_q|}
// Tiled part, one 16 x 16 tile of (i, j) per workgroup and head, operands staged through LDS:
//   cst[b][h][plane][i][j] = -scale * sum_d l_q[i,d] * {mid_k, half_k}[j,d]          constants of the centre plane
//   fix[b][h][i][j] = scale * sum_d ( half_k[j,d] (S_q_b - l_q)[i,d] + (|u_k|+|l_k|)/2 [j,d] R_q_b[i,d]
//                                      + |l_q[i,d]| R_k_b[j,d] )
// fix is the bias row of the radius plane of the scores, formed from slacks and half-widths (no cancellation);
// it replaces what the MFMA products leave in that row.
constexpr int kTile = 16, kChunk = 32;

__global__ __launch_bounds__(256) void qk_pre_kernel(Ranges rg, const float *qR, const float *kR, int ld, int B, int L,
                                                     int H, int dh, int C, float scale, float *coef, float *lqs,
                                                     float *cst, float *fix) {
  const int D = H * dh;
  const long total = (long)B * L * D;
  const long nblk = (long)gridDim.x * gridDim.y * gridDim.z;
  const long bid = blockIdx.x + (long)gridDim.x * (blockIdx.y + (long)gridDim.y * blockIdx.z);
  for (long i = bid * 256 + threadIdx.x; i < total; i += nblk * 256) {
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

  __shared__ float qs[3][kTile][kChunk + 1];     // l_q, slack of q, R_q bias
  __shared__ float ks[4][kTile][kChunk + 1];     // mid_k, half_k, (|u_k|+|l_k|)/2, R_k bias
  const int tiles = (L + kTile - 1) / kTile;
  const int i0 = (blockIdx.x / tiles) * kTile, j0 = (blockIdx.x % tiles) * kTile;
  const int h = blockIdx.y, b = blockIdx.z;
  const int ti = threadIdx.x / kTile, tj = threadIdx.x % kTile;
  float s = 0.f, rr = 0.f, fx = 0.f;
  for (int d0 = 0; d0 < dh; d0 += kChunk) {
    for (int e = threadIdx.x; e < kTile * kChunk; e += 256) {
      const int r = e / kChunk, d = e % kChunk;
      const bool dok = d0 + d < dh;
      const int i = i0 + r, j = j0 + r;
      float lq = 0.f, sq = 0.f, qb = 0.f, mk = 0.f, hk = 0.f, sk = 0.f, kb = 0.f;
      if (dok && i < L) {
        const long o = ((long)b * L + i) * rg.rld + h * dh + d0 + d;
        lq = rg.mq[o] - rg.hq[o]; sq = rg.sq[o];
        qb = qR[(((long)b * C + C - 1) * L + i) * ld + h * dh + d0 + d];
      }
      if (dok && j < L) {
        const long o = ((long)b * L + j) * rg.rld + h * dh + d0 + d;
        mk = rg.mk[o]; hk = rg.hk[o];
        float dif;
        abs_parts(mk, hk, dif, sk);
        kb = kR[(((long)b * C + C - 1) * L + j) * ld + h * dh + d0 + d];
      }
      qs[0][r][d] = lq; qs[1][r][d] = sq; qs[2][r][d] = qb;
      ks[0][r][d] = mk; ks[1][r][d] = hk; ks[2][r][d] = sk; ks[3][r][d] = kb;
    }
    __syncthreads();
#pragma unroll 8
    for (int d = 0; d < kChunk; ++d) {
      const float lq = qs[0][ti][d], hk = ks[1][tj][d];
      s = fmaf(lq, ks[0][tj][d], s);
      rr = fmaf(lq, hk, rr);
      fx += hk * qs[1][ti][d] + ks[2][tj][d] * qs[2][ti][d] + fabsf(lq) * ks[3][tj][d];
    }
    __syncthreads();
  }
  const int i = i0 + ti, j = j0 + tj;
  if (i < L && j < L) {
    float *o = cst + (((long)b * H + h) * 2) * L * L + (long)i * L + j;
    o[0] = -scale * s;
    o[(long)L * L] = -scale * rr;
    fix[(((long)b * H + h) * L + i) * L + j] = scale * fx;
  }
}

// ---- preparation for p v, one kernel.  Elementwise part: coef[b][h][plane][d][kk] (kk < L: on S_p[.., j = kk];
// kk >= L: on R_p) from v's range.  Tiled part, one 16 x 16 tile of (i, dfull) per workgroup:
//   cst[plane][b][i][D] = - sum_j lp[b,h,i,j] * {mid_v, half_v}[b,j,dfull]
//   fix[b][i][D] = sum_j ( half_v[j,d] (S_p_b - l_p)[i,j] + (|u_v|+|l_v|)/2 [j,d] R_p_b[i,j] + l_p[i,j] R_v_b[j,d] )
__global__ __launch_bounds__(256) void pv_pre_kernel(Ranges rg, const float *lp, const float *slack_p, const float *pR,
                                                     const float *vR, int ld, int B, int L, int H, int dh, int C,
                                                     float *coef, float *cst, float *fix) {
  const int D = H * dh;
  const long total = (long)B * L * D;
  const long nblk = (long)gridDim.x * gridDim.y;
  const long bid = blockIdx.x + (long)gridDim.x * blockIdx.y;
  for (long i = bid * 256 + threadIdx.x; i < total; i += nblk * 256) {
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

  __shared__ float ps[3][kTile][kChunk + 1];     // l_p, slack of p, R_p bias          [i][j]
  __shared__ float vs[4][kChunk][kTile + 1];     // mid_v, half_v, (|u_v|+|l_v|)/2, R_v bias   [j][d]
  const int itiles = (L + kTile - 1) / kTile;
  const int i0 = (blockIdx.x % itiles) * kTile, d0 = (blockIdx.x / itiles) * kTile;   // d0 runs over the full width D
  const int b = blockIdx.y;
  const int ti = threadIdx.x / kTile, td = threadIdx.x % kTile;
  const int dcol = d0 + td;                       // this thread's output column
  const int hcol = dcol < D ? dcol / dh : 0;
  // the p-side operands depend on the head of the column: staged through LDS when the tile lies in one head
  const bool one_head = d0 / dh == (min(d0 + kTile, D) - 1) / dh;
  const int h0 = d0 / dh;
  float s = 0.f, rr = 0.f, fx = 0.f;
  for (int j0 = 0; j0 < L; j0 += kChunk) {
    for (int e = threadIdx.x; e < kChunk * kTile; e += 256) {
      const int jj = e / kTile, dd = e % kTile;
      const int j = j0 + jj, dc = d0 + dd;
      float mv = 0.f, hv = 0.f, sv = 0.f, vb = 0.f;
      if (j < L && dc < D) {
        const long o = ((long)b * L + j) * rg.rld + dc;
        mv = rg.mv[o]; hv = rg.hv[o];
        float dif;
        abs_parts(mv, hv, dif, sv);
        vb = vR[(((long)b * C + C - 1) * L + j) * ld + dc];
      }
      vs[0][jj][dd] = mv; vs[1][jj][dd] = hv; vs[2][jj][dd] = sv; vs[3][jj][dd] = vb;
    }
    if (one_head) {
      for (int e = threadIdx.x; e < kTile * kChunk; e += 256) {
        const int r = e / kChunk, jj = e % kChunk;
        const int i = i0 + r, j = j0 + jj;
        float a = 0.f, sl = 0.f, pb = 0.f;
        if (i < L && j < L) {
          const long op = (((long)b * H + h0) * L + i) * L + j;
          a = lp[op]; sl = slack_p[op];
          pb = pR[((((long)b * H + h0) * C + C - 1) * L + i) * L + j];
        }
        ps[0][r][jj] = a; ps[1][r][jj] = sl; ps[2][r][jj] = pb;
      }
    }
    __syncthreads();
    const int i = i0 + ti;
    if (one_head) {
#pragma unroll 8
      for (int jj = 0; jj < kChunk; ++jj) {        // entries beyond L are zeros
        const float lpv = ps[0][ti][jj];
        s = fmaf(lpv, vs[0][jj][td], s);
        rr = fmaf(lpv, vs[1][jj][td], rr);
        fx += vs[1][jj][td] * ps[1][ti][jj] + vs[2][jj][td] * ps[2][ti][jj] + lpv * vs[3][jj][td];
      }
    } else if (i < L && dcol < D) {
      const long op = (((long)b * H + hcol) * L + i) * L;
      const float *pb = pR + ((((long)b * H + hcol) * C + C - 1) * L + i) * L;
      const int jn = min(kChunk, L - j0);
      for (int jj = 0; jj < jn; ++jj) {
        const float lpv = lp[op + j0 + jj];
        s = fmaf(lpv, vs[0][jj][td], s);
        rr = fmaf(lpv, vs[1][jj][td], rr);
        fx += vs[1][jj][td] * slack_p[op + j0 + jj] + vs[2][jj][td] * pb[j0 + jj] + lpv * vs[3][jj][td];
      }
    }
    __syncthreads();
  }
  const int i = i0 + ti;
  if (i < L && dcol < D) {
    const long t = ((long)b * L + i) * D + dcol;
    cst[t] = -s;
    cst[total + t] = -rr;
    fix[t] = fx;
  }
}

// dst[(g * C + C - 1) * X + x] = src[g * X + x]: puts recomputed bias rows into a state plane
__global__ void bias_row_put_kernel(const float *src, float *dst, long groups, int C, long X) {
  const long total = groups * X;
  for (long t = (long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long)gridDim.x * blockDim.x) {
    const long g = t / X, x = t % X;
    dst[(g * C + C - 1) * X + x] = src[t];
  }
}

unsigned blocks_for(long total) {
  long b = (total + 255) / 256;
  return (unsigned)(b > 16384 ? 16384 : (b < 1 ? 1 : b));
}

size_t align_up(size_t x) { return (x + 63) & ~(size_t)63; }   // in floats: keeps 256-byte alignment

struct AttnLayout {
  size_t rmid, rhalf, rslack, coef_qk, lqs, cst_qk, fix_qk, sS, sR, lp, slack_p, coef_pv, cst_pv, fix_pv, total;
  AttnLayout(int B, int L, int H, int D, int P, bool own_scores) {
    const size_t bld = (size_t)B * L * D, C = (size_t)P * D + 1;
    size_t o = 0;
    auto take = [&](size_t n) { size_t r = o; o += align_up(n); return r; };
    rmid = take(3 * bld); rhalf = take(3 * bld); rslack = take(3 * bld);
    coef_qk = take(4 * bld); lqs = take(2 * bld); cst_qk = take((size_t)2 * B * H * L * L);
    fix_qk = take((size_t)B * H * L * L);
    lp = take((size_t)B * H * L * L); slack_p = take((size_t)B * H * L * L);
    coef_pv = take(4 * bld); cst_pv = take(2 * bld); fix_pv = take(bld);
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
              State s, int stop_after, int32_t *status, void *ws, size_t ws_bytes, hipStream_t st,
              const float *qkv_norms, const int32_t *lengths) {
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
  TV_REQUIRE(qkv_norms == nullptr || fused, TV_E_ARG, "attention: stored norms need the fused q | k | v state");
  if (fused) {
    // qkv_norms: the eps-independent part of this concretization, stored by an earlier pass over the same state
    if (qkv_norms) { if (int rc = ranges_from_norms(qkv_norms, B, L, ld, 1, eps, rm, rh, rs, st)) return rc; }
    else if (int rc = concretize(q, B, P, D, L, ld, 1, pn, eps, rm, rh, rs, 1, st)) return rc;
    rg = Ranges{rm, rh, rs, rm + D, rh + D, rm + 2 * D, rh + 2 * D, ld};
  } else {
    TV_REQUIRE(ld == D, TV_E_SHAPE, "attention: separate q, k, v states must be densely packed");
    if (int rc = concretize(q, B, P, D, L, D, 1, pn, eps, rm, rh, rs, 1, st)) return rc;
    if (int rc = concretize(k, B, P, D, L, D, 1, pn, eps, rm + bld, rh + bld, nullptr, 1, st)) return rc;
    if (int rc = concretize(v, B, P, D, L, D, 1, pn, eps, rm + 2 * bld, rh + 2 * bld, nullptr, 1, st)) return rc;
    rg = Ranges{rm, rh, rs, rm + bld, rh + bld, rm + 2 * bld, rh + 2 * bld, D};
  }
  const int tiles = (L + kTile - 1) / kTile;
  {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(qk_pre_kernel, dim3(tiles * tiles, H, B), dim3(256), 0, st, rg, q.R, k.R, ld, B, L, H, dh, C, scale,
                       w + lay.coef_qk, w + lay.lqs, w + lay.cst_qk, w + lay.fix_qk);
  }
  TV_HIP(hipGetLastError());

  const long cll = (long)C * L * L, clx = (long)C * L * ld, cld = (long)C * L * D;   // per-group plane sizes
  // Both halves of a product in one launch (the half over y's state accumulated from fragments loaded straight
  // from memory) when the shapes allow; otherwise two launches, the second accumulating through memory.
  const bool fused_products = L % 32 == 0 && dh % 32 == 0;
  bool fix_qk_in_product = false, fix_pv_in_product = false;
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
    if (fused_products) {   // + sum_d lqs[i, d] * k-state[(r, j), d]
      g.pA = w + lay.lqs; g.pA_ld = D; g.pB = k.S; g.pB_ld = ld; g.pB_mode = 0; g.pL = L; g.pK = dh;
      g.spA[0] = bld; g.spA[1] = dh; g.spA[2] = (long)L * D;
      g.spB[0] = k.R - k.S; g.spB[1] = dh; g.spB[2] = clx;
    }
    if (dual_split_fits(g)) {   // that kernel also writes the radius plane's recomputed bias rows
      g.fix = w + lay.fix_qk; g.fix_ld = L; g.sFix[1] = (long)L * L; g.sFix[2] = (long)H * L * L;
      fix_qk_in_product = true;
    }
    if (int rc = gemm(g, st)) return rc;
  }
  if (!fused_products) {  // scores, part 2: coefficients from q's range x the state of k, accumulated.  n = (r, j)
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
  if (!fix_qk_in_product) {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(bias_row_put_kernel, dim3(blocks_for((long)B * H * L * L)), dim3(256), 0, st, w + lay.fix_qk, s.R,
                       (long)B * H, C, (long)L * L);
  }
  TV_HIP(hipGetLastError());
  if (stop_after == 1) return TV_OK;

  float *lp = w + lay.lp, *slp = w + lay.slack_p;
  // padded keys (sentences shorter than L): their score columns become a constant far below the row's maximum
  if (lengths)
    if (int rc = mask_scores(s, B * H, C, L, L, H, lengths, st)) return rc;
  if (int rc = softmax(s, B * H, P, D, L, L, H, pn, eps, lp, slp, status, st, lengths)) return rc;
  if (stop_after == 2) return TV_OK;

  {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(pv_pre_kernel, dim3(tiles * ((D + kTile - 1) / kTile), B), dim3(256), 0, st, rg, lp, slp, s.R, v.R, ld,
                       B, L, H, dh, C, w + lay.coef_pv, w + lay.cst_pv, w + lay.fix_pv);
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
    if (fused_products) {   // + sum_j lp[i, j] * v-state[(r, j), d]   (lp >= 0 after the clamp, so |lp| = lp)
      g.pA = lp; g.pA_ld = L; g.pB = v.S; g.pB_ld = ld; g.pB_mode = 1; g.pL = L; g.pK = L;
      g.spA[0] = 0; g.spA[1] = (long)L * L; g.spA[2] = (long)H * L * L;
      g.spB[0] = v.R - v.S; g.spB[1] = dh; g.spB[2] = clx;
    }
    if (dual_split_fits(g)) {
      g.fix = w + lay.fix_pv; g.fix_ld = D; g.sFix[1] = dh; g.sFix[2] = (long)L * D;
      fix_pv_in_product = true;
    }
    if (int rc = gemm(g, st)) return rc;
  }
  if (!fused_products) {  // o, part 2: lp x the state of v, accumulated.  n = (r, d)
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
  if (!fix_pv_in_product) {
    ProfScope prof(K_PREP, st, 0.0, 0.0);
    hipLaunchKernelGGL(bias_row_put_kernel, dim3(blocks_for(bld)), dim3(256), 0, st, w + lay.fix_pv, o.R, (long)B, C,
                       (long)L * D);
  }
  TV_HIP(hipGetLastError());
  return TV_OK;
}

}  // namespace tv
