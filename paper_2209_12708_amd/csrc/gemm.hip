// Batched fp32 GEMM on the CDNA matrix cores (v_mfma_f32_32x32x2_f32), the contraction behind the
// affine bound of Eq. (2) and the dot-product bounds.
//
// In centre/radius form the sign-split rule of Eq. (2) is two plain products, S_y = S_x W^T and
// R_y = R_x |W|^T: the paper's "weight pairing" (W+ + W- = W, Sec. 3.1) taken one step further, so
// that the multiply-add count equals the algorithmic one instead of twice that.  The same kernel,
// with a two-segment A operand ([S | R] concatenated along K) and index remaps on B / C, serves the
// four contractions of the two dot-product bounds.
//
// Tiling: a workgroup of 4 waves owns a BM x BN tile of C; K advances in steps of 32 staged through
// LDS (one stage; the next stage is prefetched into registers while the matrix cores run).  Each
// wave owns (BM/WM) x (BN/WN) as 32x32 MFMA tiles.  LDS rows are padded to 36 floats so that the
// 128-bit fragment reads of 16 consecutive rows hit 16 distinct bank groups.
#include <stdlib.h>
#include "common.h"

namespace tv {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));


__device__ __forceinline__ long remap_col(int n, int cq, long cstride) {
  return cq ? (long)(n / cq) * cstride + (n % cq) : (long)n;
}

template <int BM, int BN, int WM, int WN, int BMODE, int BK, bool DUAL>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs g, int mtiles, int ntiles) {
  constexpr int LS = BK + 4;              // padded LDS row length (floats) for [row][k] tiles
  constexpr int KQ = BK / 4;              // float4 groups per row of a stage
  constexpr int HK = BK / 2;              // k values per lane half
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_F4 = BM * KQ / 256 > 0 ? BM * KQ / 256 : 1;
  constexpr int B_F4 = BN * KQ / 256 > 0 ? BN * KQ / 256 : 1;
  constexpr int B1_HALF = HK * BN + 32;   // mode 1: floats per half of the stage, second half shifted by 32 banks
  constexpr int A_LDS = BM * LS;
  constexpr int B_LDS = BMODE == 0 ? BN * LS : 2 * B1_HALF;
  __shared__ __attribute__((aligned(16))) float lds[A_LDS + B_LDS];
  float *As = lds, *Bs = lds + A_LDS;

  // ---- XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs; give every XCD its
  // own M tiles and let consecutive ids on one XCD sweep the N tiles of the same M tile, so the A
  // rows are fetched into one L2 only.
  const int wid = blockIdx.x;
  int mt, nt;
  if (mtiles >= 8) {
    const int xcd = wid & 7, slot = wid >> 3;
    nt = slot % ntiles;
    mt = (slot / ntiles) * 8 + xcd;
    if (mt >= mtiles) return;
  } else {            // few M tiles (per-batch contractions over tokens): no padding of the grid
    mt = wid % mtiles;
    nt = wid / mtiles;
  }
  const int m0 = mt * BM, n0 = nt * BN;

  int z = blockIdx.y;
  const int z0 = z % g.nz0; z /= g.nz0;
  const int z1 = z % g.nz1; const int z2 = z / g.nz1;
  const float *A = g.A + z0 * g.sA[0] + z1 * g.sA[1] + z2 * g.sA[2];
  const float *A2 = g.A2 ? g.A2 + z0 * g.sA2[0] + z1 * g.sA2[1] + z2 * g.sA2[2] : nullptr;
  const float *B = g.B + z0 * g.sB[0] + z1 * g.sB[1] + z2 * g.sB[2];
  float *C = g.C + z0 * g.sC[0] + z1 * g.sC[1] + z2 * g.sC[2];
  const float *Cadd = g.Cadd ? g.Cadd + z0 * g.sAdd[0] + z1 * g.sAdd[1] + z2 * g.sAdd[2] : nullptr;
  const float *bias = g.bias ? g.bias + z0 * g.sBias[0] + z1 * g.sBias[1] + z2 * g.sBias[2] : nullptr;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int M = g.M, N = g.N, K = g.K, K1 = g.K1;

  // ---- per-thread global load slots (fixed rows / columns for the whole K loop)
  const float *a_ptr[A_F4]; const float *a2_ptr[A_F4]; int a_k[A_F4]; int a_lds[A_F4]; bool a_on[A_F4];
#pragma unroll
  for (int i = 0; i < A_F4; ++i) {
    const int f = tid + 256 * i;
    const int row = f / KQ, kq = f % KQ;
    a_on[i] = row < BM;
    int m = m0 + row; if (m >= M) m = M - 1;
    a_ptr[i] = A + (long)m * g.lda;
    a2_ptr[i] = A2 ? A2 + (long)m * g.lda : nullptr;
    a_k[i] = kq * 4;
    a_lds[i] = row * LS + kq * 4;
  }
  const float *b_ptr[B_F4]; int b_k[B_F4]; int b_lds[B_F4]; bool b_on[B_F4];
#pragma unroll
  for (int i = 0; i < B_F4; ++i) {
    const int f = tid + 256 * i;
    if (BMODE == 0) {
      const int row = f / KQ, kq = f % KQ;
      b_on[i] = row < BN;
      int n = n0 + row; if (n >= N) n = N - 1;
      b_ptr[i] = B + (long)n * g.ldb;
      b_k[i] = kq * 4;
      b_lds[i] = row * LS + kq * 4;
    } else {
      constexpr int NQ = BN / 4;
      const int k = f / NQ, nq = f % NQ;
      b_on[i] = k < BK;
      int n = n0 + nq * 4; if (n >= N) n = N - 4;
      b_ptr[i] = B + remap_col(n, g.cq, g.b_cstride);
      b_k[i] = k;
      b_lds[i] = (k / HK) * B1_HALF + (k % HK) * BN + nq * 4;
    }
  }

  float4 ra[A_F4], rb[B_F4];
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_F4; ++i) {
      const int k = k0 + a_k[i];
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (a_on[i] && k < K) {
        const float *p = (k < K1) ? a_ptr[i] + k : a2_ptr[i] + (k - K1);
        v = *reinterpret_cast<const float4 *>(p);
      }
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < B_F4; ++i) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (BMODE == 0) {
        const int k = k0 + b_k[i];
        if (b_on[i] && k < K) v = *reinterpret_cast<const float4 *>(b_ptr[i] + k);
      } else {
        const int k = k0 + b_k[i];
        if (b_on[i] && k < K) v = *reinterpret_cast<const float4 *>(b_ptr[i] + (long)k * g.ldb);
      }
      rb[i] = v;
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < A_F4; ++i)
      if (a_on[i]) *reinterpret_cast<float4 *>(As + a_lds[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_F4; ++i)
      if (b_on[i]) *reinterpret_cast<float4 *>(Bs + b_lds[i]) = rb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int l32 = lane & 31, half = lane >> 5;
  const int KT = (K + BK - 1) / BK;
  load_tile(0);
  store_tile();
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    if (kt + 1 < KT) load_tile((kt + 1) * BK);
    // MFMA step s multiplies k = s (lanes 0-31) and k = BK/2 + s (lanes 32-63) of this stage
#pragma unroll
    for (int hs = 0; hs < HK / 8; ++hs) {
      float4 af[TM][2], bf[TN][2];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const float *p = As + (wm * (BM / WM) + i * 32 + l32) * LS + half * HK + hs * 8;
        af[i][0] = *reinterpret_cast<const float4 *>(p);
        af[i][1] = *reinterpret_cast<const float4 *>(p + 4);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = wn * (BN / WN) + j * 32 + l32;
        if (BMODE == 0) {
          const float *p = Bs + col * LS + half * HK + hs * 8;
          bf[j][0] = *reinterpret_cast<const float4 *>(p);
          bf[j][1] = *reinterpret_cast<const float4 *>(p + 4);
        } else {
          const float *p = Bs + half * B1_HALF + (hs * 8) * BN + col;
          bf[j][0] = make_float4(p[0], p[BN], p[2 * BN], p[3 * BN]);
          bf[j][1] = make_float4(p[4 * BN], p[5 * BN], p[6 * BN], p[7 * BN]);
        }
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const float a = reinterpret_cast<const float *>(&af[i][0])[s];
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const float b = reinterpret_cast<const float *>(&bf[j][0])[s];
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i][j], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();
    if (kt + 1 < KT) {
      store_tile();
      __syncthreads();
    }
  }

  // ---- second product (see GemmArgs): both operands go from memory to fragments.  Lane half h of MFMA step s
  // holds k = c + 16 h + s of the 32-wide chunk c, a contiguous run of 16 floats per lane in the k-contiguous layouts.
  if (DUAL) {
    const float *pA = g.pA + z0 * g.spA[0] + z1 * g.spA[1] + z2 * g.spA[2];
    const float *pB = g.pB + z0 * g.spB[0] + z1 * g.spB[1] + z2 * g.spB[2];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row0 = m0 + wm * (BM / WM) + i * 32;
      if (row0 >= M) continue;                                   // wave-uniform
      const int r = row0 / g.pL, i0 = row0 % g.pL;
      const float *pa = pA + (long)(i0 + l32) * g.pA_ld + 16 * half;
      for (int c = 0; c < g.pK; c += 32) {
        float a2[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 v = *reinterpret_cast<const float4 *>(pa + c + 4 * q);
          a2[4 * q] = v.x; a2[4 * q + 1] = v.y; a2[4 * q + 2] = v.z; a2[4 * q + 3] = v.w;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          int n = n0 + wn * (BN / WN) + j * 32 + l32;
          if (n >= N) n = N - 1;                                 // loaded, never stored
          float b2[16];
          if (g.pB_mode == 0) {
            const float *pb = pB + ((long)r * g.pL + n) * g.pB_ld + c + 16 * half;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float4 v = *reinterpret_cast<const float4 *>(pb + 4 * q);
              b2[4 * q] = v.x; b2[4 * q + 1] = v.y; b2[4 * q + 2] = v.z; b2[4 * q + 3] = v.w;
            }
          } else {
            const float *pb = pB + ((long)r * g.pL + c + 16 * half) * g.pB_ld + n;
#pragma unroll
            for (int q = 0; q < 16; ++q) b2[q] = pb[(long)q * g.pB_ld];
          }
#pragma unroll
          for (int q = 0; q < 16; ++q) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[q], b2[q], acc[i][j], 0, 0, 0);
        }
      }
    }
  }

  // ---- epilogue.  Accumulator v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
  // does this tile contain rows of a bias block at all?  (one scalar test; 1 in C row blocks does)
  bool tile_has_bias = false;
  if (bias) {
    const int ba = m0 / g.bias_T, bb = (min(m0 + BM, M) - 1) / g.bias_T;
    tile_has_bias = (ba % g.bias_C) + (bb - ba) >= g.bias_C - 1;
  }
  long col[TN]; bool con[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn * (BN / WN) + j * 32 + l32;
    con[j] = n < N;
    col[j] = remap_col(con[j] ? n : 0, g.cq, g.cstride);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int mb = m0 + wm * (BM / WM) + i * 32 + 4 * half;
    if (Cadd) {     // residual / accumulate: issue all the loads of this 32-row tile before using them
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float add[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = mb + 8 * (v >> 2) + (v & 3);
          add[v] = (m < M && con[j]) ? Cadd[(long)m * g.ldc + col[j]] : 0.f;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] += add[v];
      }
    }
    if (tile_has_bias) {   // uniform branch: the plain store loop below never waits on a load
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = mb + 8 * (v >> 2) + (v & 3);
        // rows are ordered (group, coefficient row, t); the last coefficient row is the bias row
        const int blk = m / g.bias_T;
        if (m < M && blk % g.bias_C == g.bias_C - 1) {
          const float *brow = bias + ((long)(blk / g.bias_C) * g.bias_T + m % g.bias_T) * g.bias_ld;
#pragma unroll
          for (int j = 0; j < TN; ++j)
            if (con[j]) acc[i][j][v] += brow[col[j]];
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = mb + 8 * (v >> 2) + (v & 3);
      if (m >= M) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
        if (con[j]) C[(long)m * g.ldc + col[j]] = acc[i][j][v];
    }
  }
}

template <int BM, int BN, int WM, int WN, int BK = 32>
int launch(const GemmArgs &g, hipStream_t st) {
  const int mtiles = (g.M + BM - 1) / BM, ntiles = (g.N + BN - 1) / BN;
  const long groups = mtiles >= 8 ? (long)((mtiles + 7) / 8) * 8 * ntiles : (long)mtiles * ntiles;
  const long nz = (long)g.nz0 * g.nz1 * g.nz2;
  TV_REQUIRE(groups < (1L << 31) && nz <= 65535L * 32768L, TV_E_SHAPE, "gemm: grid too large");
  dim3 grid((unsigned)groups, (unsigned)nz, 1), block(256, 1, 1);
  if (g.pA) {
    if (g.b_mode == 0)
      hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, 0, BK, true>), grid, block, 0, st, g, mtiles, ntiles);
    else
      hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, 1, BK, true>), grid, block, 0, st, g, mtiles, ntiles);
  } else if (g.b_mode == 0)
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, 0, BK, false>), grid, block, 0, st, g, mtiles, ntiles);
  else
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, 1, BK, false>), grid, block, 0, st, g, mtiles, ntiles);
  TV_HIP(hipGetLastError());
  return TV_OK;
}

}  // namespace

int gemm(const GemmArgs &g, hipStream_t st) {
  TV_REQUIRE(g.A && g.B && g.C, TV_E_NULL, "gemm: null operand");
  TV_REQUIRE(g.M > 0 && g.N > 0 && g.K > 0, TV_E_SHAPE, "gemm: empty problem %d x %d x %d", g.M, g.N, g.K);
  TV_REQUIRE(g.K % 4 == 0 && g.lda % 4 == 0 && g.ldb % 4 == 0, TV_E_SHAPE,
             "gemm: K, lda, ldb must be multiples of 4 (K=%d lda=%ld ldb=%ld)", g.K, g.lda, g.ldb);
  TV_REQUIRE(g.A2 ? (g.K1 % 4 == 0 && g.K1 > 0 && g.K1 < g.K) : true, TV_E_SHAPE, "gemm: bad K split");
  TV_REQUIRE(g.b_mode == 0 || (g.N % 4 == 0 && (g.cq == 0 || g.cq % 4 == 0)), TV_E_SHAPE,
             "gemm: column groups must be multiples of 4");
  TV_REQUIRE(g.bias == nullptr || (g.bias_T > 0 && g.bias_C > 0), TV_E_ARG, "gemm: bias without row structure");
  TV_REQUIRE(g.pA == nullptr || (g.pB && g.pL > 0 && g.pL % 32 == 0 && g.pK > 0 && g.pK % 32 == 0 && g.M % 32 == 0 &&
                                 g.pA_ld % 4 == 0 && g.pB_ld % 4 == 0 && (g.pB_mode == 0 || g.pB_mode == 1)),
             TV_E_SHAPE, "gemm: second product needs pL, pK, M multiples of 32 (pL=%d pK=%d M=%d)", g.pL, g.pK, g.M);
  GemmArgs a = g;
  if (!a.A2) a.K1 = a.K;
  const double nz = (double)g.nz0 * g.nz1 * g.nz2, mn = (double)g.M * g.N;
  const double k2 = g.pA ? g.pK : 0;      // the second product reads its y operand once: M / pL blocks of pL x pK
  ProfScope prof(g.kind, st, 2.0 * mn * (g.K + k2) * nz,
                 4.0 * nz * ((double)g.M * g.K + (double)g.N * g.K + mn * (g.Cadd ? 2.0 : 1.0) +
                             (g.pA ? (double)g.M * (g.pB_mode == 0 ? k2 * g.N / g.pL : (double)g.N * k2 / g.pL) : 0.0)));
  if (dual_split_fits(a)) return gemm_dual_split(a, st);
  TV_REQUIRE(a.fix == nullptr, TV_E_ARG, "gemm: bias-row replacement needs the split dual kernel");
  // tile shape by problem shape: small M (per-batch contractions over tokens) vs small N (head width)
  if (a.M <= 32) return launch<32, 128, 1, 4>(a, st);
  if (a.M <= 64) return launch<64, 128, 2, 2>(a, st);
  if (a.N <= 32) return launch<128, 32, 4, 1>(a, st);
  if (a.N <= 64) return launch<128, 64, 2, 2>(a, st);
  // short K: the smaller tile doubles the workgroups in flight, which hides the epilogue better (measured)
  if (a.K <= 256 && a.N % 128 == 0) return launch<64, 128, 2, 2>(a, st);
  return launch<128, 128, 2, 2>(a, st);
}

}  // namespace tv
