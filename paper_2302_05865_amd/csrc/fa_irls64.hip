// K3 for 16 < p <= 64: the p x p part of the Flag Aggregator (normalisation, IRLS by repeated
// weighted PCA, coefficients) in one workgroup of sixteen wavefronts, every matrix product on
// the fp64 matrix core.
//
// Same mathematics as the p <= 16 fast path (fa_irls16.hip, namespace fastp; Eq. 5 with the
// regulariser of Sec. 2.3 option (2), Alg. 1's IRLS step and direction): R with R^T R = K~
// from a pivoted Cholesky factorisation, per solve M = R C R^T, the projector P onto the m
// leading eigenvectors of M by trace-correcting purification (X <- X^2 if trace X > m, else
// 2X - X^2, from X_0 = M / trace M), residuals from Z = (I - P) R, and at the end a basis of
// range(P) from a pivoted Cholesky of P.  What differs is the scale: matrices of order
// N = 16 T (T = 2, 3, 4) are kept in LDS as T x T tiles of 16 x 16, each tile in the register
// order of the matrix instruction's accumulator (entry r of lane l = element
// (4 r + l / 16, l % 16)), so that a wavefront moves a tile between LDS and registers with
// four conflict-free 8-byte accesses per lane and can use it directly
//   * as B operand (rows of the tile are the contraction index), and
//   * as A operand of the *transposed* tile (for a symmetric matrix: of tile (J, I)).
// One wavefront owns one output tile of a product; symmetric results are computed for I <= J
// and mirrored.  Steering of the purification: every wavefront publishes trace and squared
// Frobenius norm of its tile, all wavefronts add the published numbers in the same order
// after the step's barrier, so they take identical decisions.
//
// The same kernel has a mode for workers that send several gradients (blocks of columns, see
// MODE below); in that mode it is also built for a single tile (p <= 16).
//
// If the purification cannot converge (tied eigenvalues m, m+1) the kernel leaves
// info->status = FA_ST_RETRY and touches nothing else; the caller then runs the any-p Jacobi
// kernel, which starts from the same inputs.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fa.h"
#include "fa_internal.h"

namespace {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int NW = 16;                 // wavefronts in the workgroup
constexpr int NTHREADS = 64 * NW;
constexpr int MAX_PURIFY = 200;

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xf, 0xf, false);
  hi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}
template <int CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned x) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
// sum over each 16-lane row; every lane of the row gets it
__device__ __forceinline__ double row_sum(double x) {
  x += dpp_f64<0x128>(x);   // row_ror:8
  x += dpp_f64<0x124>(x);   // row_ror:4
  x += dpp_f64<0x122>(x);   // row_ror:2
  x += dpp_f64<0x121>(x);   // row_ror:1
  return x;
}
__device__ __forceinline__ double lane_bcast(double x, int srclane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(x), srclane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(x), srclane);
  return __hiloint2double(hi, lo);
}
// deterministic sum over the wavefront, same value in every lane
__device__ __forceinline__ double wave_sum(double x) {
  x = row_sum(x);
  return ((lane_bcast(x, 0) + lane_bcast(x, 16)) + lane_bcast(x, 32)) + lane_bcast(x, 48);
}
// 1/sqrt(x): hardware estimate plus two Newton steps
__device__ __forceinline__ double rsq2(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double hx = 0.5 * x;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const double e = fma(-hx * y, y, 0.5);
    y = fma(y, e, y);
  }
  return y;
}

// ---- tiles ---------------------------------------------------------------------------------
// A matrix is stored as T x T tiles of 16 x 16.  Lane l = 16 q + c of a wavefront holds rows
// 4e + q (e = 0..3), column c of a tile, as the matrix instruction delivers them; entry e of
// lane l sits at e * FA_ES + sw(l) doubles into the tile.  Both the lane-parallel access
// (fixed e) and the transposed store (lane (q, c), fixed source entry r, goes to entry c / 4,
// lane 16 (c % 4) + 4 r + q) then touch every LDS bank once per half wavefront: the entry
// stride 68 spreads the four destination entries over banks, and sw() moves the bit of c
// that would otherwise be lost into the bit that q leaves constant within a half wavefront.
constexpr int FA_ES = 68, FA_TILE = 272;
__device__ __forceinline__ int sw(int l) { return l ^ ((l >> 5) << 1); }
template <int T, typename P>
__device__ __forceinline__ v4d load_tile(P base, int I, int J, int lane) {
  const double* t = base + (I * T + J) * FA_TILE + sw(lane);
  return v4d{t[0], t[FA_ES], t[2 * FA_ES], t[3 * FA_ES]};
}
template <int T>
__device__ __forceinline__ void store_tile(double* base, int I, int J, int lane, const v4d& v) {
  double* t = base + (I * T + J) * FA_TILE + sw(lane);
  t[0] = v[0]; t[FA_ES] = v[1]; t[2 * FA_ES] = v[2]; t[3 * FA_ES] = v[3];
}
// the same values written as the transposed tile (J, I): element (4r + q, c) of (I, J) is
// element (c, 4r + q) of (J, I), i.e. entry c / 4 of lane 16 (c % 4) + 4r + q
template <int T>
__device__ __forceinline__ void store_tile_transposed(double* base, int I, int J, int lane,
                                                      const v4d& v) {
  const int c16 = lane & 15, q4 = lane >> 4;
  double* t = base + (J * T + I) * FA_TILE + (c16 >> 2) * FA_ES + sw((c16 & 3) * 16 + q4);
#pragma unroll
  for (int r = 0; r < 4; ++r) t[4 * r] = v[r];
}
// offset of element (i, j) in the tiled storage
template <int T>
__device__ __forceinline__ int eidx(int i, int j) {
  return ((i >> 4) * T + (j >> 4)) * FA_TILE + ((i & 15) >> 2) * FA_ES +
         sw((i & 3) * 16 + (j & 15));
}
// offset of element (a, j) of a matrix kept in A-operand order: tile (a/16, j/16), entry
// (j%16)/4 of lane ((j%16)%4) * 16 + a%16   [lane (i, k) supplies element (i, 4s + k)]
template <int T>
__device__ __forceinline__ int aidx(int a, int j) {
  return ((a >> 4) * T + (j >> 4)) * FA_TILE + ((j & 15) >> 2) * FA_ES +
         sw((j & 3) * 16 + (a & 15));
}
__device__ __forceinline__ v4d mma4(const v4d& a, const v4d& b, v4d acc) {
#pragma unroll
  for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s], b[s], acc, 0, 0, 0);
  return acc;
}
// the k-th pair (I <= J) of the upper triangle: the T diagonal tiles first (the wavefronts
// that start first hold them, one per SIMD), then the rest row by row
template <int T>
__device__ __forceinline__ void upper_pair(int k, int* I, int* J) {
  if (k < T) { *I = k; *J = k; return; }
  int i = 0, rem = k - T;
  while (rem >= T - 1 - i) { rem -= T - 1 - i; ++i; }
  *I = i; *J = i + 1 + rem;
}

struct Small {
  double s[64], dinv[64], w[64], wn[64], r1[64], beta[64], rinv[64], gd[64], rho[64];
  double dgx[2][64], dgy[2][64];   // [step parity]: diagonals of X_k and of X_k^2
  double red[NW];
  int piv[64], used[64];
  // workers that send several gradients: first column and width of the block a column is in,
  // 1 / tr(g^T g) of that block
  int gf[64], gc[64];
  double ginv[64];
  int dec[4];   // word of purification step g at [g & 3]: g << 4 | trace ok (4) | converged (2) | square (1)
  int flag[2];  // [step parity] a wavefront gave up waiting for that step's steering word
};

}  // namespace

// MODE 0: Eq. 5.  MODE 1: terms residual^(1/a) with the constant a of Sec. 2.2 Step 2 other than
// Eq. 5's a = 2 (a kernel of its own: the powers must not take registers from the a = 2 code).
// MODE 2: workers that send several gradients (Sec. 2.1; Sec. 2.2, the extension to
// g_i in R^{n x k}): the p columns are nworkers blocks of sizes[i] consecutive columns; a block's
// value is tr(g^T Y Y^T g) / tr(g^T g), the IRLS re-weights whole blocks, pair terms exist
// between blocks of equal width (Frobenius distance, column l against column l); any exponent.
template <int T, int MODE>
__global__ __launch_bounds__(NTHREADS) void fa_irls64_kernel(const double* __restrict__ Kg, int p,
                                                             int nworkers,
                                                             const int* __restrict__ sizes,
                                                             int m, int iters, double lambda,
                                                             double tol, double delta,
                                                             double expo,
                                                             double rank_tol, double pair_tol,
                                                             double* __restrict__ cg,
                                                             fa_info* __restrict__ info,
                                                             double* __restrict__ gws,
                                                             double* __restrict__ Ml,
                                                             int spin_budget, fa_resume* rs) {
  constexpr int N = 16 * T, TT = T * T, NTP = T * (T + 1) / 2, MSZ = TT * FA_TILE;
  constexpr int EPT = (N * N + NTHREADS - 1) / NTHREADS;   // matrix entries per thread
  extern __shared__ __attribute__((aligned(16))) double lds[];
  double* B0 = lds;
  double* B1 = lds + MSZ;
  double* B2 = lds + 2 * MSZ;
  double* RA = lds + 3 * MSZ;
  Small& sm = *reinterpret_cast<Small*>(lds + 4 * MSZ);
  double* Rb = gws;                 // R in tile order (B operand), global
  double* D2I = gws + MSZ;          // 1 / D_ij^2 in tile order, 0 for dropped pairs
  double* RtG = gws + 2 * MSZ;      // rows of the Cholesky factor of K~, row-major N x N
  // Ml: last weighted-PCA matrix, row-major N x N, then rank, m (for the eigengap diagnostic)

  const int tid = threadIdx.x, lane = tid & 63;
  // in a scalar register: everything decided per wavefront is a scalar branch
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c16 = lane & 15, q4 = lane >> 4;
  constexpr bool GEN = MODE != 0, GRP = MODE == 2;
  const int P = GRP ? nworkers : p;                       // workers
  const double coef = (lambda > 0.0 && P > 1) ? lambda / (double)(P - 1) : 0.0;
  const int it0 = rs ? rs->it0 : 0;
  const bool scaled = rs && rs->scaled;
  bool isdiag[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) isdiag[r] = (4 * r + q4) == c16;

  // ---- Gram, norms, status -----------------------------------------------------------------
  if (tid < 64) {
    double si = tid < p ? Kg[tid * p + tid] : 0.0;
    if (tid < p && scaled) si *= rs->uinv[tid] * rs->uinv[tid];
    sm.s[tid] = si;
    sm.dinv[tid] = si > 0.0 ? 1.0 / sqrt(si) : 0.0;
    sm.w[tid] = si > 0.0 ? 1.0 : 0.0;
    sm.used[tid] = 0;
    sm.rho[tid] = 0.0;
    if (tid < 4) sm.dec[tid] = 0;   // tag 0 is never used
  }
  __syncthreads();
  if constexpr (GRP) {
    if (tid < 64) {
      int first = tid, cnt = 1;
      if (tid < p) {
        int c = 0;
        for (int i = 0; i < nworkers; ++i) {
          const int k = sizes[i];
          if (tid < c + k) { first = c; cnt = k; break; }
          c += k;
        }
      }
      double gs = 0.0;
      for (int l = 0; l < cnt; ++l) gs += sm.s[first + l];
      sm.gf[tid] = first; sm.gc[tid] = cnt;
      sm.ginv[tid] = gs > 0.0 ? 1.0 / gs : 0.0;
      sm.w[tid] = gs > 0.0 ? 1.0 : 0.0;
    }
    __syncthreads();
  }
  bool bad = false, live = false;
#pragma unroll
  for (int q = 0; q < EPT; ++q) {
    const int e = tid + q * NTHREADS;
    if (e < N * N) {
      const int i = e / N, j = e - i * N;
      const bool in = i < p && j < p;
      double kv = in ? Kg[i * p + j] : 0.0;
      if (in && scaled) kv *= rs->uinv[i] * rs->uinv[j];
      if (in) info->K[i * p + j] = kv;
      bad = bad || !(fabs(kv) <= 1.79e308);
      const double si = sm.s[i], sj = sm.s[j];
      live = live || (i == j && si > 0.0);
      B0[e] = (i == j) ? (si > 0.0 ? 1.0 : 0.0) : kv * sm.dinv[i] * sm.dinv[j];   // K~, row-major
      double d2 = si + sj - 2.0 * kv;
      bool livep = in && i != j && d2 > pair_tol * (si + sj);
      if constexpr (GRP) {
        // D^2 between two blocks: column l of one against column l of the other; only blocks
        // of equal width have one, and it sits at the column pairs at the same place in them
        livep = false;
        if (in && i != j) {
          const int fi = sm.gf[i], fj = sm.gf[j], ki = sm.gc[i];
          if (fi != fj && ki == sm.gc[j] && i - fi == j - fj) {
            double ssum = 0.0;
            d2 = 0.0;
            for (int l = 0; l < ki; ++l) {
              const double sa = sm.s[fi + l], sb = sm.s[fj + l];
              d2 += sa + sb - 2.0 * Kg[(fi + l) * p + fj + l];
              ssum += sa + sb;
            }
            livep = d2 > pair_tol * ssum;
          }
        }
      }
      D2I[eidx<T>(i, j)] = livep ? 1.0 / d2 : 0.0;
    }
  }
  const int nbad = __syncthreads_or(bad ? 1 : 0);
  const int nlive = __syncthreads_or(live ? 1 : 0);
  if (nbad || !nlive) {
    const int st = nbad ? 4 : 5;
    if (tid < p) {
      const double cv = nbad ? nan("") : 0.0;
      cg[tid] = cv;
      info->c[tid] = cv; info->s[tid] = sm.s[tid]; info->v[tid] = 0.0; info->w[tid] = 0.0;
    }
    for (int idx = tid; idx < p * m; idx += NTHREADS) info->A[idx] = 0.0;
    if (tid == 0) {
      info->status = st; info->p = p; info->m = m; info->rank = 0; info->iters_done = 0;
      info->sweeps = 0; info->eigengap = 0.0;
    }
    return;
  }

  // ---- pivoted Cholesky of K~ (B0, row-major) -> rows in B1; right-looking: after a pivot
  // row is taken the whole remaining matrix is updated at once, by all threads ----------------
  auto pivoted_cholesky = [&](double* S, double* rows, double tolv, int max_rank) -> int {
    int rank = 0;
    for (int k = 0; k < max_rank; ++k) {
      // every wavefront finds the pivot for itself (same data, same answer): the largest
      // remaining diagonal entry as seen in fp32, ties to the lowest index
      const double d = (lane < N && !sm.used[lane]) ? S[lane * N + lane] : 0.0;
      const float df = d > 0.0 ? (float)d : 0.0f;
      unsigned key = (__float_as_uint(df) & ~63u) | (unsigned)(63 - lane);
      key = max(key, dpp_u32<0x128>(key));
      key = max(key, dpp_u32<0x124>(key));
      key = max(key, dpp_u32<0x122>(key));
      key = max(key, dpp_u32<0x121>(key));
      const unsigned k0 = (unsigned)__builtin_amdgcn_readlane((int)key, 0);
      const unsigned k1 = (unsigned)__builtin_amdgcn_readlane((int)key, 16);
      const unsigned k2 = (unsigned)__builtin_amdgcn_readlane((int)key, 32);
      const unsigned k3 = (unsigned)__builtin_amdgcn_readlane((int)key, 48);
      const unsigned kmax = max(max(k0, k1), max(k2, k3));
      const int pv = 63 - (int)(kmax & 63u);
      const double dp = (pv < N && !sm.used[pv]) ? S[pv * N + pv] : 0.0;
      if (!(dp > tolv)) break;                       // uniform: everyone read the same value
      const double rsv = rsq2(dp);
      double ai[EPT], aj[EPT];
#pragma unroll
      for (int q = 0; q < EPT; ++q) {
        const int e = tid + q * NTHREADS;
        const int i = e < N * N ? e / N : 0, j = e < N * N ? e - i * N : 0;
        ai[q] = S[pv * N + i] * rsv;
        aj[q] = S[pv * N + j] * rsv;
      }
      const double rk = (tid < N && !sm.used[tid]) ? S[pv * N + tid] * rsv : 0.0;
      __syncthreads();                               // row pv has been read by everyone
#pragma unroll
      for (int q = 0; q < EPT; ++q) {
        const int e = tid + q * NTHREADS;
        if (e < N * N) {
          const int i = e / N, j = e - i * N;
          const bool dead = i == pv || j == pv || sm.used[i] || sm.used[j];
          S[e] = dead ? 0.0 : fma(-ai[q], aj[q], S[e]);
        }
      }
      if (tid < N) rows[k * N + tid] = rk;
      __syncthreads();                               // used[] is read above, written below
      if (tid == 0) { sm.piv[k] = pv; sm.rinv[k] = rsv; sm.used[pv] = 1; }
      rank = k + 1;
      __syncthreads();
    }
    for (int e = tid; e < N * N; e += NTHREADS)
      if (e / N >= rank) rows[e] = 0.0;
    if (tid < N && tid >= rank) { sm.piv[tid] = 0; sm.rinv[tid] = 0.0; }
    __syncthreads();
    return rank;
  };
  const int rank = pivoted_cholesky(B0, B1, rank_tol, N);
  const int mm = m < rank ? m : rank;

  // ---- R = R~ D^1/2 in both operand orders; R 1; Cholesky rows kept for the epilogue --------
#pragma unroll
  for (int q = 0; q < EPT; ++q) {
    const int e = tid + q * NTHREADS;
    if (e < N * N) {
      const int a = e / N, j = e - a * N;
      const double rt = B1[e];
      const double rv = rt * sqrt(sm.s[j]);
      RA[aidx<T>(a, j)] = rv;
      Rb[eidx<T>(a, j)] = rv;
      RtG[e] = rt;
    }
  }
  if (tid < 64) sm.used[tid] = 0;   // the second factorisation (epilogue) starts afresh
  __syncthreads();
  {
    // R 1: sixteen threads per row
    const int a = tid >> 4, l16 = tid & 15;
    double acc = 0.0;
    if (a < N)
      for (int j = l16; j < N; j += 16) {
        const double x = RA[aidx<T>(a, j)];
        acc += GRP ? x / (double)sm.gc[j] : x;          // a block counts with its mean column
      }
    acc = row_sum(acc);
    if (a < N && l16 == 0) sm.r1[a] = acc;
  }
  // the Cholesky pivots are needed again in the epilogue
  int piv_keep = tid < 64 ? sm.piv[tid] : 0;
  double rinv_keep = tid < 64 ? sm.rinv[tid] : 0.0;

  // ---- pair part of C (B2, tile order): uniform weights, or what an earlier launch left ------
#pragma unroll
  for (int q = 0; q < EPT; ++q) {
    const int e = tid + q * NTHREADS;
    if (e < N * N) {
      const int i = e / N, j = e - i * N;
      double v = 0.0;
      if (i < p && j < p && i != j)
        v = it0 > 0 ? rs->cp[i * p + j] : -2.0 * coef * D2I[eidx<T>(i, j)];
      B2[eidx<T>(i, j)] = v;
    }
  }
  if (it0 > 0 && tid < p) sm.w[tid] = sm.s[tid] > 0.0 ? rs->w[tid] : 0.0;
  double prev_obj = it0 > 0 ? rs->prev_obj : 0.0;
  __syncthreads();

  // this wavefront's output tile in products with a full (wave < TT) or symmetric
  // (wave < NTP, I <= J) result
  const int fI = wave / T, fJ = wave % T;
  int uI = 0, uJ = 0;
  if (wave < NTP) upper_pair<T>(wave, &uI, &uJ);
  const double rs_delta = 1.0 / sqrt(delta);
  int iters_done = 0, steps = 0, gstep = 0;
  double* cur = B0;   // where the projector of the last solve is
  double* nxt = B1;
  int failed = 0;

  for (int it = 0; it < iters; ++it) {
    // ---- C: diagonal from the data weights and the row sums of the pair part ---------------
    {
      const int i = tid >> 4, l16 = tid & 15;
      double acc = 0.0;
      if (i < N)
        for (int j = l16; j < N; j += 16) acc += (j != i) ? B2[eidx<T>(i, j)] : 0.0;
      acc = row_sum(acc);
      __syncthreads();
      if (i < N && l16 == 0)
        B2[eidx<T>(i, i)] = sm.w[i] * (GRP ? sm.ginv[i] : sm.dinv[i] * sm.dinv[i]) - acc;
    }
    __syncthreads();
    // ---- W = C R^T (B1): A operand = C (symmetric: tile (K, I)), B operand = R^T tile (K, J),
    // which is R's tile (J, K) in A-operand order ---------------------------------------------
    if (wave < TT) {
      v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int K = 0; K < T; ++K)
        acc = mma4(load_tile<T>(B2, K, fI, lane), load_tile<T>(RA, fJ, K, lane), acc);
      store_tile<T>(B1, fI, fJ, lane, acc);
    }
    __syncthreads();
    // ---- M = R W (B0, both triangles), its trace ----------------------------------------------
    if (wave < NTP) {
      v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int K = 0; K < T; ++K)
        acc = mma4(load_tile<T>(RA, uI, K, lane), load_tile<T>(B1, K, uJ, lane), acc);
      store_tile<T>(B0, uI, uJ, lane, acc);
      if (uI != uJ) store_tile_transposed<T>(B0, uI, uJ, lane, acc);
      double td = 0.0;
      if (uI == uJ) {
#pragma unroll
        for (int r = 0; r < 4; ++r) td += isdiag[r] ? acc[r] : 0.0;
      }
      td = wave_sum(td);
      if (lane == 0) sm.red[wave] = td;
    }
    __syncthreads();
    double hi = 0.0;
#pragma unroll
    for (int k = 0; k < NTP; ++k) hi += sm.red[k];
    // the matrix itself, row-major, for the eigengap diagnostic
    if (wave < TT) {
      const v4d mt = load_tile<T>(B0, fI, fJ, lane);
#pragma unroll
      for (int r = 0; r < 4; ++r) Ml[(16 * fI + 4 * r + q4) * N + 16 * fJ + c16] = mt[r];
    }
    cur = B0; nxt = B1;
    if (mm < rank) {
      // ---- X_0 = M / trace(M) (slightly less: any scale with eigenvalues in [0, 1] will do)
      const double sc = __builtin_amdgcn_rcp(hi) * (1.0 - 1e-7);
      if (wave < TT) {
        v4d x = load_tile<T>(B0, fI, fJ, lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] *= sc;
        store_tile<T>(B0, fI, fJ, lane, x);
      }
      // ---- purification ---------------------------------------------------------------------
      // A wavefront's fp64 vector instructions do not get a turn while older wavefronts of
      // its SIMD have matrix instructions to issue, and every dependent LDS round trip or
      // cross-lane sum costs hundreds of cycles, so measuring and deciding stay off the
      // multiplying wavefronts' path:
      //  - wavefronts 0..NTP-1 multiply (one tile of X_k^2 each); those with a diagonal tile
      //    leave the diagonals of X_k and X_k^2 in LDS;
      //  - during step k wavefront NTP (on the SIMD with the fewest multiplying wavefronts)
      //    sums the diagonals left in step k-1 (trace(X_{k-1}), trace(X_{k-1}^2) =
      //    |X_{k-1}|_F^2) and publishes the word of step k: "X_{k-1} was a projector" (then
      //    X_k, its polished successor, is the result) and "square X_k", from trace(X_k) =
      //    |X_{k-1}|_F^2 after a squaring and 2 trace(X_{k-1}) - |X_{k-1}|_F^2 otherwise;
      //  - the multiplying wavefronts pick the word up after their products; everybody else
      //    reads it at the top of the next step, after the barrier.
      // Waits: the steering wavefront waits for nobody, so the readers' bounded spin ends.  One
      // that runs out of its budget of polls raises the step's flag, skips its store and goes
      // on to the step's barrier like everybody else; all read that flag right after the
      // barrier, at the top of the next step, and leave the loop together with the solve marked
      // as failed (the last step of the loop cannot raise it unseen: MAX_PURIFY is even and a
      // failed solve is what running out of steps means anyway).
      ++gstep;                        // a tag of its own between solves: no stale word matches
      bool sq_prev = hi * sc > (double)mm, conv = false;
      int wprev = 0;                  // the word of the previous step
      bool reread = wave > NTP;       // ... fetched from LDS by those who did not use it then
      if (tid == 0) { sm.flag[0] = 0; sm.flag[1] = 0; }
      __syncthreads();
      // One step: X_k in cu, X_{k+1} into nx.  Written for fixed buffers (the loop below
      // alternates two instances) so that every LDS address is loop invariant: a wavefront
      // that leaves the barrier behind older ones of its SIMD can put its loads in flight at
      // once, without a vector instruction that would wait for their products.
      // Returns false when the loop is over.
      auto step = [&](double* cu, double* nx, int k) __attribute__((always_inline)) -> bool {
        ++gstep;                      // tags the words: never repeats within a launch
        // the previous step's flag: raised before the last barrier, if at all, and written by
        // nobody in this step (which has the other one), so every wavefront reads the same
        if (k > 0 && __builtin_amdgcn_readfirstlane(sm.flag[(k - 1) & 1])) {
          conv = false;
          return false;
        }
        if (k > 0) {
          // in place since the last barrier: its publisher waits for nobody
          if (reread) wprev = __builtin_amdgcn_readfirstlane(sm.dec[(gstep - 1) & 3]);
          if (wprev & 2) {            // X_{k-1}, left alone in nx, is the result
            conv = (wprev & 4) != 0;
            cur = nx; nxt = cu;
            return false;
          }
        }
        if (wave < NTP) {
          // own tile (uI, uJ) of X_k^2 = sum_K X(K, uI)^T X(K, uJ); the operands of the
          // next K are on their way from LDS while this K is multiplied
          v4d y = {0.0, 0.0, 0.0, 0.0};
          v4d a = load_tile<T>(cu, 0, uI, lane), b = load_tile<T>(cu, 0, uJ, lane);
#pragma unroll
          for (int K = 0; K < T; ++K) {
            v4d an = a, bn = b;
            if (K + 1 < T) {
              an = load_tile<T>(cu, K + 1, uI, lane);
              bn = load_tile<T>(cu, K + 1, uJ, lane);
            } else {
              an = load_tile<T>(cu, uI, uJ, lane);       // the tile itself, for the update
            }
            __builtin_amdgcn_sched_barrier(0);           // keep those loads ahead of the products
            y = mma4(a, b, y);
            a = an; b = bn;
          }
          const v4d x = a;
          if (uI == uJ) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (isdiag[r]) {
                sm.dgx[k & 1][16 * uI + c16] = x[r];
                sm.dgy[k & 1][16 * uI + c16] = y[r];
              }
          }
          // this step's word (there already, as a rule)
          int word = 0;               // tag 0 is never used
          for (int tries = 0; (word >> 4) != gstep && tries < spin_budget; ++tries)
            word = __builtin_amdgcn_readfirstlane(__hip_atomic_load(
                &sm.dec[gstep & 3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
          const bool gave_up = (word >> 4) != gstep;
          if (gave_up) { sm.flag[k & 1] = 1; reread = true; }
          wprev = word;
          if (!gave_up && !(word & 2)) {
            v4d xn;
            if (word & 1) {
              xn = y;
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) xn[r] = fma(2.0, x[r], -y[r]);
            }
            store_tile<T>(nx, uI, uJ, lane, xn);
            if (uI != uJ) store_tile_transposed<T>(nx, uI, uJ, lane, xn);
          }
        } else if (wave == NTP) {
          int word = gstep << 4;
          if (k == 0) {
            word |= sq_prev ? 1 : 0;
          } else {
            // both sums in one pass: the lower half wavefront adds up one diagonal, the
            // upper half the other (entries N..63 are never written: masked)
            const double* dg = lane < 32 ? sm.dgx[(k - 1) & 1] : sm.dgy[(k - 1) & 1];
            const int l32 = lane & 31;
            const double d0 = l32 < N ? dg[l32] : 0.0, d1 = l32 + 32 < N ? dg[l32 + 32] : 0.0;
            const double hs = row_sum(d0 + d1);
            const double trx = lane_bcast(hs, 0) + lane_bcast(hs, 16);
            const double fro = lane_bcast(hs, 32) + lane_bcast(hs, 48);
            if (trx - fro < 1e-10) word |= 2 | (fabs(trx - (double)mm) < 0.25 ? 4 : 0);
            if ((sq_prev ? fro : fma(2.0, trx, -fro)) > (double)mm) word |= 1;
            sq_prev = (word & 1) != 0;
          }
          if (lane == 0) __hip_atomic_store(&sm.dec[gstep & 3], word, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_WORKGROUP);
          wprev = word;
        }
        steps = steps + 1;
        __syncthreads();
        return true;
      };
      for (int k = 0; k < MAX_PURIFY; k += 2)
        if (!step(B0, B1, k) || !step(B1, B0, k + 1)) break;
      if (!conv) { failed = 1; break; }
    } else {
      // m >= rank: Y spans all of span(G)
      if (wave < TT) {
        v4d x;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          x[r] = (fI == fJ && isdiag[r] && 16 * fI + c16 < rank) ? 1.0 : 0.0;
        store_tile<T>(cur, fI, fJ, lane, x);
      }
      __syncthreads();
    }
    // ---- Z = (I - P) R (nxt): A operand = I - P (symmetric), B operand = R from global -------
    if (wave < TT) {
      v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int K = 0; K < T; ++K) {
        v4d q = load_tile<T>(cur, K, fI, lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) q[r] = (K == fI && isdiag[r]) ? 1.0 - q[r] : -q[r];
        acc = mma4(q, load_tile<T>((const double*)Rb, K, fJ, lane), acc);
      }
      store_tile<T>(nxt, fI, fJ, lane, acc);
    }
    __syncthreads();
    // ---- Gq = Z^T Z (symmetric; tile (I, J) = sum_K Z(K, I)^T Z(K, J)); its diagonal ----------
    v4d gq = {0.0, 0.0, 0.0, 0.0};
    if (wave < NTP) {
#pragma unroll
      for (int K = 0; K < T; ++K)
        gq = mma4(load_tile<T>(nxt, K, uI, lane), load_tile<T>(nxt, K, uJ, lane), gq);
      if (uI == uJ) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (isdiag[r]) sm.gd[16 * uI + c16] = gq[r];
      }
    }
    __syncthreads();
    if constexpr (GRP) {
      // a block's residual adds entries of Gq that other wavefronts hold: all of it into LDS
      // (over Z, which nobody reads any more)
      if (wave < NTP) {
        store_tile<T>(nxt, uI, uJ, lane, gq);
        if (uI != uJ) store_tile_transposed<T>(nxt, uI, uJ, lane, gq);
      }
      __syncthreads();
    }
    // ---- residuals, objective, next weights (pair part straight into C = B2) -------------------
    double part = 0.0;
    if (wave < NTP) {
      v4d cpn;
      if constexpr (!GEN) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i = 16 * uI + 4 * r + q4, j = 16 * uJ + c16;
          double cv = 0.0;
          if (i == j) {
            // |(I - P) r_j|^2 / |g_j|^2 = 1 - v_j
            const double rho = gq[r] * sm.dinv[j] * sm.dinv[j];
            const bool livej = sm.s[j] > 0.0;
            const double rsj = rsq2(rho > 1e-300 ? rho : 1e-300);
            if (livej) part += rho * rsj;
            sm.rho[j] = rho;
            sm.wn[j] = livej ? (rsj < rs_delta ? rsj : rs_delta) : 0.0;
          } else {
            const double d2i = D2I[eidx<T>(i, j)];
            if (d2i > 0.0 && coef > 0.0) {
              double num = sm.gd[i] + sm.gd[j] - 2.0 * gq[r];
              num = num > 0.0 ? num : 0.0;
              const double rho = num * d2i;
              const double rsv = rsq2(rho > 1e-300 ? rho : 1e-300);
              // ordered pairs: an off-diagonal tile stands for its mirror image too
              part += (uI == uJ ? 1.0 : 2.0) * coef * (rho * rsv);
              cv = -2.0 * coef * d2i * (rsv < rs_delta ? rsv : rs_delta);
            }
          }
          cpn[r] = cv;
        }
      } else {
        // the general exponent: same places, powers instead of square roots (rolled: once per
        // solve, and inlined copies of pow() are long)
#pragma unroll 1
        for (int r = 0; r < 4; ++r) {
          const int i = 16 * uI + 4 * r + q4, j = 16 * uJ + c16;
          const double gqr = r == 0 ? gq[0] : r == 1 ? gq[1] : r == 2 ? gq[2] : gq[3];
          double rho = 0.0, scale = 0.0;       // residual; factor of its term in the objective
          bool diag = i == j, use = false;
          double d2i = 0.0;
          if constexpr (!GRP) {
            if (diag) {
              rho = gqr * sm.dinv[j] * sm.dinv[j];
              use = sm.s[j] > 0.0;
              scale = 1.0;
            } else {
              d2i = D2I[eidx<T>(i, j)];
              if (d2i > 0.0 && coef > 0.0) {
                double num = sm.gd[i] + sm.gd[j] - 2.0 * gqr;
                num = num > 0.0 ? num : 0.0;
                rho = num * d2i;
                use = true;
                scale = (uI == uJ ? 1.0 : 2.0) * coef;
              }
            }
          } else {
            // the block's numbers, the same at each of its columns; its term of the objective
            // is counted at its first column (pair terms: at the blocks' first columns)
            const int fi = sm.gf[i], fj = sm.gf[j], kj = sm.gc[j];
            if (diag) {
              double bot = 0.0;
              for (int l = 0; l < kj; ++l) bot += sm.gd[fj + l];
              rho = bot * sm.ginv[j];
              use = sm.ginv[j] > 0.0;
              scale = j == fj ? 1.0 : 0.0;
            } else {
              d2i = D2I[eidx<T>(i, j)];
              if (d2i > 0.0 && coef > 0.0) {
                double num = 0.0;
                for (int l = 0; l < kj; ++l)
                  num += sm.gd[fi + l] + sm.gd[fj + l] - 2.0 * nxt[eidx<T>(fi + l, fj + l)];
                num = num > 0.0 ? num : 0.0;
                rho = num * d2i;
                use = true;
                scale = i == fi ? (uI == uJ ? 1.0 : 2.0) * coef : 0.0;
              }
            }
          }
          const double tv = fa_term_pow(rho, expo), wv = fa_weight_pow(rho, delta, expo);
          if (use) part += scale * tv;
          if (diag) { sm.rho[j] = rho; sm.wn[j] = use ? wv : 0.0; }
          const double cv = (!diag && use) ? -2.0 * coef * d2i * wv : 0.0;
          if (r == 0) cpn[0] = cv; else if (r == 1) cpn[1] = cv; else if (r == 2) cpn[2] = cv; else cpn[3] = cv;
        }
      }
      store_tile<T>(B2, uI, uJ, lane, cpn);
      if (uI != uJ) store_tile_transposed<T>(B2, uI, uJ, lane, cpn);
      part = wave_sum(part);
      if (lane == 0) sm.red[wave] = part;
    }
    __syncthreads();
    double obj = 0.0;
#pragma unroll
    for (int k = 0; k < NTP; ++k) obj += sm.red[k];
    if (tid == 0 && it0 + it < FA_ITERS_MAX) info->objective[it0 + it] = obj;
    iters_done = it + 1;
    const bool stop = it0 + it > 0 && fabs(prev_obj - obj) < tol;
    prev_obj = obj;
    __syncthreads();   // red[] is reused by the next solve
    if (stop) break;
    if (tid < 64) sm.w[tid] = sm.wn[tid];
  }
  if (failed) {
    if (tid == 0) info->status = FA_ST_RETRY;
    return;
  }
  // ---- epilogue ----------------------------------------------------------------------------
  // P (cur, tile order) -> row-major copy in nxt, its pivoted Cholesky rows U_m -> RA's place
  double* Sp = nxt;
  double* Um = RA;      // R in A order is no longer needed
#pragma unroll
  for (int q = 0; q < EPT; ++q) {
    const int e = tid + q * NTHREADS;
    if (e < N * N) Sp[e] = cur[eidx<T>(e / N, e % N)];
  }
  __syncthreads();
  // pivots of the first factorisation survive in registers; the second one overwrites sm.piv
  const int nb = pivoted_cholesky(Sp, Um, 1e-6, mm);
  if (nb != mm) {
    if (tid == 0) info->status = FA_ST_RETRY;
    return;
  }
  // beta = U_m (R 1)   (U_m rows k, columns a)
  {
    const int k = tid >> 4, l16 = tid & 15;
    double acc = 0.0;
    if (k < N)
      for (int a = l16; a < N; a += 16) acc = fma(Um[k * N + a], sm.r1[a], acc);
    acc = row_sum(acc);
    if (k < N && l16 == 0) sm.beta[k] = k < mm ? acc : 0.0;
  }
  // restore the first factorisation's pivots and reciprocal diagonal
  __syncthreads();
  if (tid < 64) { sm.piv[tid] = piv_keep; sm.rinv[tid] = rinv_keep; }
  // right-hand sides B[a][k] = U_m[k][a] into B2's place (row-major N x N), then back
  // substitution with the upper triangular U_R[a][l] = R~[a][piv[l]] (rows from global):
  // column-oriented, all threads: once row a of the solution is known it is taken out of all
  // earlier rows at once.  The solution row a belongs to worker piv[a].
  // (B2 still holds the pair part of C, which the resume state wants)
  double* Bs = cur;     // the projector's tiles are no longer needed
  __syncthreads();
#pragma unroll
  for (int q = 0; q < EPT; ++q) {
    const int e = tid + q * NTHREADS;
    if (e < N * N) {
      const int a = e / N, k = e - a * N;
      Bs[e] = (a < rank && k < mm) ? Um[k * N + a] : 0.0;
    }
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < EPT; ++q) {
    const int e = tid + q * NTHREADS;
    if (e < N * N) {
      const int a = e / N, l = e - a * N;
      Sp[e] = (a < rank && l < rank) ? RtG[a * N + sm.piv[l]] : 0.0;   // Sp is free again
    }
  }
  __syncthreads();
  for (int a = rank - 1; a >= 0; --a) {
    const double ri = sm.rinv[a];
    if (tid < N) Bs[a * N + tid] *= ri;            // solution row a
    __syncthreads();
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
      const int e = tid + q * NTHREADS;
      if (e < N * N) {
        const int i = e / N, k = e - i * N;
        if (i < a) Bs[e] = fma(-Sp[i * N + a], Bs[a * N + k], Bs[e]);
      }
    }
    __syncthreads();
  }
  // A[piv[a]][k] = dinv[piv[a]] * solution[a][k];  c = A beta / p
  for (int idx = tid; idx < p * m; idx += NTHREADS) info->A[idx] = 0.0;
  __syncthreads();
  if (tid < N * 16) {
    const int a = tid >> 4, l16 = tid & 15;
    double acc = 0.0;
    if (a < rank) {
      const int i = sm.piv[a];
      const double di = sm.dinv[i];
      for (int k = l16; k < mm; k += 16) {
        const double av = Bs[a * N + k] * di;
        if (i < p && k < m) info->A[i * m + k] = av;
        acc = fma(av, sm.beta[k], acc);
      }
    }
    acc = row_sum(acc);
    if (a < rank && l16 == 0) sm.gd[sm.piv[a]] = acc / (double)P;     // c of that column
  }
  if (tid < 64) sm.used[tid] = 0;
  __syncthreads();
  if (tid < rank) sm.used[sm.piv[tid]] = 1;
  __syncthreads();
  if (tid < p) {
    const double cv = sm.used[tid] ? sm.gd[tid] : 0.0;   // workers outside the pivot set: 0
    cg[tid] = cv;
    info->c[tid] = cv;
    info->s[tid] = sm.s[tid];
    info->v[tid] = (GRP ? sm.ginv[tid] > 0.0 : sm.s[tid] > 0.0) ? 1.0 - sm.rho[tid] : 0.0;
    info->w[tid] = sm.w[tid];
  }
  if (rs) {
    // weights for the solve that would come next
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
      const int e = tid + q * NTHREADS;
      if (e < N * N) {
        const int i = e / N, j = e - i * N;
        if (i < p && j < p) rs->cp[i * p + j] = i != j ? B2[eidx<T>(i, j)] : 0.0;
      }
    }
    if (tid < p) rs->w[tid] = sm.w[tid];
    if (tid == 0) { rs->prev_obj = prev_obj; rs->it0 = it0 + iters_done; }
  }
  if (tid == 0) {
    info->status = 0;
    info->p = p; info->m = m; info->rank = rank;
    info->iters_done = it0 + iters_done;
    info->sweeps = steps;
    info->eigengap = nan("");        // filled in on demand by fa_get_info
    Ml[N * N] = (double)rank;
    Ml[N * N + 1] = (double)m;
  }
}

template <int T>
static constexpr size_t lds_bytes() {
  return (size_t)4 * T * T * FA_TILE * sizeof(double) + sizeof(Small);
}

template <int T, int MODE>
static hipError_t launch_tm(const double* Kd, int p, int nworkers, const int* sizes_d, int m,
                            double lambda, int iters, double tol, double delta, double expo,
                            double rank_tol, double pair_tol, double* cd, fa_info* info_d,
                            double* tiles_ws, double* mlast, int spin_budget, fa_resume* rs,
                            hipStream_t st, const fa_ktime* tm) {
  FA_LAUNCH(tm, (fa_irls64_kernel<T, MODE>), dim3(1), dim3(NTHREADS), lds_bytes<T>(), st, Kd, p,
            nworkers, sizes_d, m, iters, lambda, tol, delta, expo, rank_tol, pair_tol, cd, info_d,
            tiles_ws, mlast, spin_budget, rs);
  return hipGetLastError();
}

template <int T>
static hipError_t launch_t(const double* Kd, int p, int nworkers, const int* sizes_d, int m,
                           double lambda, int iters, double tol, double delta, double expo,
                           double rank_tol, double pair_tol, double* cd, fa_info* info_d,
                           double* tiles_ws, double* mlast, int spin_budget, fa_resume* rs,
                           hipStream_t st, const fa_ktime* tm) {
  if (nworkers > 0)
    return launch_tm<T, 2>(Kd, p, nworkers, sizes_d, m, lambda, iters, tol, delta, expo, rank_tol,
                           pair_tol, cd, info_d, tiles_ws, mlast, spin_budget, rs, st, tm);
  if constexpr (T > 1) {
    if (expo == 0.5)
      return launch_tm<T, 0>(Kd, p, 0, nullptr, m, lambda, iters, tol, delta, expo, rank_tol,
                             pair_tol, cd, info_d, tiles_ws, mlast, spin_budget, rs, st, tm);
    return launch_tm<T, 1>(Kd, p, 0, nullptr, m, lambda, iters, tol, delta, expo, rank_tol,
                           pair_tol, cd, info_d, tiles_ws, mlast, spin_budget, rs, st, tm);
  }
  return hipErrorInvalidValue;      // single columns at p <= 16 have a solver of their own
}

template <int T, int MODE>
static hipError_t prepare_t() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(fa_irls64_kernel<T, MODE>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes<T>());
}

hipError_t fa_irls64_prepare(void) {
  hipError_t e = prepare_t<1, 2>();
#define FA_X(t)                                        \
  if (e == hipSuccess) e = prepare_t<t, 0>();          \
  if (e == hipSuccess) e = prepare_t<t, 1>();          \
  if (e == hipSuccess) e = prepare_t<t, 2>();
  FA_X(2) FA_X(3) FA_X(4)
#undef FA_X
  return e;
}

hipError_t fa_launch_irls64(const double* Kd, int p, int nworkers, const int* sizes_d, int m,
                            double lambda, int iters, double tol, double delta, double exponent_a,
                            double rank_tol, double pair_tol, double* cd, fa_info* info_d,
                            double* tiles_ws, double* mlast, int spin_budget, fa_resume* rs,
                            hipStream_t st, const fa_ktime* tm) {
  const double expo = exponent_a == 2.0 ? 0.5 : 1.0 / exponent_a;
  switch ((p + 15) / 16) {
#define FA_X(t)                                                                                  \
    case t:                                                                                      \
      return launch_t<t>(Kd, p, nworkers, sizes_d, m, lambda, iters, tol, delta, expo, rank_tol, \
                         pair_tol, cd, info_d, tiles_ws, mlast, spin_budget, rs, st, tm);
    FA_X(1) FA_X(2) FA_X(3) FA_X(4)
#undef FA_X
  }
  return hipErrorInvalidValue;
}
