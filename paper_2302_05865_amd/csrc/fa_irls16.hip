// K3 for p <= 16: the p x p part of the Flag Aggregator (normalisation, IRLS by repeated
// weighted PCA, coefficients) in one workgroup.  Two paths:
//   * fast path (namespace fastp, wave 0): projector by matrix-core purification, no eigensolver;
//   * Jacobi path (rest of this file, 256 threads): full eigen-decomposition per solve, used
//     when the purification cannot converge (tied eigenvalues) or when asked for.
//
// The Jacobi path:
//
// Same mathematics as fa_irls_core.inc (Eq. 5 / Sec. 2.3 option (2) objective, Alg. 1 IRLS
// step and direction; see the header of that file for the R-factor formulation).  What
// differs is how the symmetric eigenproblem is scheduled, because at p = 15 the twenty
// eigen-solves are a serial chain of ~1000 rotation rounds and every cycle of a round counts:
//
//  * wave 0 is the Jacobi "master".  The 16 x 16 matrix M sits in LDS; lane (t, u) owns the
//    2 x 2 block (rows of pair t, columns of pair u) of the current round-robin pairing.
//    Each lane reads the two diagonal blocks it depends on and computes both plane rotations
//    itself (no broadcast step), applies them to its block and writes it back.  A single
//    wavefront needs no workgroup barrier between rounds: its LDS operations complete in
//    order.  Rotations use two reciprocal square roots and no division.
//  * the rotations are logged to LDS; waves 1 and 2 replay the log of the previous sweep
//    on the rows of R (gradients in the current eigenbasis) and of Ut (accumulated
//    eigenvectors) while the master is already running the next sweep.  One workgroup
//    barrier per sweep.
//  * a sweep whose largest relative off-diagonal was below 1e-9 is the last one (Jacobi
//    converges quadratically), so no verification sweep is spent.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fa.h"
#include "fa_internal.h"

namespace {

constexpr int NP = 16;        // padded matrix order
constexpr int LD = 17;        // leading dimension in LDS (odd: spreads banks)
constexpr int NROUND = 15;    // rounds of one round-robin sweep
constexpr int NPAIR = 8;      // disjoint pairs per round
constexpr int MAX_SWEEPS = 40;

struct __attribute__((aligned(16))) Rot {
  double c, s;
  int p, q;
  int active;
  int pad;
};

struct Smem {
  double M[NP * LD], R[NP * LD], Ut[NP * LD], T[NP * LD], D2inv[NP * LD], Vt[NP * LD];
  double s[NP], dinv[NP], w[NP], rho[NP], v[NP], lam0[NP], mu[NP], beta[NP];
  Rot log[2][NROUND][NPAIR];
  double red[4];
  int pos[NP], order[NP];
  int done[2], sweeps, status, rank;
};

// 1/sqrt(x) from the hardware estimate plus NR Newton steps.
template <int NR>
__device__ __forceinline__ double rsq_nr(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double hx = 0.5 * x;
#pragma unroll
  for (int k = 0; k < NR; ++k) {
    const double e = fma(-hx * y, y, 0.5);
    y = fma(y, e, y);
  }
  return y;
}

// Plane rotation for the index pair (a,b) of a symmetric matrix, zeroing A_ab:
//   x_a' = c x_a - s x_b,  x_b' = s x_a + c x_b.
// With zeta = A_bb - A_aa, N = 2 A_ab sign(zeta), D = |zeta| + sqrt(zeta^2 + 4 A_ab^2):
//   tan = N / D,  c = D / sqrt(D^2 + N^2),  s = N / sqrt(D^2 + N^2)
// (the small-angle root of the Jacobi equation; two reciprocal square roots, no division).
// *big: the off-diagonal entry exceeded 1e-9 relative to sqrt(|A_aa A_bb|).
__device__ __forceinline__ void rotation(double aaa, double abb, double aab, double* c, double* s,
                                         bool* active, bool* big) {
  const double dd = fabs(aaa * abb);
  const double o2 = aab * aab;
  const bool act = (o2 > 1e-30 * dd) && (fabs(aab) > 1e-300);
  const double zeta = abb - aaa;
  const double nn = zeta < 0.0 ? -2.0 * aab : 2.0 * aab;
  const double h2 = fma(zeta, zeta, 4.0 * o2);
  const double dn = fma(h2, rsq_nr<1>(act ? h2 : 1.0), fabs(zeta));
  const double wn = rsq_nr<2>(act ? fma(dn, dn, nn * nn) : 1.0);
  *c = act ? dn * wn : 1.0;
  *s = act ? nn * wn : 0.0;
  *active = act;
  *big = act && (o2 > 1e-18 * dd);
}

// Round-robin pairing of 16 indices: index 15 stays, the others advance cyclically.
// Slot t of round 0 holds (15, 0) for t = 0 and (t, 15 - t) otherwise.
__device__ __forceinline__ int rr_next(int x) { return x >= 14 ? (x == 15 ? 15 : 0) : x + 1; }

__device__ __forceinline__ void wave_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// One sweep by the master wavefront (all 64 lanes of wave 0).  Returns true when the sweep
// made M diagonal to working precision (nothing above 1e-9 relative was met).
__device__ __forceinline__ bool master_sweep(double* __restrict__ M, Rot (*lg)[NPAIR], int lane) {
  const int t = lane >> 3, u = lane & 7;
  int a0 = t == 0 ? 15 : t, b0 = t == 0 ? 0 : 15 - t;
  int a1 = u == 0 ? 15 : u, b1 = u == 0 ? 0 : 15 - u;
  bool big = false, any = false;
#pragma unroll 1
  for (int round = 0; round < NROUND; ++round) {
    const int ra0 = a0 * LD, rb0 = b0 * LD, ra1 = a1 * LD, rb1 = b1 * LD;
    const double daa0 = M[ra0 + a0], dbb0 = M[rb0 + b0], dab0 = M[ra0 + b0];
    const double daa1 = M[ra1 + a1], dbb1 = M[rb1 + b1], dab1 = M[ra1 + b1];
    const double b00 = M[ra0 + a1], b01 = M[ra0 + b1];
    const double b10 = M[rb0 + a1], b11 = M[rb0 + b1];
    double c0, s0, c1, s1;
    bool act0, act1, g0, g1;
    rotation(daa0, dbb0, dab0, &c0, &s0, &act0, &g0);
    rotation(daa1, dbb1, dab1, &c1, &s1, &act1, &g1);
    const bool round_active = __ballot(act0 || act1) != 0ull;
    big = big || (__ballot(g0 || g1) != 0ull);
    any = any || round_active;
    if (u == 0) {
      Rot e;
      e.c = c0; e.s = s0; e.p = a0; e.q = b0; e.active = act0 ? 1 : 0; e.pad = 0;
      lg[round][t] = e;
    }
    if (round_active) {
      const double x00 = c0 * b00 - s0 * b10, x01 = c0 * b01 - s0 * b11;
      const double x10 = s0 * b00 + c0 * b10, x11 = s0 * b01 + c0 * b11;
      const double d00 = c1 * x00 - s1 * x01, d01 = s1 * x00 + c1 * x01;
      double d10 = c1 * x10 - s1 * x11;
      const double d11 = s1 * x10 + c1 * x11;
      if (t == u) d10 = d01;     // keep the diagonal block exactly symmetric
      M[ra0 + a1] = d00; M[ra0 + b1] = d01;
      M[rb0 + a1] = d10; M[rb0 + b1] = d11;
    }
    a0 = rr_next(a0); b0 = rr_next(b0); a1 = rr_next(a1); b1 = rr_next(b1);
    wave_fence();
  }
  return !any || !big;
}

// Replay one sweep's log on the rows of X (16 columns) by one wavefront.
__device__ __forceinline__ void replay_sweep(double* __restrict__ X, const Rot (*lg)[NPAIR],
                                             int lane) {
#pragma unroll 1
  for (int round = 0; round < NROUND; ++round) {
    const int j = lane & 15;
    const Rot e0 = lg[round][lane >> 4], e1 = lg[round][4 + (lane >> 4)];
    const double x0 = X[e0.p * LD + j], y0 = X[e0.q * LD + j];
    const double x1 = X[e1.p * LD + j], y1 = X[e1.q * LD + j];
    if (e0.active) {
      X[e0.p * LD + j] = e0.c * x0 - e0.s * y0;
      X[e0.q * LD + j] = e0.s * x0 + e0.c * y0;
    }
    if (e1.active) {
      X[e1.p * LD + j] = e1.c * x1 - e1.s * y1;
      X[e1.q * LD + j] = e1.s * x1 + e1.c * y1;
    }
    wave_fence();
  }
}

// Diagonalise sm.M (16 x 16, live part in the leading block) and apply the same rotations
// to the rows of XA (by wave 1) and XB (by wave 2); either may be null.  Leaves pos/order
// (descending eigenvalues of the first `nlive` diagonal entries) in sm.pos / sm.order.
__device__ __forceinline__ void jacobi16(Smem& sm, double* XA, double* XB, int nlive) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int sweep = 0;
  for (; sweep < MAX_SWEEPS; ++sweep) {
    const int buf = sweep & 1;
    if (wave == 0) {
      const bool fin = master_sweep(sm.M, sm.log[buf], lane);
      if (lane == 0) {
        sm.done[buf] = (fin || sweep + 1 == MAX_SWEEPS) ? 1 : 0;
        sm.sweeps += 1;
      }
    } else if (sweep > 0) {
      if (wave == 1 && XA) replay_sweep(XA, sm.log[buf ^ 1], lane);
      if (wave == 2 && XB) replay_sweep(XB, sm.log[buf ^ 1], lane);
    }
    __syncthreads();
    if (sm.done[buf]) break;
  }
  // the last sweep's log; meanwhile the master ranks the eigenvalues
  const int buf = sweep & 1;
  if (wave == 1 && XA) replay_sweep(XA, sm.log[buf], lane);
  if (wave == 2 && XB) replay_sweep(XB, sm.log[buf], lane);
  if (wave == 0 && lane < NP) {
    if (lane < nlive) {
      const double va = sm.M[lane * LD + lane];
      int k = 0;
      for (int b = 0; b < nlive; ++b) {
        const double vb = sm.M[b * LD + b];
        if (vb > va || (vb == va && b < lane)) ++k;
      }
      sm.pos[lane] = k;
      sm.order[k] = lane;
      sm.mu[lane] = va;
    } else {
      sm.pos[lane] = lane;
      sm.order[lane] = lane;
      sm.mu[lane] = 0.0;
    }
  }
  __syncthreads();
}

// Deterministic sum over the workgroup (fixed butterfly inside each wave, waves in order).
__device__ __forceinline__ double block_sum(double x, Smem& sm) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.red[threadIdx.x >> 6] = x;
  __syncthreads();
  return ((sm.red[0] + sm.red[1]) + sm.red[2]) + sm.red[3];
}

}  // namespace


// ==========================================================================================
// Fast path (wave 0 only): the weighted PCA needs only the *projector* P onto the m leading
// eigenvectors of M = R C R^T -- the residuals 1 - v_i = |(I-P) r_i|^2 / s_i, the pair
// residuals and the final direction are all functions of P.  P is computed without an
// eigensolver, by trace-correcting purification: scale M into [0,1], then repeat
//     X <- X^2          if that brings trace(X) closer to m,
//     X <- 2X - X^2     otherwise,
// which drives every eigenvalue to 0 or 1 while steering exactly m of them to 1.  Each step is
// one 16 x 16 fp64 product = four v_mfma_f64_16x16x4_f64 on registers: for a symmetric X the
// accumulator layout (register r of lane l = entry (4r + l/16, l%16)) is at once the A- and
// the B-operand layout, so the iteration never leaves the register file.  trace(X^2) =
// |X|_F^2 is reduced on the vector ALU while the matrix core multiplies.
// R comes from a pivoted Cholesky factorisation of the normalised Gram matrix (R^T R = K~,
// rank-revealing), so no eigen-decomposition is needed at set-up either.
// If the purification does not converge (eigenvalues m and m+1 tie), the Jacobi path below
// redoes the whole solve.
namespace fastp {

constexpr int LDF = 17;
constexpr int LDZ = 18;          // column pitch of Zs (16-byte aligned rows of 16 doubles)
constexpr int MAX_PURIFY = 128;

struct Fmem {
  double Kt[16 * LDF];   // Gram, then normalised Gram
  double Rt[16 * LDF];   // rows of R~ (pivoted Cholesky): R~^T R~ = K~
  double Rr[16 * LDF];   // R = R~ D^1/2
  double Xi[16 * LDF];   // inverse of the pivot block of R~
  double Bm[16 * LDF];   // right inverse of R: R Bm = I_r   (p x r)
  double Ps[16 * LDF];   // projector
  double Um[16 * LDF];   // orthonormal basis of range(P) (r x mm), as rows: Um[k][a]
  double Am[16 * LDF];   // A (p x m)
  __attribute__((aligned(16))) double Zs[16 * LDZ];   // [0..15]: diag(Z^T Z), Z = (I-P) R
  double s[16], dinv[16], r1[16], beta[16], rinv[16];
  int piv[16];
};

typedef double v4d __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xf, 0xf, false);
  hi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}
// sum / max over each 16-lane row (lanes l with equal l/16); every lane of the row gets it
__device__ __forceinline__ double row_sum(double x) {
  x += dpp_f64<0x128>(x);   // row_ror:8
  x += dpp_f64<0x124>(x);   // row_ror:4
  x += dpp_f64<0x122>(x);   // row_ror:2
  x += dpp_f64<0x121>(x);   // row_ror:1
  return x;
}
__device__ __forceinline__ double row_max(double x) {
  x = fmax(x, dpp_f64<0x128>(x));
  x = fmax(x, dpp_f64<0x124>(x));
  x = fmax(x, dpp_f64<0x122>(x));
  x = fmax(x, dpp_f64<0x121>(x));
  return x;
}
__device__ __forceinline__ double lane_bcast(double x, int srclane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(x), srclane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(x), srclane);
  return __hiloint2double(hi, lo);
}
// Sum over the four lanes c, 16 + c, 32 + c, 48 + c, in every one of them: (t0 + t1) + (t2 + t3).
// v_permlane16_swap / v_permlane32_swap with both operands the same value return the even rows
// (the lower half) and the odd rows (the upper half) side by side.
__device__ __forceinline__ double rows_sum(double t) {
  int lo = __double2loint(t), hi = __double2hiint(t);
  auto a = __builtin_amdgcn_permlane16_swap((unsigned)lo, (unsigned)lo, false, false);
  auto b = __builtin_amdgcn_permlane16_swap((unsigned)hi, (unsigned)hi, false, false);
  const double s = __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
  lo = __double2loint(s); hi = __double2hiint(s);
  a = __builtin_amdgcn_permlane32_swap((unsigned)lo, (unsigned)lo, false, false);
  b = __builtin_amdgcn_permlane32_swap((unsigned)hi, (unsigned)hi, false, false);
  return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}
// deterministic sum over the wavefront, same value in every lane
__device__ __forceinline__ double wave_sum(double x) {
  x = row_sum(x);
  return ((lane_bcast(x, 0) + lane_bcast(x, 16)) + lane_bcast(x, 32)) + lane_bcast(x, 48);
}

// |X|_F^2 over the wavefront in two stages, so that the second stage of one purification
// step can be issued next to the first stage of the following one (fp64 vector operations
// have a long dependent latency; two interleaved chains fit under one 16 x 16 product).
__device__ __forceinline__ double fro2_stage1(const v4d& x) {
  double t = fma(x[0], x[0], x[1] * x[1]) + fma(x[2], x[2], x[3] * x[3]);
  t += dpp_f64<0x128>(t);
  t += dpp_f64<0x124>(t);
  return t;
}
__device__ __forceinline__ double fro2_stage2(double t) {
  t += dpp_f64<0x122>(t);
  t += dpp_f64<0x121>(t);
  return (lane_bcast(t, 0) + lane_bcast(t, 16)) + (lane_bcast(t, 32) + lane_bcast(t, 48));
}

__device__ __forceinline__ v4d mm16(const v4d& a, const v4d& b) {
  v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s], b[s], acc, 0, 0, 0);
  return acc;
}

template <int CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned x) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}

// Greedy diagonal-pivoted Cholesky of the PSD matrix S (16 x 16 in LDS): rows[k][j] with
// rows^T rows = S.  Stops at max_rank rows or when the chosen remaining diagonal entry is
// <= tol.  Right-looking, on the matrix core: S is kept in the accumulator's register order
// (entry r of lane (q, c) = element (4r + q, c)); the pivot row pv = 4 r' + q' is then entry r'
// of the sixteen lanes (q', c), which is also where a matrix instruction takes column k = q' of
// its A operand and row k = q' of its B operand from - so with that row, scaled, in those lanes
// and zero in the others one instruction subtracts the rank-one term from all of S.  The pivot
// is the largest remaining diagonal entry as seen in fp32 (any near-largest pivot serves; ties
// go to the lowest index).  The loop is kept rolled on purpose: this code runs once per call,
// and straight-line code that is executed once costs more in instruction fetch than it
// saves.  It must be inlined: as a called function it slowed the whole solver by 10 %.
// Returns the number of rows; piv[k] is the column chosen at step k, rinv[k] = 1/rows[k][piv[k]].
#ifndef FA_CHOL_ATTR
#define FA_CHOL_ATTR __forceinline__
#endif
__device__ FA_CHOL_ATTR int pivoted_cholesky(const double* S, double* rows, int* piv, double* rinv,
                                             double tol, int max_rank, int lane) {
  const int c16 = lane & 15, q4 = lane >> 4;
  v4d s;
#pragma unroll
  for (int r = 0; r < 4; ++r) s[r] = S[(4 * r + q4) * LDF + c16];
  // element (c, c) is entry c / 4 of the lane (c % 4, c)
  const bool hasd = (c16 & 3) == q4;
  const int rd = c16 >> 2;
  int rank = 0;
#pragma unroll 1
  for (int k = 0; k < max_rank; ++k) {
    const double d = rd == 0 ? s[0] : rd == 1 ? s[1] : rd == 2 ? s[2] : s[3];
    const float df = (hasd && d > 0.0) ? (float)d : 0.0f;
    unsigned key = hasd ? ((__float_as_uint(df) & ~15u) | (unsigned)(15 - c16)) : 0u;
    key = max(key, dpp_u32<0x128>(key));   // row_ror:8
    key = max(key, dpp_u32<0x124>(key));   // row_ror:4
    key = max(key, dpp_u32<0x122>(key));   // row_ror:2
    key = max(key, dpp_u32<0x121>(key));   // row_ror:1
    const unsigned k0 = (unsigned)__builtin_amdgcn_readlane((int)key, 0);
    const unsigned k1 = (unsigned)__builtin_amdgcn_readlane((int)key, 16);
    const unsigned k2 = (unsigned)__builtin_amdgcn_readlane((int)key, 32);
    const unsigned k3 = (unsigned)__builtin_amdgcn_readlane((int)key, 48);
    const int pv = 15 - (int)(max(max(k0, k1), max(k2, k3)) & 15u);
    const int qp = pv & 3, rp = pv >> 2;
    // row pv of what is left of S, in the lanes (qp, c); its diagonal entry is in lane (qp, pv)
    const double rowv = rp == 0 ? s[0] : rp == 1 ? s[1] : rp == 2 ? s[2] : s[3];
    const double dp = lane_bcast(rowv, 16 * qp + pv);
    if (!(dp > tol)) break;
    const double rs = rsq_nr<2>(dp);
    const double a = q4 == qp ? rowv * rs : 0.0;
    if (q4 == qp) rows[k * LDF + c16] = a;
    if (lane == 0) { piv[k] = pv; rinv[k] = rs; }
    s = __builtin_amdgcn_mfma_f64_16x16x4f64(-a, a, s, 0, 0, 0);
    // row and column pv are done with (what the update leaves there is rounding noise)
#pragma unroll
    for (int r = 0; r < 4; ++r) s[r] = (c16 == pv || (q4 == qp && rp == r)) ? 0.0 : s[r];
    rank = k + 1;
  }
  wave_fence();
  for (int k = rank; k < 16; ++k) {
    if (lane < 16) rows[k * LDF + c16] = 0.0;
    if (lane == 0) { piv[k] = 0; rinv[k] = 0.0; }
  }
  wave_fence();
  return rank;
}

// Returns 1 when the solve was completed here (including the error statuses), 0 when the
// caller must fall back to the Jacobi path.
__device__ int solve(const double* __restrict__ Kg, int p, int m, int iters, double lambda,
                     double tol, double delta, double expo, double rank_tol, double pair_tol,
                     double* __restrict__ cg, fa_info* __restrict__ info,
                     double* __restrict__ mlast, Fmem& fm, fa_resume* rs) {
  const int lane = threadIdx.x & 63;
  const int c16 = lane & 15, q4 = lane >> 4;
  const double coef = (lambda > 0.0 && p > 1) ? lambda / (double)(p - 1) : 0.0;
  const int it0 = rs ? rs->it0 : 0;                    // solves done by earlier launches
  const bool scaled = rs && rs->scaled;

  // ---- Gram, norms, status ---------------------------------------------------------------
  bool bad = false;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = 4 * r + q4;
    const bool in = i < p && c16 < p;
    double kv = in ? Kg[i * p + c16] : 0.0;
    if (in && scaled) kv *= rs->uinv[i] * rs->uinv[c16];   // Gram of scaled columns
    fm.Kt[i * LDF + c16] = kv;
    if (in) info->K[i * p + c16] = kv;
    bad = bad || !(fabs(kv) <= 1.79e308);
  }
  wave_fence();
  const double sj = fm.Kt[c16 * LDF + c16];            // |g_j|^2 of this lane's column
  const double dj = sj > 0.0 ? 1.0 / sqrt(sj) : 0.0;
  const bool any_bad = __ballot(bad) != 0ull;
  const bool any_live = __ballot(sj > 0.0) != 0ull;
  if (lane < 16) { fm.s[lane] = sj; fm.dinv[lane] = dj; }
  wave_fence();
  if (any_bad || !any_live) {
    const int st = any_bad ? 4 : 5;
    if (lane < p) {
      const double cv = any_bad ? nan("") : 0.0;
      cg[lane] = cv;
      info->c[lane] = cv; info->s[lane] = sj; info->v[lane] = 0.0; info->w[lane] = 0.0;
    }
    for (int idx = lane; idx < p * m; idx += 64) info->A[idx] = 0.0;
    if (lane == 0) {
      info->status = st; info->p = p; info->m = m; info->rank = 0; info->iters_done = 0;
      info->sweeps = 0; info->eigengap = 0.0;
    }
    return 1;
  }

  // ---- pairwise distances (registers, entry (4r+q4, c16)), normalised Gram (LDS) ---------
  double d2inv[4], kt[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = 4 * r + q4;
    const double si = fm.s[i], di = fm.dinv[i];
    const double kv = fm.Kt[i * LDF + c16];
    const double d2 = si + sj - 2.0 * kv;
    const bool livep = i < p && c16 < p && i != c16 && d2 > pair_tol * (si + sj);
    d2inv[r] = livep ? 1.0 / d2 : 0.0;
    kt[r] = i == c16 ? (si > 0.0 ? 1.0 : 0.0) : kv * di * dj;
  }
  wave_fence();
#pragma unroll
  for (int r = 0; r < 4; ++r) fm.Kt[(4 * r + q4) * LDF + c16] = kt[r];
  wave_fence();

  // ---- R from the pivoted Cholesky factorisation of K~; rank; right inverse --------------
  const int rank = pivoted_cholesky(fm.Kt, fm.Rt, fm.piv, fm.rinv, rank_tol, 16, lane);
  // Xi = inverse of the (upper triangular, in pivot order) block U = R~[:, piv]; lane c16
  // solves U x = e_c16 by back substitution, column-oriented: once x_k is known it is taken
  // out of all earlier equations at once (independent multiply-adds, no dependent chain)
  {
    double bcol[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bcol[i] = (i == c16) ? 1.0 : 0.0;
#pragma unroll
    for (int k = 15; k >= 0; --k) {
      if (k < rank) {
        const double xk = bcol[k] * fm.rinv[k];
        const int pk = fm.piv[k];
#pragma unroll
        for (int i = 0; i < k; ++i) bcol[i] = fma(-fm.Rt[i * LDF + pk], xk, bcol[i]);
        bcol[k] = xk;
      } else {
        bcol[k] = 0.0;
      }
    }
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (lane < 16) fm.Xi[k * LDF + c16] = (c16 < rank) ? bcol[k] : 0.0;
    wave_fence();
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = 4 * r + q4;
    fm.Bm[i * LDF + c16] = 0.0;
    fm.Rr[i * LDF + c16] = (i < rank) ? fm.Rt[i * LDF + c16] * sqrt(sj) : 0.0;
    fm.Um[i * LDF + c16] = 0.0;
  }
  wave_fence();
  for (int k = lane >> 4; k < rank; k += 4) {
    const int i = fm.piv[k];
    fm.Bm[i * LDF + c16] = (c16 < rank) ? fm.Xi[k * LDF + c16] * fm.dinv[i] : 0.0;
  }
  wave_fence();
  v4d ra, rb;   // R as A operand (entry (c16, 4s+q4)) and as B operand (entry (4s+q4, c16))
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    ra[s] = fm.Rr[c16 * LDF + 4 * s + q4];
    rb[s] = fm.Rr[(4 * s + q4) * LDF + c16];
  }
  if (lane < 16) {
    double a4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) a4[jj & 3] += fm.Rr[lane * LDF + jj];
    fm.r1[lane] = (a4[0] + a4[1]) + (a4[2] + a4[3]);   // R 1
  }
  wave_fence();

  // ---- IRLS ------------------------------------------------------------------------------
  const int mm = m < rank ? m : rank;
  bool isdiag[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) isdiag[r] = (4 * r + q4) == c16;
  const bool livej = sj > 0.0;
  double wj = livej ? 1.0 : 0.0;                      // IRLS weight of this lane's column
  double rhoj = 0.0, rsj = 0.0;
  const double rs_delta = 1.0 / sqrt(delta);          // the weight floor, as a cap on 1/sqrt(rho)
  v4d cp;                                              // pair part of C, entry (4r+q4, c16)
#pragma unroll
  for (int r = 0; r < 4; ++r) cp[r] = -2.0 * coef * d2inv[r];
  double prev_obj = 0.0;
  if (it0 > 0) {
    // continue from the weights the previous launch (or the streamed residuals) left
    wj = (livej && c16 < p) ? rs->w[c16] : 0.0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = 4 * r + q4;
      cp[r] = (i < p && c16 < p && i != c16) ? rs->cp[i * p + c16] : 0.0;
    }
    prev_obj = rs->prev_obj;
  }
  v4d x = {0.0, 0.0, 0.0, 0.0}, mk = {0.0, 0.0, 0.0, 0.0};
  int iters_done = 0, steps = 0;
  for (int it = 0; it < iters; ++it) {
    // C = diag(w/s) + Laplacian of the pair part;  M = R C R^T via W = C R^T, M = R W
    // (the pair part is symmetric, bit for bit: the sum of row j is the sum of column j, which
    // is spread over the four lanes that hold column j)
    v4d c;
    const double csum = rows_sum((cp[0] + cp[1]) + (cp[2] + cp[3]));
#pragma unroll
    for (int r = 0; r < 4; ++r) c[r] = isdiag[r] ? wj * dj * dj - csum : cp[r];
    const v4d wmat = mm16(c, ra);
    mk = mm16(ra, wmat);
    if (mm < rank) {
      // scale into [0, 1]: M is PSD, so 0 <= eigenvalues <= trace(M)
      double tr = 0.0;
#pragma unroll
      for (int r = 0; r < 4; ++r) tr += isdiag[r] ? mk[r] : 0.0;
      const double hi = wave_sum(tr);
      // any scale that keeps the eigenvalues in [0, 1] will do: the hardware reciprocal,
      // shaded down by more than its error
      const double sc = __builtin_amdgcn_rcp(hi) * (1.0 - 1e-7);
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = mk[r] * sc;
      // Steering: square when trace(X) > m, else X <- 2X - X^2.  trace(X) is carried along
      // (after a square it is the previous |X|_F^2, otherwise 2 trace(X) - |X|_F^2), so the
      // only reduction per step is |X|_F^2, and its result is not needed before the end of
      // the *next* step: the reduction is split in two halves (second half for X_{k-1},
      // first half for X_k) issued beside the four matrix-core instructions of X_k^2.
      // The same numbers, one step late, say when X is nearly a projector:
      // trace(X_{k-1}) - |X_{k-1}|_F^2 is the distance of X_{k-1} from idempotency.  The flag
      // is acted upon at the top of the next step (a branch on a value computed long before
      // costs nothing; a branch on the end of the reduction chain would stall every step):
      // two steps after the distance fell below 1e-8 the iterate has converged (each step
      // squares the error at one end of the spectrum and doubles it at the other), and there
      // trace and |X|_F^2 are measured exactly, because the carried trace drifts by rounding.
      double tXp = 2.0, tX = hi * sc;      // trace(X_{k-1}) (dummy for k = 0), trace(X_k)
      double pend = tX * (1.0 / 16.0);     // stage-1 partial of |X_{k-1}|_F^2: stage 2 gives tX
      bool sqp = true;                     // with the above, step 0 computes trace(X_0) = tX
      bool conv = false;
      int k_end = MAX_PURIFY;
      // Two loops: the steps run in an inner loop of their own until the iterate is nearly
      // idempotent, the exact test sits outside it.  (With the test inside one loop, never
      // taken until the end, every step was a quarter slower: 700 against 534 cycles.)
      // One step X_k (xi) -> X_{k+1} (xo); returns "X_{k-1} was nearly idempotent".  The loop
      // runs two of them per pass, from x into a second set of registers and back, which
      // spares the copies of a rotated loop and gives the scheduler two steps to interleave
      // (522 against 593 cycles per step on a stand-alone copy of the loop).
      auto one_step = [&](const v4d& xi, v4d& xo) __attribute__((always_inline)) -> bool {
        const v4d y = mm16(xi, xi);
        const double tYp = fro2_stage2(pend);              // |X_{k-1}|_F^2
        pend = fro2_stage1(xi);
        tX = sqp ? tYp : fma(2.0, tXp, -tYp);              // trace(X_k)
        const bool nr = (tXp - tYp < 1e-8);
        const bool sq = tX > (double)mm;
        if (sq) {
#pragma unroll
          for (int r = 0; r < 4; ++r) xo[r] = y[r];
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) xo[r] = fma(2.0, xi[r], -y[r]);
        }
        tXp = tX;
        sqp = sq;
        steps = steps + 1;
        return nr;
      };
      for (int k = 0; k < MAX_PURIFY;) {
        bool near = false;
        do {
          v4d x2;
          near = one_step(x, x2);
          ++k;
          if (near || k >= MAX_PURIFY) {
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = x2[r];
            break;
          }
          near = one_step(x2, x);
          ++k;
        } while (!near && k < MAX_PURIFY);
        if (!near) break;
        double td = 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r) td += isdiag[r] ? x[r] : 0.0;
        tX = wave_sum(td);
        if (tX - fro2_stage2(fro2_stage1(x)) < 1e-12) {
          // idempotent; it is the wanted projector only if its trace is m (the maps are
          // monotone, so the eigenvalue order is kept whatever the steering did)
          conv = fabs(tX - (double)mm) < 0.25;
          k_end = k;
          break;
        }
        // not yet: go on from the exact trace
        tXp = 2.0; sqp = true; pend = tX * (1.0 / 16.0);
      }
      if (!conv) return -(1000 + it * 1000 + k_end);
    } else {
      // m >= rank: Y spans all of span(G)
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = (isdiag[r] && c16 < rank) ? 1.0 : 0.0;
    }
    // Z = (I - P) R
    v4d qm;
#pragma unroll
    for (int r = 0; r < 4; ++r) qm[r] = isdiag[r] ? 1.0 - x[r] : -x[r];
    const v4d z = mm16(qm, rb);
    // Q = Z^T Z straight from the accumulator registers (for A = tile^T the register layout
    // of Z is both operands): |z_j|^2 = q_jj is the residual of worker j, and the pair
    // residuals come from |z_i - z_j|^2 = q_ii + q_jj - 2 q_ij, entry (i, j) of Q sitting in
    // the lane that owns pair (i, j).  (The cancellation is of the same kind as in D_ij^2
    // itself; pairs closer than pair_tol never get here.)
    const v4d qz = mm16(z, z);
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (isdiag[r]) fm.Zs[c16] = qz[r];                 // diag(Q), one entry per diagonal lane
    wave_fence();
    const double qjj = fm.Zs[c16];
    rhoj = qjj * dj * dj;                                // 1 - v_j
    // sqrt(rho) = rho * rsqrt(rho) and max(rho, delta)^(-1/2) = min(rsqrt(rho), delta^(-1/2)):
    // one reciprocal square root per residual, no division
    double part, wnext;
    if (expo == 0.5) {
      rsj = rsq_nr<2>(rhoj > 1e-300 ? rhoj : 1e-300);
      part = (q4 == 0 && livej) ? rhoj * rsj : 0.0;
      wnext = rsj < rs_delta ? rsj : rs_delta;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const double qii = fm.Zs[4 * r + q4];
        const double dz2 = fma(-2.0, qz[r], qii + qjj);
        const double rho = (dz2 > 0.0 ? dz2 : 0.0) * d2inv[r];
        const bool lp = d2inv[r] > 0.0;
        const double rs = rsq_nr<2>(rho > 1e-300 ? rho : 1e-300);
        part += lp ? coef * (rho * rs) : 0.0;            // ordered pair (i, j)
        cp[r] = lp ? -2.0 * coef * d2inv[r] * (rs < rs_delta ? rs : rs_delta) : 0.0;
      }
    } else {
      // the general exponent: same places, powers instead of square roots (rolled: this code
      // runs once per solve, and five inlined copies of pow() are a thousand instructions)
      part = (q4 == 0 && livej) ? fa_term_pow(rhoj, expo) : 0.0;
      wnext = fa_weight_pow(rhoj, delta, expo);
#pragma unroll 1
      for (int r = 0; r < 4; ++r) {
        const double qii = fm.Zs[4 * r + q4];
        const double qzr = r == 0 ? qz[0] : r == 1 ? qz[1] : r == 2 ? qz[2] : qz[3];
        const double di2 = r == 0 ? d2inv[0] : r == 1 ? d2inv[1] : r == 2 ? d2inv[2] : d2inv[3];
        const double dz2 = fma(-2.0, qzr, qii + qjj);
        const double rho = (dz2 > 0.0 ? dz2 : 0.0) * di2;
        const bool lp = di2 > 0.0;
        part += lp ? coef * fa_term_pow(rho, expo) : 0.0;
        const double cv = lp ? -2.0 * coef * di2 * fa_weight_pow(rho, delta, expo) : 0.0;
        if (r == 0) cp[0] = cv; else if (r == 1) cp[1] = cv; else if (r == 2) cp[2] = cv; else cp[3] = cv;
      }
    }
    wave_fence();
    const double obj = wave_sum(part);
    if (lane == 0 && it0 + it < FA_ITERS_MAX) info->objective[it0 + it] = obj;
    iters_done = it + 1;
    const bool stop = it0 + it > 0 && fabs(prev_obj - obj) < tol;
    prev_obj = obj;
    if (stop) break;
    wj = livej ? wnext : 0.0;
  }

  // ---- epilogue: basis of range(P), A = B U_m, c = A (U_m^T R 1) / p ---------------------
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = 4 * r + q4;
    fm.Ps[i * LDF + c16] = x[r];
    mlast[i * 16 + c16] = mk[r];
  }
  wave_fence();
  // P = U U^T with orthonormal U: the rows produced by the pivoted Cholesky of a projector
  const int nb = pivoted_cholesky(fm.Ps, fm.Um, fm.piv, fm.rinv, 1e-6, mm, lane);
  if (nb != mm) return -2;
  v4d ba, ub;   // B as A operand: B[c16][4s+q4];  U_m as B operand: U[a = 4s+q4][k = c16]
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    ba[s] = fm.Bm[c16 * LDF + 4 * s + q4];
    ub[s] = fm.Um[c16 * LDF + 4 * s + q4];              // Um is stored as rows k: Um[k][a]
  }
  const v4d am = mm16(ba, ub);                           // A[4r+q4][c16]
  if (lane < 16) {
    double a4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int a = 0; a < 16; ++a) a4[a & 3] = fma(fm.Um[lane * LDF + a], fm.r1[a], a4[a & 3]);
    fm.beta[lane] = (a4[0] + a4[1]) + (a4[2] + a4[3]);   // (U_m^T R 1)[k]
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = 4 * r + q4;
    fm.Am[i * LDF + c16] = am[r];
    if (i < p && c16 < m) info->A[i * m + c16] = am[r];
  }
  wave_fence();
  if (lane < 16 && lane < p) {
    double a4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int k = 0; k < 16; ++k) a4[k & 3] = fma(fm.Am[lane * LDF + k], fm.beta[k], a4[k & 3]);
    double acc = (a4[0] + a4[1]) + (a4[2] + a4[3]);
    acc /= (double)p;
    cg[lane] = acc;
    info->c[lane] = acc;
    info->s[lane] = sj;
    info->v[lane] = livej ? 1.0 - rhoj : 0.0;
    info->w[lane] = wj;
  }
  if (lane == 0) {
    info->status = 0;
    info->p = p; info->m = m; info->rank = rank;
    info->iters_done = it0 + iters_done;
    info->sweeps = steps;
    info->eigengap = nan("");        // filled in on demand by fa_get_info (needs eigenvalues)
    mlast[256] = (double)rank;
    mlast[257] = (double)m;
  }
  // weights for the solve that would come next (only once nothing above can fail any more:
  // the Jacobi path restarts from the state as this launch found it)
  if (rs) {
    if (lane < 16 && c16 < p) rs->w[c16] = wj;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = 4 * r + q4;
      if (i < p && c16 < p) rs->cp[i * p + c16] = i != c16 ? cp[r] : 0.0;
    }
    if (lane == 0) { rs->prev_obj = prev_obj; rs->it0 = it0 + iters_done; }
  }
  return 1;
}

}  // namespace fastp

__global__ __launch_bounds__(256) void fa_irls16_kernel(const double* __restrict__ Kg,
                                                        int p, int m, int iters, double lambda,
                                                        double tol, double delta, double expo,
                                                        double rank_tol,
                                                        double pair_tol, double* __restrict__ cg,
                                                        fa_info* __restrict__ info,
                                                        double* __restrict__ mlast,
                                                        int use_purification, fa_resume* rs) {
  __shared__ Smem sm;
  __shared__ fastp::Fmem fm;
  __shared__ int fast_done;
  const int tid = threadIdx.x;
  if (use_purification) {
    if (tid < 64) {
      const int ok = fastp::solve(Kg, p, m, iters, lambda, tol, delta, expo, rank_tol, pair_tol, cg,
                                  info, mlast, fm, rs);
      if (tid == 0) fast_done = ok;
    }
    __syncthreads();
    if (fast_done > 0) return;
  }
  const int ri = tid >> 4, ci = tid & 15;       // this thread's entry of a 16 x 16 matrix
  const double coef = (lambda > 0.0 && p > 1) ? lambda / (double)(p - 1) : 0.0;

  // ---- setup: norms, status, normalised Gram, pairwise distances ------------------------
  if (tid == 0) { sm.sweeps = 0; sm.status = 0; sm.rank = 0; }
  const int it0 = rs ? rs->it0 : 0;
  const bool scaled = rs && rs->scaled;
  if (tid < NP) {
    double si = tid < p ? Kg[tid * p + tid] : 0.0;
    if (tid < p && scaled) si *= rs->uinv[tid] * rs->uinv[tid];
    sm.s[tid] = si;
    sm.dinv[tid] = si > 0.0 ? 1.0 / sqrt(si) : 0.0;
    sm.w[tid] = si > 0.0 ? 1.0 : 0.0;
    sm.v[tid] = 0.0; sm.rho[tid] = 0.0; sm.beta[tid] = 0.0;
  }
  __syncthreads();
  const bool in = ri < p && ci < p;
  double kij = in ? Kg[ri * p + ci] : 0.0;
  if (in && scaled) kij *= rs->uinv[ri] * rs->uinv[ci];
  if (in) info->K[ri * p + ci] = kij;
  {
    const bool bad = !(fabs(kij) <= 1.79e308);
    const bool live = tid < NP && sm.s[tid] > 0.0;
    const int nbad = __syncthreads_or(bad ? 1 : 0);
    const int nlive = __syncthreads_or(live ? 1 : 0);
    if (tid == 0) sm.status = nbad ? 4 : (nlive ? 0 : 5);
    __syncthreads();
  }
  if (sm.status != 0) {
    const int st = sm.status;
    if (tid < p) {
      const double cv = st == 4 ? nan("") : 0.0;
      cg[tid] = cv;
      info->c[tid] = cv; info->s[tid] = sm.s[tid]; info->v[tid] = 0.0; info->w[tid] = 0.0;
    }
    for (int idx = tid; idx < p * m; idx += 256) info->A[idx] = 0.0;
    if (tid == 0) {
      info->status = st; info->p = p; info->m = m; info->rank = 0; info->iters_done = 0;
      info->sweeps = 0; info->eigengap = 0.0;
    }
    return;
  }
  {
    double kt = kij * sm.dinv[ri] * sm.dinv[ci];
    if (ri == ci) kt = sm.s[ri] > 0.0 ? 1.0 : 0.0;
    sm.M[ri * LD + ci] = kt;
    sm.Ut[ri * LD + ci] = ri == ci ? 1.0 : 0.0;
    const double d2 = sm.s[ri] + sm.s[ci] - 2.0 * kij;
    const bool livep = in && ri != ci && d2 > pair_tol * (sm.s[ri] + sm.s[ci]);
    sm.D2inv[ri * LD + ci] = livep ? 1.0 / d2 : 0.0;
    sm.R[ri * LD + ci] = 0.0;
    sm.T[ri * LD + ci] = 0.0;
    sm.Vt[ri * LD + ci] = 0.0;
  }
  __syncthreads();

  // ---- eigen-decomposition of the normalised Gram; rank; R = L^1/2 V^T D^1/2 ------------
  jacobi16(sm, sm.Ut, nullptr, p);
  if (tid < NP) sm.lam0[tid] = tid < p ? sm.mu[sm.order[tid]] : 0.0;   // sorted, descending
  __syncthreads();
  {
    const double lmax = sm.lam0[0];
    const bool cnt = tid < p && sm.lam0[tid] > rank_tol * lmax;
    const int r = __syncthreads_count(cnt ? 1 : 0);
    if (tid == 0) sm.rank = r;
    __syncthreads();
  }
  const int r = sm.rank;
  {
    double vt = 0.0, rv = 0.0;
    if (ri < r && ci < p) {
      vt = sm.Ut[sm.order[ri] * LD + ci];
      rv = sqrt(sm.lam0[ri]) * vt * sqrt(sm.s[ci]);
    }
    __syncthreads();
    sm.Vt[ri * LD + ci] = vt;
    sm.R[ri * LD + ci] = rv;
    sm.Ut[ri * LD + ci] = ri == ci ? 1.0 : 0.0;
  }
  // pair part of C for the first, uniform-weight solve (PCA of the normalised gradients);
  // kept per thread for entry (ri, ci): C_ij = -2 coef w_ij / D_ij^2
  double cpair = (ri != ci) ? -2.0 * coef * sm.D2inv[ri * LD + ci] : 0.0;
  if (it0 > 0) {
    cpair = (in && ri != ci) ? rs->cp[ri * p + ci] : 0.0;
    if (tid < p) sm.w[tid] = sm.s[tid] > 0.0 ? rs->w[tid] : 0.0;
  }
  __syncthreads();

  // ---- IRLS ----------------------------------------------------------------------------
  const int mm = m < r ? m : r;
  double prev_obj = it0 > 0 ? rs->prev_obj : 0.0;
  int iters_done = 0;
  for (int it = 0; it < iters; ++it) {
    // T = R C with the diagonal of C folded in:
    //   T[a][j] = sum_{i != j} (R[a][i] - R[a][j]) C_ij + R[a][j] w_j / s_j
    sm.M[ri * LD + ci] = cpair;        // M's storage carries the pair part of C for a moment
    __syncthreads();
    {
      double acc = 0.0;
      if (ri < r && ci < p) {
        const double rj = sm.R[ri * LD + ci];
#pragma unroll
        for (int i = 0; i < NP; ++i) acc += (sm.R[ri * LD + i] - rj) * sm.M[i * LD + ci];
        acc += rj * sm.w[ci] * sm.dinv[ci] * sm.dinv[ci];
      }
      sm.T[ri * LD + ci] = acc;
    }
    __syncthreads();
    {
      double acc = 0.0;
      if (ri < r && ci < r) {
        const int a = ri < ci ? ri : ci, b = ri < ci ? ci : ri;   // same sum on both sides
#pragma unroll
        for (int j = 0; j < NP; ++j) acc += sm.T[a * LD + j] * sm.R[b * LD + j];
      }
      sm.M[ri * LD + ci] = acc;
    }
    __syncthreads();
    jacobi16(sm, sm.R, sm.Ut, r);

    // explained variances, residuals (the part of g_i outside Y), pair residuals, Eq. 5
    double part = 0.0;
    if (tid < p) {
      double top = 0.0, bot = 0.0;
#pragma unroll
      for (int a = 0; a < NP; ++a) {
        const double x = sm.R[a * LD + tid];
        if (sm.pos[a] < m) top += x * x; else bot += x * x;
      }
      const double d2 = sm.dinv[tid] * sm.dinv[tid];
      sm.v[tid] = top * d2;
      sm.rho[tid] = bot * d2;
      if (sm.s[tid] > 0.0) part += expo == 0.5 ? sqrt(bot * d2) : fa_term_pow(bot * d2, expo);
    }
    cpair = 0.0;
    if (coef > 0.0 && ri != ci) {
      const double dinv2 = sm.D2inv[ri * LD + ci];
      if (dinv2 > 0.0) {
        const int i = ri < ci ? ri : ci, j = ri < ci ? ci : ri;   // same sum for (i,j),(j,i)
        double bot = 0.0;
#pragma unroll
        for (int a = 0; a < NP; ++a) {
          const double x = sm.R[a * LD + i] - sm.R[a * LD + j];
          bot += sm.pos[a] >= m ? x * x : 0.0;
        }
        const double rho = bot * dinv2;
        part += coef * (expo == 0.5 ? sqrt(rho) : fa_term_pow(rho, expo));   // ordered pair (ri, ci)
        cpair = -2.0 * coef * dinv2 *
                (expo == 0.5 ? 1.0 / sqrt(rho > delta ? rho : delta) : fa_weight_pow(rho, delta, expo));
      }
    }
    const double obj = block_sum(part, sm);
    if (tid == 0 && it0 + it < FA_ITERS_MAX) info->objective[it0 + it] = obj;
    iters_done = it + 1;
    const bool stop = it0 + it > 0 && fabs(prev_obj - obj) < tol;
    prev_obj = obj;
    if (stop) break;
    if (tid < p) {
      const double rho = sm.rho[tid];
      sm.w[tid] = sm.s[tid] <= 0.0 ? 0.0
                  : expo == 0.5 ? 1.0 / sqrt(rho > delta ? rho : delta) : fa_weight_pow(rho, delta, expo);
    }
    __syncthreads();
  }
  __syncthreads();
  if (rs) {
    if (in) rs->cp[ri * p + ci] = ri != ci ? cpair : 0.0;
    if (tid < p) rs->w[tid] = sm.w[tid];
    if (tid == 0) { rs->prev_obj = prev_obj; rs->it0 = it0 + iters_done; }
  }

  // ---- epilogue: A = D^-1/2 V L^-1/2 U_m,  c = (1/p) A (Y^T G 1) --------------------------
  if (tid < NP) {
    double acc = 0.0;
    if (tid < mm) {
      const int a = sm.order[tid];
      for (int j = 0; j < p; ++j) acc += sm.R[a * LD + j];
    }
    sm.beta[tid] = acc;
  }
  {
    double tv = 0.0;
    if (ri < mm && ci < r) tv = sm.Ut[sm.order[ri] * LD + ci] / sqrt(sm.lam0[ci]);
    sm.T[ri * LD + ci] = tv;
  }
  __syncthreads();
  {
    // A[i][k], i = ri (worker), k = ci (basis vector)
    double acc = 0.0;
    if (ri < p && ci < mm) {
      for (int b = 0; b < r; ++b) acc += sm.Vt[b * LD + ri] * sm.T[ci * LD + b];
      acc *= sm.dinv[ri];
    }
    sm.M[ri * LD + ci] = acc;
    if (ri < p && ci < m) info->A[ri * m + ci] = acc;
  }
  __syncthreads();
  if (tid < p) {
    double acc = 0.0;
    for (int k = 0; k < mm; ++k) acc += sm.M[tid * LD + k] * sm.beta[k];
    acc /= (double)p;
    cg[tid] = acc;
    info->c[tid] = acc;
    info->s[tid] = sm.s[tid];
    info->v[tid] = sm.v[tid];
    info->w[tid] = sm.w[tid];
  }
  if (tid == 0) {
    info->status = 0;
    info->p = p; info->m = m; info->rank = r;
    info->iters_done = it0 + iters_done;
    info->sweeps = sm.sweeps;
    double gap = __builtin_inf();
    if (m < r) gap = (sm.mu[sm.order[m - 1]] - sm.mu[sm.order[m]]) / sm.mu[sm.order[0]];
    info->eigengap = gap;
  }
}

hipError_t fa_launch_irls16(const double* Kd, int p, int m, double lambda, int iters, double tol,
                            double delta, double exponent_a, double rank_tol, double pair_tol,
                            double* cd,
                            fa_info* info_d, double* mlast, int use_purification,
                            fa_resume* rs, hipStream_t st, const fa_ktime* tm) {
  FA_LAUNCH(tm, fa_irls16_kernel, dim3(1), dim3(256), 0, st, Kd, p, m, iters, lambda, tol, delta,
            exponent_a == 2.0 ? 0.5 : 1.0 / exponent_a, rank_tol, pair_tol, cd, info_d, mlast,
            use_purification, rs);
  return hipGetLastError();
}
