// K3 for p <= 16: the p x p part of the Flag Aggregator (normalisation, IRLS by repeated
// weighted PCA, coefficients) as one 256-thread workgroup with a latency-tuned Jacobi.
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

__device__ __forceinline__ double rsq_nr(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double hx = 0.5 * x;
  double e = fma(-hx * y, y, 0.5);
  y = fma(y, e, y);
  e = fma(-hx * y, y, 0.5);
  y = fma(y, e, y);
  return y;
}

// Plane rotation zeroing A_pq:  x_p' = c x_p - s x_q,  x_q' = s x_p + c x_q.
// *big: the off-diagonal entry exceeded 1e-9 relative to sqrt(|A_pp A_qq|).
__device__ __forceinline__ void rotation(double app, double aqq, double apq, double* c, double* s,
                                         bool* active, bool* big) {
  const double dd = fabs(app * aqq);
  const double o2 = apq * apq;
  const bool act = (o2 > 1e-30 * dd) && (fabs(apq) > 1e-300);
  const double zeta = aqq - app;
  const double nn = zeta < 0.0 ? -2.0 * apq : 2.0 * apq;
  const double h2 = fma(zeta, zeta, 4.0 * o2);
  const double h = h2 * rsq_nr(act ? h2 : 1.0);
  const double dn = fabs(zeta) + h;
  const double wn = rsq_nr(act ? fma(dn, dn, nn * nn) : 1.0);
  *c = act ? dn * wn : 1.0;
  *s = act ? nn * wn : 0.0;
  *active = act;
  *big = act && (o2 > 1e-18 * dd);
}

__device__ __forceinline__ void pair_of(int round, int t, int* p, int* q) {
  int a, b;
  if (t == 0) {
    a = NP - 1; b = round;
  } else {
    a = round + t; if (a >= NP - 1) a -= NP - 1;
    b = round - t; if (b < 0) b += NP - 1;
  }
  *p = a < b ? a : b;
  *q = a < b ? b : a;
}

__device__ __forceinline__ void wave_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// One sweep by the master wavefront (all 64 lanes of wave 0).  Returns true when the sweep
// made M diagonal to working precision (nothing above 1e-9 relative was met).
__device__ bool master_sweep(double* M, Rot (*lg)[NPAIR], int lane) {
  const int t = lane >> 3, u = lane & 7;
  bool big = false, any = false;
  for (int round = 0; round < NROUND; ++round) {
    int p0, q0, p1, q1;
    pair_of(round, t, &p0, &q0);
    pair_of(round, u, &p1, &q1);
    const double app0 = M[p0 * LD + p0], aqq0 = M[q0 * LD + q0], apq0 = M[p0 * LD + q0];
    const double app1 = M[p1 * LD + p1], aqq1 = M[q1 * LD + q1], apq1 = M[p1 * LD + q1];
    const double b00 = M[p0 * LD + p1], b01 = M[p0 * LD + q1];
    const double b10 = M[q0 * LD + p1], b11 = M[q0 * LD + q1];
    double c0, s0, c1, s1;
    bool a0, a1, g0, g1;
    rotation(app0, aqq0, apq0, &c0, &s0, &a0, &g0);
    rotation(app1, aqq1, apq1, &c1, &s1, &a1, &g1);
    const bool round_active = __ballot(a0 || a1) != 0ull;
    big = big || (__ballot(g0 || g1) != 0ull);
    any = any || round_active;
    if (u == 0) {
      Rot e;
      e.c = c0; e.s = s0; e.p = p0; e.q = q0; e.active = a0 ? 1 : 0; e.pad = 0;
      lg[round][t] = e;
    }
    if (round_active) {
      const double x00 = c0 * b00 - s0 * b10, x01 = c0 * b01 - s0 * b11;
      const double x10 = s0 * b00 + c0 * b10, x11 = s0 * b01 + c0 * b11;
      double d00 = c1 * x00 - s1 * x01, d01 = s1 * x00 + c1 * x01;
      double d10 = c1 * x10 - s1 * x11, d11 = s1 * x10 + c1 * x11;
      if (t == u && a0) { d01 = 0.0; d10 = 0.0; }
      M[p0 * LD + p1] = d00; M[p0 * LD + q1] = d01;
      M[q0 * LD + p1] = d10; M[q0 * LD + q1] = d11;
    }
    wave_fence();
  }
  return !any || !big;
}

// Replay one sweep's log on the rows of X (16 columns) by one wavefront.
__device__ void replay_sweep(double* X, const Rot (*lg)[NPAIR], int lane) {
  for (int round = 0; round < NROUND; ++round) {
#pragma unroll
    for (int k = lane; k < NPAIR * NP; k += 64) {
      const int t = k >> 4, j = k & 15;
      const Rot e = lg[round][t];
      if (e.active) {
        const double x = X[e.p * LD + j], y = X[e.q * LD + j];
        X[e.p * LD + j] = e.c * x - e.s * y;
        X[e.q * LD + j] = e.s * x + e.c * y;
      }
    }
    wave_fence();
  }
}

// Diagonalise sm.M (16 x 16, live part in the leading block) and apply the same rotations
// to the rows of XA (by wave 1) and XB (by wave 2); either may be null.  Leaves pos/order
// (descending eigenvalues of the first `nlive` diagonal entries) in sm.pos / sm.order.
__device__ void jacobi16(Smem& sm, double* XA, double* XB, int nlive) {
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
__device__ double block_sum(double x, Smem& sm) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.red[threadIdx.x >> 6] = x;
  __syncthreads();
  return ((sm.red[0] + sm.red[1]) + sm.red[2]) + sm.red[3];
}

}  // namespace

__global__ __launch_bounds__(256) void fa_irls16_kernel(const double* __restrict__ Kg,
                                                        int p, int m, int iters, double lambda,
                                                        double tol, double delta, double rank_tol,
                                                        double pair_tol, double* __restrict__ cg,
                                                        fa_info* __restrict__ info) {
  __shared__ Smem sm;
  const int tid = threadIdx.x;
  const int ri = tid >> 4, ci = tid & 15;       // this thread's entry of a 16 x 16 matrix
  const double coef = (lambda > 0.0 && p > 1) ? lambda / (double)(p - 1) : 0.0;

  // ---- setup: norms, status, normalised Gram, pairwise distances ------------------------
  if (tid == 0) { sm.sweeps = 0; sm.status = 0; sm.rank = 0; }
  if (tid < NP) {
    const double si = tid < p ? Kg[tid * p + tid] : 0.0;
    sm.s[tid] = si;
    sm.dinv[tid] = si > 0.0 ? 1.0 / sqrt(si) : 0.0;
    sm.w[tid] = si > 0.0 ? 1.0 : 0.0;
    sm.v[tid] = 0.0; sm.rho[tid] = 0.0; sm.beta[tid] = 0.0;
  }
  __syncthreads();
  const bool in = ri < p && ci < p;
  const double kij = in ? Kg[ri * p + ci] : 0.0;
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
  __syncthreads();

  // ---- IRLS ----------------------------------------------------------------------------
  const int mm = m < r ? m : r;
  double prev_obj = 0.0;
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
        for (int i = 0; i < p; ++i) acc += (sm.R[ri * LD + i] - rj) * sm.M[i * LD + ci];
        acc += rj * sm.w[ci] * sm.dinv[ci] * sm.dinv[ci];
      }
      sm.T[ri * LD + ci] = acc;
    }
    __syncthreads();
    {
      double acc = 0.0;
      if (ri < r && ci < r) {
        const int a = ri < ci ? ri : ci, b = ri < ci ? ci : ri;   // same sum on both sides
        for (int j = 0; j < p; ++j) acc += sm.T[a * LD + j] * sm.R[b * LD + j];
      }
      sm.M[ri * LD + ci] = acc;
    }
    __syncthreads();
    jacobi16(sm, sm.R, sm.Ut, r);

    // explained variances, residuals (the part of g_i outside Y), pair residuals, Eq. 5
    double part = 0.0;
    if (tid < p) {
      double top = 0.0, bot = 0.0;
      for (int a = 0; a < r; ++a) {
        const double x = sm.R[a * LD + tid];
        if (sm.pos[a] < m) top += x * x; else bot += x * x;
      }
      const double d2 = sm.dinv[tid] * sm.dinv[tid];
      sm.v[tid] = top * d2;
      sm.rho[tid] = bot * d2;
      if (sm.s[tid] > 0.0) part += sqrt(bot * d2);
    }
    cpair = 0.0;
    if (coef > 0.0 && ri != ci) {
      const double dinv2 = sm.D2inv[ri * LD + ci];
      if (dinv2 > 0.0) {
        const int i = ri < ci ? ri : ci, j = ri < ci ? ci : ri;   // same sum for (i,j),(j,i)
        double bot = 0.0;
        for (int a = 0; a < r; ++a)
          if (sm.pos[a] >= m) {
            const double x = sm.R[a * LD + i] - sm.R[a * LD + j];
            bot += x * x;
          }
        const double rho = bot * dinv2;
        part += coef * sqrt(rho);                  // ordered pair (ri, ci)
        cpair = -2.0 * coef * dinv2 / sqrt(rho > delta ? rho : delta);
      }
    }
    const double obj = block_sum(part, sm);
    if (tid == 0) info->objective[it] = obj;
    iters_done = it + 1;
    const bool stop = it > 0 && fabs(prev_obj - obj) < tol;
    prev_obj = obj;
    if (stop) break;
    if (tid < p) {
      const double rho = sm.rho[tid];
      sm.w[tid] = sm.s[tid] > 0.0 ? 1.0 / sqrt(rho > delta ? rho : delta) : 0.0;
    }
    __syncthreads();
  }
  __syncthreads();

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
    info->iters_done = iters_done;
    info->sweeps = sm.sweeps;
    double gap = __builtin_inf();
    if (m < r) gap = (sm.mu[sm.order[m - 1]] - sm.mu[sm.order[m]]) / sm.mu[sm.order[0]];
    info->eigengap = gap;
  }
}

hipError_t fa_launch_irls16(const double* Kd, int p, int m, double lambda, int iters, double tol,
                            double delta, double rank_tol, double pair_tol, double* cd,
                            fa_info* info_d, hipStream_t st) {
  hipLaunchKernelGGL(fa_irls16_kernel, dim3(1), dim3(256), 0, st, Kd, p, m, iters, lambda, tol,
                     delta, rank_tol, pair_tol, cd, info_d);
  return hipGetLastError();
}
