// Host build of the library's p x p solver text (csrc/fa_irls_core.inc) as a plain
// sequential program: one "thread", barriers are no-ops.  TEST-ONLY: it lets the CPU test
// suite check the solver's logic (phases, indexing, Jacobi ordering) against the oracle
// without a GPU.  The shipped library never contains or calls this build.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "fa.h"
#include "fa_resume.h"

#define FA_FN static
#define FA_TID 0
#define FA_NT 1
#define FA_FOR(i, n) for (int i = 0; i < (n); ++i)
#define FA_SYNC() ((void)0)
#include "fa_irls_core.inc"

// launches = 1: the whole IRLS in one call of the solver.  launches > 1: the same IRLS driven
// one solve per call through the resume state, as the re-streaming schedule drives it.
static int emulate(const double* K, int p, int m, double lambda, int iters, double tol,
                   double delta, double rank_tol, double pair_tol, double* c, fa_info* info,
                   int stepwise, double a, int nworkers = 0, const int* sizes = 0) {
  if (p < 1 || p > FA_P_MAX || m < 1 || m > p || iters < 1 || iters > FA_ITERS_MAX) return 1;
  const int ld = p | 1;
  const size_t msz = (size_t)p * ld;
  double* buf = (double*)calloc(6 * msz + 20 * FA_P_MAX + 8, sizeof(double));
  int* ibuf = (int*)calloc(10 * FA_P_MAX + 16, sizeof(int));
  if (!buf || !ibuf) return 2;
  fa_irls_mem sm;
  sm.ld = ld;
  double* q = buf;
  sm.R = q; q += msz; sm.Ut = q; q += msz; sm.CM = q; q += msz; sm.T = q; q += msz;
  sm.D2inv = q; q += msz; sm.Vt = q; q += msz;
  sm.s = q; q += FA_P_MAX; sm.dinv = q; q += FA_P_MAX; sm.w = q; q += FA_P_MAX;
  sm.rho = q; q += FA_P_MAX; sm.v = q; q += FA_P_MAX; sm.lam0 = q; q += FA_P_MAX;
  sm.mu = q; q += FA_P_MAX; sm.beta = q; q += FA_P_MAX;
  sm.ginv = q; q += FA_P_MAX; sm.ctop = q; q += FA_P_MAX; sm.cbot = q; q += FA_P_MAX;
  sm.rot_c = q; q += FA_P_MAX; sm.rot_s = q; q += FA_P_MAX; sm.red = q; q += 8;
  int* qi = ibuf;
  sm.rot_p = qi; qi += FA_P_MAX; sm.rot_q = qi; qi += FA_P_MAX; sm.pos = qi; qi += FA_P_MAX;
  sm.order = qi; qi += FA_P_MAX; sm.gfirst = qi; qi += FA_P_MAX; sm.gcnt = qi; qi += FA_P_MAX;
  sm.flag = qi; qi += 8;
  fa_irls_args ar;
  ar.p = p; ar.m = m; ar.iters = iters; ar.lambda = lambda; ar.tol = tol; ar.delta = delta;
  ar.rank_tol = rank_tol; ar.pair_tol = pair_tol; ar.expo = 1.0 / a;
  ar.nworkers = nworkers; ar.sizes = sizes;
  memset(info, 0, sizeof(*info));
  if (!stepwise) {
    fa_irls_solve(K, ar, sm, c, info, (fa_resume*)0);
  } else {
    fa_resume* rs = (fa_resume*)calloc(1, sizeof(fa_resume));
    if (!rs) return 2;
    ar.iters = 1;
    for (int it = 0; it < iters; ++it) {
      fa_irls_solve(K, ar, sm, c, info, rs);
      if (info->iters_done < it + 1) break;   // cannot happen: one solve per call
      if (it > 0 && tol > 0.0 && fabs(info->objective[it - 1] - info->objective[it]) < tol) break;
    }
    free(rs);
  }
  free(buf); free(ibuf);
  return 0;
}

extern "C" int fa_irls_emulate(const double* K, int p, int m, double lambda, int iters, double tol,
                               double delta, double rank_tol, double pair_tol, double* c,
                               fa_info* info) {
  return emulate(K, p, m, lambda, iters, tol, delta, rank_tol, pair_tol, c, info, 0, 2.0);
}

extern "C" int fa_irls_emulate_stepwise(const double* K, int p, int m, double lambda, int iters,
                                        double tol, double delta, double rank_tol,
                                        double pair_tol, double* c, fa_info* info) {
  return emulate(K, p, m, lambda, iters, tol, delta, rank_tol, pair_tol, c, info, 1, 2.0);
}

extern "C" int fa_irls_emulate_exponent(const double* K, int p, int m, double lambda, int iters,
                                        double tol, double delta, double rank_tol,
                                        double pair_tol, double a, double* c, fa_info* info) {
  return emulate(K, p, m, lambda, iters, tol, delta, rank_tol, pair_tol, c, info, 0, a);
}

// workers that send several gradients: p columns in nworkers blocks of sizes[i] columns
extern "C" int fa_irls_emulate_grouped(const double* K, int p, const int* sizes, int nworkers,
                                       int m, double lambda, int iters, double tol, double delta,
                                       double rank_tol, double pair_tol, double* c,
                                       fa_info* info) {
  int tot = 0;
  for (int i = 0; i < nworkers; ++i) { if (sizes[i] < 1) return 1; tot += sizes[i]; }
  if (nworkers < 1 || tot != p) return 1;
  return emulate(K, p, m, lambda, iters, tol, delta, rank_tol, pair_tol, c, info, 0, 2.0,
                 nworkers, sizes);
}
