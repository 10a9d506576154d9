// Internal interface between the C ABI (fa_api.hip) and the kernel launchers
// (fa_kernels.hip).  Not installed; include/fa.h is the public header.
#ifndef FA_INTERNAL_H_
#define FA_INTERNAL_H_

#include <hip/hip_runtime_api.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "fa.h"
#include "fa_resume.h"

#define FA_IRLS_THREADS 256   // workgroup size of the p x p solver
#define FA_ST_RETRY (-1)      // device-side status: the matrix-core solver gave up, run Jacobi

// layout of the p x p solvers' global workspace (doubles)
#define FA_GWS_GENERIC (2 * FA_P_MAX * (FA_P_MAX + 1))    // any-p Jacobi kernel: D2inv, Vt
// 16 < p <= 64 matrix-core kernel: three matrices as (p_max/16)^2 tiles of 272 doubles
#define FA_GWS_TILES (3 * (FA_P_MAX / 16) * (FA_P_MAX / 16) * 272)
#define FA_GWS_MLAST_OFF (FA_GWS_GENERIC + FA_GWS_TILES)  // last weighted-PCA matrix N x N, rank, m
#define FA_GWS_DOUBLES (FA_GWS_MLAST_OFF + FA_P_MAX * FA_P_MAX + 2)

// Optional per-kernel timing: when a launcher gets a non-null fa_ktime, the kernel is
// launched with these events attached to the dispatch itself (they carry the kernel's own
// begin/end timestamps; no marker packets are put between the kernels).
typedef struct { hipEvent_t start, stop; } fa_ktime;
#define FA_GRAM_WAVES_PER_CU 16 // most wavefronts a Gram workgroup (one per compute unit) has

// K1: partial Grams of G, one per launched workgroup, into `partials` (up to max_blocks *
// T(T+1)/2 * 256 doubles, T = ceil(p/16)); max_blocks = workgroups (one per compute unit);
// *nparts receives how many partials were written.  layout: fa_layout (for FA_ROW_MAJOR ldg is
// the row pitch in elements, p <= ldg <= 16 ceil(p/16)).  gram_mode: fa_gram_mode
// (FA_GRAM_BF16_MATRIX, and FA_GRAM_AUTO from FA_GRAM_AUTO_MIN_ROWS rows on, hand the cases of
// fa_gram_lp_applies to the bf16 matrix-core kernel).
// gate (device, may be null): the pass does nothing unless *gate != 0 (fp64 kernel only).
hipError_t fa_launch_gram_partials(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                   int layout, int gram_mode, int max_blocks, double* partials,
                                   int* nparts, hipStream_t st, const fa_ktime* tm,
                                   const int* gate = nullptr);
// whether that call hands the pass to the bf16 matrix-core kernel
bool fa_gram_takes_matrix_core(int p, int64_t n, int dtype, int layout, int gram_mode);
// K1 + K2 into Kd, with the fp64 pass standing by behind a matrix-core pass in case its fp32
// sums overflowed (flag_d: one int of device scratch; see fa_kernels.hip).
hipError_t fa_launch_gram(const void* G, int64_t ldg, int p, int64_t n, int dtype, int layout,
                          int gram_mode, int max_blocks, double* partials, double* Kd,
                          int* flag_d, int* nparts, hipStream_t st, const fa_ktime* tm_gram,
                          const fa_ktime* tm_reduce);
// K1 on the bf16 matrix core (fa_gram_lp.hip): same partials, for worker-major G without
// column scales, where fa_gram_lp_applies (bf16 storage, or fp32 storage at p > 16).
bool fa_gram_lp_applies(int p, int dtype);
hipError_t fa_launch_gram_lp_partials(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                      int max_blocks, double* partials, int* nparts,
                                      hipStream_t st, const fa_ktime* tm);
hipError_t fa_gram_lp_prepare(void);
// Row and column i of K from one pass over n rows of gradient i and of the gradients that
// hold those rows too (bit j of `resident` set; i itself is always included): K[i][j] and
// K[j][i] += g_i . g_j over those rows, in fp64.  G points at the first of the rows in gradient
// 0.  partials: max_parts * FA_ROW_JB doubles of scratch.  Worker-major G.
#define FA_ROW_JB 16          // gradients paired with gradient i in one pass
hipError_t fa_launch_gram_row(const void* G, int64_t ldg, int p, int64_t n, int dtype, int i,
                              uint64_t resident, double* partials, int max_parts, double* Kd,
                              hipStream_t st);
hipError_t fa_launch_zero(double* dst, int count, hipStream_t st);
// K2: their fixed-order sum into Kd (p*p doubles, row-major).  colscale (device, p doubles,
// may be null): entry (i, j) is multiplied by colscale[i] colscale[j], i.e. the result is
// diag(u) K diag(u), the Gram matrix of the columns scaled by u.
hipError_t fa_launch_gram_reduce(const double* partials, int nparts, int p, double* Kd,
                                 const double* colscale, hipStream_t st, const fa_ktime* tm,
                                 const int* gate = nullptr);

// K3: p x p solver.  Kd p*p doubles; cd p doubles out; info_d device fa_info; gws global
// workspace of FA_GWS_DOUBLES doubles.  solver: 0 = default (matrix-core purification, with
// the Jacobi solvers as fallback), 1 = p <= 16 Jacobi path, 2 = any-p Jacobi kernel.
// Every solver takes any exponent_a > 1 (the constant a of Sec. 2.2 Step 2).
// spin_budget: see fa_config.wide_spin_budget.
// rs (device, may be null): continue the IRLS from the weights left there by an earlier
// launch and leave the next ones (see fa_resume.h).
hipError_t fa_launch_irls(const double* Kd, int p, int m, double lambda, int iters, double tol,
                          double delta, double rank_tol, double pair_tol, double exponent_a,
                          double* cd,
                          fa_info* info_d, double* gws, int solver, int spin_budget,
                          fa_resume* rs, hipStream_t st, const fa_ktime* tm);
hipError_t fa_launch_irls_grouped(const double* Kd, int q, int nworkers, const int* sizes_d, int m,
                                  double lambda, int iters, double tol, double delta,
                                  double rank_tol, double pair_tol, double exponent_a, double* cd,
                                  fa_info* info_d, double* gws, int solver, int spin_budget,
                                  hipStream_t st);
// Launch attributes (dynamic LDS above the default limit) of every kernel that needs them, on
// the current device; called by fa_create.
hipError_t fa_kernels_prepare(void);
hipError_t fa_irls64_prepare(void);
// One term of the objective, residual^(1/a), and the weight the majorisation step gives it,
// max(residual, delta)^(1/a - 1), for the constant a of Sec. 2.2 Step 2 (expo = 1/a; a = 2,
// expo = 1/2, is Eq. 5 and has its own square-root code in the matrix-core solvers).
__device__ __forceinline__ double fa_term_pow(double rho, double expo) {
  return rho > 0.0 ? pow(rho, expo) : 0.0;
}
__device__ __forceinline__ double fa_weight_pow(double rho, double delta, double expo) {
  return pow(rho > delta ? rho : delta, expo - 1.0);
}

// K3 for p <= 16 (latency-tuned single-workgroup solver, static LDS).
// mlast: 258 doubles; the fast path leaves the last weighted-PCA matrix there (16 x 16, then
// rank and m) for fa_launch_gap.  use_purification = 0 forces the Jacobi path.  exponent_a:
// the constant a of Sec. 2.2 Step 2 (terms residual^(1/a); 2 is Eq. 5).
hipError_t fa_launch_irls16(const double* Kd, int p, int m, double lambda, int iters, double tol,
                            double delta, double exponent_a, double rank_tol, double pair_tol,
                            double* cd,
                            fa_info* info_d, double* mlast, int use_purification,
                            fa_resume* rs, hipStream_t st, const fa_ktime* tm);
// K3 for 16 < p <= 64 (sixteen wavefronts, tiled matrix-core products).  tiles_ws:
// FA_GWS_TILES doubles; mlast as above with N = 16 ceil(p/16).  May leave
// info_d->status = FA_ST_RETRY, in which case the any-p kernel must run next.  exponent_a as
// for fa_launch_irls16.  nworkers > 0: the p columns are nworkers blocks of sizes_d[i]
// consecutive columns (device memory), one block per worker; then any p <= 64 is taken.
// nworkers = 0: one column per worker, 16 < p <= 64 only.
hipError_t fa_launch_irls64(const double* Kd, int p, int nworkers, const int* sizes_d, int m,
                            double lambda, int iters, double tol, double delta, double exponent_a,
                            double rank_tol, double pair_tol, double* cd, fa_info* info_d,
                            double* tiles_ws, double* mlast, int spin_budget, fa_resume* rs,
                            hipStream_t st, const fa_ktime* tm);
// eigengap (mu_m - mu_{m+1}) / mu_1 of the N x N matrix left in mlast (then rank, m), into
// info_d->eigengap.
hipError_t fa_launch_gap(const double* mlast, int N, fa_info* info_d, hipStream_t st);

// K5: partial results of P = G^T (G A) (p x m), A row-major p x m in device memory; one
// partial of ceil(p/16) * ceil(m/16) * 256 doubles per workgroup; then their fixed-order sum
// into Pd (p*m doubles, row-major).
hipError_t fa_launch_proj_partials(const void* G, int64_t ldg, int p, int m, int64_t n, int dtype,
                                   int max_blocks, const double* Acoef, double* partials,
                                   int* nparts, hipStream_t st, const fa_ktime* tm);
hipError_t fa_launch_proj_reduce(const double* partials, int nparts, int p, int m, double* Pd,
                                 hipStream_t st, const fa_ktime* tm);
// K6: IRLS weights, objective and next column scales from the streamed projections.
hipError_t fa_launch_restream_weights(const fa_info* info_d, const double* Pd, int p, int m,
                                      double lambda, double delta, double pair_tol,
                                      double exponent_a, fa_resume* rs, hipStream_t st);

// K4: out = sum_i c[i*cstride] g_i.
hipError_t fa_launch_combine(const void* G, int64_t ldg, int p, int64_t n, int dtype, int layout,
                             const double* c, int cstride, float* out, int max_blocks,
                             hipStream_t st, const fa_ktime* tm);

// Y = G A, eight columns per pass over G (either layout): column a of Y at Y + a*ldy.
hipError_t fa_launch_combine_multi(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                   int layout, const double* A, int m, float* Y, int64_t ldy,
                                   int max_blocks, hipStream_t st);
// Multi-Krum in p-space: coefficients (1/q on the q selected workers), scores and the 0/1
// selection from the Gram matrix; f = Byzantine workers provided for (p - f - 2 >= 1).
hipError_t fa_launch_krum(const double* Kd, int p, int f, int q, double* cd, double* scores_d,
                          int* selected_d, hipStream_t st);
// Streamed check of a basis: W = Y^T [Y | G] (m rows, 16 ceil(m/16) + p columns, row-major).
hipError_t fa_launch_cross(const float* Y, int64_t ldy, int m, const void* G, int64_t ldg, int p,
                           int64_t n, int dtype, int layout, int max_parts, double* partials,
                           double* Wd, hipStream_t st);

#define FA_LAUNCH(tm, kern, grid, block, lds, st, ...)                                          \
  do {                                                                                           \
    if (tm)                                                                                      \
      hipExtLaunchKernelGGL(kern, grid, block, lds, st, (tm)->start, (tm)->stop, 0, __VA_ARGS__); \
    else                                                                                         \
      hipLaunchKernelGGL(kern, grid, block, lds, st, __VA_ARGS__);                               \
  } while (0)

#endif
