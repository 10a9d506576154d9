// C ABI of the Flag Aggregator library (see include/fa.h): argument checking, workspace
// ownership, and the order in which the kernels are enqueued.  No arithmetic happens here.
#include <hip/hip_runtime.h>

#include <math.h>
#include <pthread.h>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "fa.h"
#include "fa_internal.h"

struct fa_ctx {
  int device;
  hipStream_t stream;
  fa_config cfg;
  int num_cus;
  int gram_max_blocks;
  int combine_max_blocks;
  double* partials;   // gram_max_blocks * 2 ceil(p_max/16)^2 * 256
  double* Kd;         // FA_P_MAX^2
  double* cd;         // FA_P_MAX
  double* gws;        // FA_GWS_DOUBLES: the p x p solvers' global workspace
  fa_info* info_d;
  int has_solution;   // info_d holds an A from a completed fa_aggregate / fa_irls
  int last_p, last_m;
  int profiling;
  fa_resume* rs_d;    // IRLS state of the re-streaming schedule
  double* Pd;         // streamed projections, FA_P_MAX^2
  int* sizes_d;       // FA_P_MAX: block widths of fa_aggregate_grouped
  int* flag_d;        // "the matrix-core Gram pass overflowed" (read by its fp64 stand-by)
  double* check_h;    // pinned host staging of fa_check_basis: FA_P_MAX * 2 FA_P_MAX doubles
  fa_ktime tm[4];     // per-kernel begin/end events (profiling)
  fa_ktime tm_r[2];   // re-streaming schedule: weighted Gram pass and projection pass of the
                      // last iteration
  int ev_recorded_r;
  int ev_recorded;
  int last_nparts;    // partial Grams written by the last Gram pass
  int arr_p;          // fa_gram_begin: gradients expected this round (0: no round open)
  int64_t arr_n;
  uint64_t arrived;   // bit j: gradient j is complete
  int64_t arr_rows[FA_P_MAX];   // rows of gradient j announced so far (a prefix)
};

static int elem_size(int dtype) { return dtype == FA_F32 ? 4 : 2; }

extern "C" void fa_default_config(fa_config* cfg) {
  if (!cfg) return;
  cfg->n_max = 0;
  cfg->p_max = FA_P_MAX;
  cfg->dtype = FA_F32;
  cfg->stream = nullptr;
  cfg->clamp_delta = 1e-6;
  cfg->rank_tol = 1e-12;
  cfg->pair_tol = 1e-12;
  cfg->exponent_a = 2.0;
  cfg->layout = FA_WORKER_MAJOR;
  cfg->solver = FA_SOLVER_AUTO;
  cfg->wide_spin_budget = 1 << 22;
  cfg->gram = FA_GRAM_AUTO;
}

extern "C" const char* fa_status_string(fa_status s) {
  switch (s) {
    case FA_OK: return "ok";
    case FA_ERR_ARG: return "invalid argument";
    case FA_ERR_ALLOC: return "allocation failed";
    case FA_ERR_DEVICE: return "HIP call failed";
    case FA_ERR_NONFINITE: return "input holds NaN or Inf";
    case FA_ERR_ZERO_INPUT: return "all gradients are zero";
    case FA_ERR_TOO_LARGE: return "p exceeds FA_STATIC_P_MAX, the limit of the static workspace";
  }
  return "unknown status";
}

extern "C" const char* fa_version(void) { return "fa-mi355x 0.1 (gfx950)"; }

extern "C" fa_status fa_create(const fa_config* cfg, fa_ctx** out_ctx) {
  if (!cfg || !out_ctx) return FA_ERR_ARG;
  *out_ctx = nullptr;
  if (cfg->n_max < 1 || cfg->p_max < 1 || cfg->p_max > FA_P_MAX) return FA_ERR_ARG;
  if (cfg->dtype != FA_F32 && cfg->dtype != FA_BF16) return FA_ERR_ARG;
  if (cfg->layout != FA_WORKER_MAJOR && cfg->layout != FA_ROW_MAJOR) return FA_ERR_ARG;
  if (cfg->solver < FA_SOLVER_AUTO || cfg->solver > FA_SOLVER_JACOBI) return FA_ERR_ARG;
  if (cfg->wide_spin_budget < 0) return FA_ERR_ARG;
  if (cfg->gram != FA_GRAM_AUTO && cfg->gram != FA_GRAM_FP64 && cfg->gram != FA_GRAM_BF16_MATRIX)
    return FA_ERR_ARG;
  if (!(cfg->clamp_delta > 0.0) || !(cfg->rank_tol >= 0.0) || !(cfg->pair_tol >= 0.0) ||
      !(cfg->exponent_a >= 1.0) || !(cfg->exponent_a <= 1e6))
    return FA_ERR_ARG;
  fa_ctx* c = new (std::nothrow) fa_ctx;
  if (!c) return FA_ERR_ALLOC;
  memset(c, 0, sizeof(*c));
  c->cfg = *cfg;
  c->stream = (hipStream_t)cfg->stream;
  if (hipGetDevice(&c->device) != hipSuccess) { delete c; return FA_ERR_DEVICE; }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, c->device) != hipSuccess) { delete c; return FA_ERR_DEVICE; }
  c->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  c->gram_max_blocks = c->num_cus;                 // one Gram workgroup per compute unit
  c->combine_max_blocks = 1 << 20;
  const int T = (cfg->p_max + 15) / 16;
  // per workgroup: tile pairs of the Gram pass, T x TM tiles of the projections (<= T^2), and a
  // tile row of the basis check, up to T x 2T tiles
  const size_t ntp = (size_t)2 * T * T;
  const size_t part_bytes = (size_t)c->gram_max_blocks * ntp * 256 * sizeof(double);
  bool ok = true;
  ok = ok && hipMalloc((void**)&c->partials, part_bytes) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->Kd, sizeof(double) * FA_P_MAX * FA_P_MAX) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->cd, sizeof(double) * (FA_P_MAX + 8)) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->gws, sizeof(double) * FA_GWS_DOUBLES) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->info_d, sizeof(fa_info)) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->rs_d, sizeof(fa_resume)) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->Pd, sizeof(double) * FA_P_MAX * FA_P_MAX) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->sizes_d, sizeof(int) * FA_P_MAX) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->flag_d, 64) == hipSuccess;
  ok = ok && hipHostMalloc((void**)&c->check_h, sizeof(double) * FA_P_MAX * 2 * FA_P_MAX,
                           hipHostMallocDefault) == hipSuccess;
  if (!ok) { fa_destroy(c); return FA_ERR_ALLOC; }
  if (hipMemset(c->info_d, 0, sizeof(fa_info)) != hipSuccess) { fa_destroy(c); return FA_ERR_DEVICE; }
  for (int i = 0; i < 4; ++i)
    if (hipEventCreate(&c->tm[i].start) != hipSuccess ||
        hipEventCreate(&c->tm[i].stop) != hipSuccess) { fa_destroy(c); return FA_ERR_DEVICE; }
  for (int i = 0; i < 2; ++i)
    if (hipEventCreate(&c->tm_r[i].start) != hipSuccess ||
        hipEventCreate(&c->tm_r[i].stop) != hipSuccess) { fa_destroy(c); return FA_ERR_DEVICE; }
  // per-function launch attributes (large dynamic LDS) on this context's device
  if (fa_kernels_prepare() != hipSuccess || fa_irls64_prepare() != hipSuccess ||
      fa_gram_lp_prepare() != hipSuccess) {
    fa_destroy(c);
    return FA_ERR_DEVICE;
  }
  *out_ctx = c;
  return FA_OK;
}

extern "C" void fa_destroy(fa_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  if (c->partials) (void)hipFree(c->partials);
  if (c->Kd) (void)hipFree(c->Kd);
  if (c->cd) (void)hipFree(c->cd);
  if (c->gws) (void)hipFree(c->gws);
  if (c->info_d) (void)hipFree(c->info_d);
  if (c->rs_d) (void)hipFree(c->rs_d);
  if (c->Pd) (void)hipFree(c->Pd);
  if (c->sizes_d) (void)hipFree(c->sizes_d);
  if (c->flag_d) (void)hipFree(c->flag_d);
  if (c->check_h) (void)hipHostFree(c->check_h);
  for (int i = 0; i < 4; ++i) {
    if (c->tm[i].start) (void)hipEventDestroy(c->tm[i].start);
    if (c->tm[i].stop) (void)hipEventDestroy(c->tm[i].stop);
  }
  for (int i = 0; i < 2; ++i) {
    if (c->tm_r[i].start) (void)hipEventDestroy(c->tm_r[i].start);
    if (c->tm_r[i].stop) (void)hipEventDestroy(c->tm_r[i].stop);
  }
  delete c;
}

extern "C" fa_status fa_set_stream(fa_ctx* c, void* stream) {
  if (!c) return FA_ERR_ARG;
  c->stream = (hipStream_t)stream;
  return FA_OK;
}

static bool check_matrix_shape(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                               int layout) {
  if (!G || p < 1 || n < 1) return false;
  if (((uintptr_t)G & 15u) != 0) return false;
  if (layout == FA_ROW_MAJOR)   // ldg = row pitch; a tile row must fit the tile width
    return ldg >= p && ldg <= 16 * ((p + 15) / 16);
  if (ldg < n) return false;
  if ((ldg * elem_size(dtype)) % 16 != 0 && p > 1) return false;
  return true;
}

static bool check_matrix_args(const fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n) {
  if (!c) return false;
  if (p > c->cfg.p_max || n > c->cfg.n_max) return false;
  return check_matrix_shape(G, ldg, p, n, c->cfg.dtype, c->cfg.layout);
}

static bool check_solver_args(int p, int m, double lambda, int iters, double tol) {
  if (m < 1 || m > p) return false;
  if (!(lambda >= 0.0) || !isfinite(lambda)) return false;
  if (iters < 1 || iters > FA_ITERS_MAX) return false;
  if (!(tol >= 0.0)) return false;
  return true;
}

extern "C" fa_status fa_aggregate(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n, int m,
                                  double lambda, int iters, double tol, float* out) {
  if (!check_matrix_args(c, G, ldg, p, n) || !out || ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (!check_solver_args(p, m, lambda, iters, tol)) return FA_ERR_ARG;
  hipStream_t st = c->stream;
  const bool prof = c->profiling != 0;
  c->ev_recorded = 0;
  // S1: norms and Gram matrix, per-workgroup partials;  S2: their fixed-order sum
  int nparts = 0;
  if (fa_launch_gram(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cfg.gram, c->gram_max_blocks,
                     c->partials, c->Kd, c->flag_d, &nparts, st, prof ? &c->tm[0] : nullptr,
                     prof ? &c->tm[1] : nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  // S3-S5: p x p IRLS and coefficients
  if (fa_launch_irls(c->Kd, p, m, lambda, iters, tol, c->cfg.clamp_delta, c->cfg.rank_tol,
                     c->cfg.pair_tol, c->cfg.exponent_a, c->cd, c->info_d, c->gws, c->cfg.solver, c->cfg.wide_spin_budget, nullptr, st,
                     prof ? &c->tm[2] : nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  // S6: out = G c
  if (fa_launch_combine(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out, c->combine_max_blocks, st,
                        prof ? &c->tm[3] : nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  if (prof) c->ev_recorded = 1;
  c->last_nparts = nparts;
  c->has_solution = 1;
  c->last_p = p;
  c->last_m = m;
  return FA_OK;
}

// ---------------------------------------------------------------------------------------------
// fa_aggregate without a context and without any allocation: the workspace is this array in
// the device image (every GPU holds its own copy at its own address).  In host code the
// array's name is only a handle for hipGetSymbolAddress; the kernels get the looked-up
// address, as they get the context's buffers in fa_aggregate.
namespace {

constexpr int kStaticBlocks = 256;                       // partial Grams: one per compute unit
constexpr int kStaticTiles = (FA_STATIC_P_MAX / 16) * (FA_STATIC_P_MAX / 16 + 1) / 2;
constexpr size_t kOffPartials = 0;
constexpr size_t kOffK = kOffPartials + sizeof(double) * kStaticBlocks * kStaticTiles * 256;
constexpr size_t kOffC = kOffK + sizeof(double) * FA_P_MAX * FA_P_MAX;
constexpr size_t kOffGws = kOffC + sizeof(double) * (FA_P_MAX + 8);
constexpr size_t kOffInfo = kOffGws + sizeof(double) * FA_GWS_DOUBLES;
constexpr size_t kOffFlag = kOffInfo + ((sizeof(fa_info) + 63) / 64) * 64;
constexpr size_t kStaticUsed = kOffFlag + 64;
static_assert(kStaticUsed <= FA_STATIC_SCRATCH_BYTES, "the static workspace is too small");
static_assert(kOffK % 256 == 0 && kOffC % 8 == 0 && kOffGws % 8 == 0 && kOffInfo % 8 == 0,
              "alignment of the parts of the static workspace");

constexpr int kMaxDevices = 64;
struct StaticDev {
  unsigned char* base;   // device address of `scratch` on this GPU; null until looked up
  int blocks;            // Gram workgroups: min(compute units, kStaticBlocks)
};
StaticDev g_static_dev[kMaxDevices];
pthread_mutex_t g_static_mu = PTHREAD_MUTEX_INITIALIZER;

}  // namespace

static __device__ __align__(256) unsigned char scratch[FA_STATIC_SCRATCH_BYTES];

// the record of the previous call must not be mistaken for this one's
__global__ void fa_static_clear_kernel(fa_info* info) {
  if (threadIdx.x == 0) {
    info->status = 0; info->p = 0; info->m = 0; info->rank = 0; info->iters_done = 0;
    info->sweeps = 0;
  }
}

// Once per device, with that device current: the address of its copy of the array, its
// compute-unit count, the kernels' launch attributes.  None of these allocates.
static fa_status static_setup(int dev, StaticDev* out) {
  if (dev < 0 || dev >= kMaxDevices) return FA_ERR_DEVICE;
  fa_status st = FA_OK;
  pthread_mutex_lock(&g_static_mu);
  if (!g_static_dev[dev].base) {
    void* ptr = nullptr;
    int cus = 0;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        fa_kernels_prepare() != hipSuccess || fa_irls64_prepare() != hipSuccess ||
        fa_gram_lp_prepare() != hipSuccess) {
      st = FA_ERR_DEVICE;
    } else {
      g_static_dev[dev].blocks = cus > 0 && cus < kStaticBlocks ? cus : kStaticBlocks;
      g_static_dev[dev].base = static_cast<unsigned char*>(ptr);
    }
  }
  if (st == FA_OK) *out = g_static_dev[dev];
  pthread_mutex_unlock(&g_static_mu);
  return st;
}

extern "C" fa_status fa_aggregate_static(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                         int m, double lambda, int iters, double tol, float* out,
                                         void* stream) {
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_ARG;
  if (p > FA_STATIC_P_MAX) return FA_ERR_TOO_LARGE;
  if (!check_matrix_shape(G, ldg, p, n, dtype, FA_WORKER_MAJOR) || !out ||
      ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (!check_solver_args(p, m, lambda, iters, tol)) return FA_ERR_ARG;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FA_ERR_DEVICE;
  StaticDev sd;
  const fa_status sst = static_setup(dev, &sd);
  if (sst != FA_OK) return sst;
  hipStream_t st = (hipStream_t)stream;
  double* partials = reinterpret_cast<double*>(sd.base + kOffPartials);
  double* Kd = reinterpret_cast<double*>(sd.base + kOffK);
  double* cd = reinterpret_cast<double*>(sd.base + kOffC);
  double* gws = reinterpret_cast<double*>(sd.base + kOffGws);
  fa_info* info_d = reinterpret_cast<fa_info*>(sd.base + kOffInfo);
  fa_config cfg;
  fa_default_config(&cfg);
  hipLaunchKernelGGL(fa_static_clear_kernel, dim3(1), dim3(64), 0, st, info_d);
  if (hipGetLastError() != hipSuccess) return FA_ERR_DEVICE;
  int nparts = 0;
  int* flag_d = reinterpret_cast<int*>(sd.base + kOffFlag);
  if (fa_launch_gram(G, ldg, p, n, dtype, FA_WORKER_MAJOR, cfg.gram, sd.blocks, partials, Kd,
                     flag_d, &nparts, st, nullptr, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_irls(Kd, p, m, lambda, iters, tol, cfg.clamp_delta, cfg.rank_tol, cfg.pair_tol,
                     cfg.exponent_a, cd, info_d, gws, cfg.solver, cfg.wide_spin_budget, nullptr,
                     st, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_combine(G, ldg, p, n, dtype, FA_WORKER_MAJOR, cd, 1, out, 1 << 20, st,
                        nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  return FA_OK;
}

extern "C" fa_status fa_aggregate_restream(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n,
                                           int m, double lambda, int iters, float* out) {
  if (!check_matrix_args(c, G, ldg, p, n) || !out || ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (!check_solver_args(p, m, lambda, iters, 0.0)) return FA_ERR_ARG;
  if (c->cfg.layout != FA_WORKER_MAJOR) return FA_ERR_ARG;   // measurement schedule: one layout
  hipStream_t st = c->stream;
  const bool prof = c->profiling != 0;
  c->ev_recorded = 0;
  c->ev_recorded_r = 0;
  // start from uniform weights: the state cleared by a kernel (a fill kernel, not a memset
  // node, so that the sequence may be recorded into a graph)
  static_assert(sizeof(fa_resume) % sizeof(double) == 0, "fa_resume is cleared as doubles");
  if (fa_launch_zero(reinterpret_cast<double*>(c->rs_d), (int)(sizeof(fa_resume) / sizeof(double)),
                     st) != hipSuccess)
    return FA_ERR_DEVICE;
  const double* A_d = reinterpret_cast<const double*>(reinterpret_cast<const char*>(c->info_d) +
                                                      offsetof(fa_info, A));
  const double* u_d = reinterpret_cast<const double*>(reinterpret_cast<const char*>(c->rs_d) +
                                                      offsetof(fa_resume, u));
  int nparts = 0;
  for (int it = 0; it < iters; ++it) {
    const bool last = it == iters - 1;
    // pass 1 over G: Gram matrix of the columns scaled by u_i = sqrt(w_i)/|g_i| (plain at
    // first); the scales are applied to the p x p sums, G^T W G = diag(u) (G^T G) diag(u)
    // (fp64 accumulation whatever the context's mode: the streamed residuals 1 - v of pass 2
    // are differences of exact projections and need a basis that is orthonormal to 1e-13)
    if (fa_launch_gram_partials(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, FA_GRAM_FP64,
                                c->gram_max_blocks, c->partials, &nparts, st,
                                (prof && last) ? &c->tm_r[0] : nullptr) != hipSuccess)
      return FA_ERR_DEVICE;
    if (fa_launch_gram_reduce(c->partials, nparts, p, c->Kd, it == 0 ? nullptr : u_d, st,
                              nullptr) != hipSuccess)
      return FA_ERR_DEVICE;
    // one weighted PCA with the current weights
    if (fa_launch_irls(c->Kd, p, m, lambda, 1, 0.0, c->cfg.clamp_delta, c->cfg.rank_tol,
                       c->cfg.pair_tol, c->cfg.exponent_a, c->cd, c->info_d, c->gws, c->cfg.solver, c->cfg.wide_spin_budget, c->rs_d, st,
                       nullptr) != hipSuccess)
      return FA_ERR_DEVICE;
    // pass 2 over G: projections on the new basis, then the next weights from them
    if (fa_launch_proj_partials(G, ldg, p, m, n, c->cfg.dtype, c->gram_max_blocks, A_d,
                                c->partials, &nparts, st,
                                (prof && last) ? &c->tm_r[1] : nullptr) != hipSuccess)
      return FA_ERR_DEVICE;
    if (fa_launch_proj_reduce(c->partials, nparts, p, m, c->Pd, st, nullptr) != hipSuccess)
      return FA_ERR_DEVICE;
    if (fa_launch_restream_weights(c->info_d, c->Pd, p, m, lambda, c->cfg.clamp_delta,
                                   c->cfg.pair_tol, c->cfg.exponent_a, c->rs_d, st) != hipSuccess)
      return FA_ERR_DEVICE;
  }
  if (fa_launch_combine(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out, c->combine_max_blocks, st,
                        nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  if (prof) c->ev_recorded_r = 1;
  c->last_nparts = 0;
  c->has_solution = 1;
  c->last_p = p;
  c->last_m = m;
  return FA_OK;
}

extern "C" fa_status fa_get_restream_info(fa_ctx* c, float ms[2], double* v_streamed,
                                          double* objective_streamed) {
  if (!c) return FA_ERR_ARG;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
  if (ms) {
    if (!c->ev_recorded_r) return FA_ERR_ARG;
    for (int k = 0; k < 2; ++k)
      if (hipEventElapsedTime(&ms[k], c->tm_r[k].start, c->tm_r[k].stop) != hipSuccess)
        return FA_ERR_DEVICE;
  }
  const char* base = reinterpret_cast<const char*>(c->rs_d);
  if (v_streamed &&
      hipMemcpy(v_streamed, base + offsetof(fa_resume, v_streamed), sizeof(double) * FA_P_MAX,
                hipMemcpyDeviceToHost) != hipSuccess)
    return FA_ERR_DEVICE;
  if (objective_streamed &&
      hipMemcpy(objective_streamed, base + offsetof(fa_resume, obj_streamed),
                sizeof(double) * FA_ITERS_MAX, hipMemcpyDeviceToHost) != hipSuccess)
    return FA_ERR_DEVICE;
  return FA_OK;
}

extern "C" fa_status fa_get_info(fa_ctx* c, fa_info* host_out) {
  if (!c || !host_out) return FA_ERR_ARG;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
  if (hipMemcpy(host_out, c->info_d, sizeof(fa_info), hipMemcpyDeviceToHost) != hipSuccess)
    return FA_ERR_DEVICE;
  if (host_out->status == FA_OK && host_out->eigengap != host_out->eigengap) {
    // the purification path needs no eigenvalues; get the diagnostic gap now, off the hot path
    const int N = 16 * ((host_out->p + 15) / 16);
    if (fa_launch_gap(c->gws + FA_GWS_MLAST_OFF, N, c->info_d, c->stream) != hipSuccess)
      return FA_ERR_DEVICE;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
    if (hipMemcpy(&host_out->eigengap,
                  reinterpret_cast<const char*>(c->info_d) + offsetof(fa_info, eigengap),
                  sizeof(double), hipMemcpyDeviceToHost) != hipSuccess)
      return FA_ERR_DEVICE;
  }
  return FA_OK;
}

extern "C" fa_status fa_gram(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n,
                             double* K_host) {
  if (!check_matrix_args(c, G, ldg, p, n) || !K_host) return FA_ERR_ARG;
  int nparts = 0;
  if (fa_launch_gram(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cfg.gram, c->gram_max_blocks,
                     c->partials, c->Kd, c->flag_d, &nparts, c->stream, nullptr, nullptr) !=
      hipSuccess)
    return FA_ERR_DEVICE;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
  if (hipMemcpy(K_host, c->Kd, sizeof(double) * p * p, hipMemcpyDeviceToHost) != hipSuccess)
    return FA_ERR_DEVICE;
  return FA_OK;
}

extern "C" fa_status fa_gram_begin(fa_ctx* c, int p, int64_t n) {
  if (!c || p < 1 || p > c->cfg.p_max || n < 1 || n > c->cfg.n_max) return FA_ERR_ARG;
  if (c->cfg.layout != FA_WORKER_MAJOR) return FA_ERR_ARG;
  if (fa_launch_zero(c->Kd, FA_P_MAX * FA_P_MAX, c->stream) != hipSuccess) return FA_ERR_DEVICE;
  c->arr_p = p;
  c->arr_n = n;
  c->arrived = 0;
  for (int j = 0; j < FA_P_MAX; ++j) c->arr_rows[j] = 0;
  return FA_OK;
}

extern "C" fa_status fa_gram_update_rows(fa_ctx* c, const void* G, int64_t ldg, int i,
                                         int64_t row0, int64_t nrows) {
  if (!c || c->arr_p < 1 || i < 0 || i >= c->arr_p) return FA_ERR_ARG;
  const int64_t n = c->arr_n, row1 = row0 + nrows;
  const int es = elem_size(c->cfg.dtype);
  // the rows of a gradient are announced in order, each once; a piece starts on a 16-byte
  // boundary of the gradient
  if (nrows < 1 || row0 != c->arr_rows[i] || row1 > n || (row0 * es) % 16 != 0) return FA_ERR_ARG;
  if (!check_matrix_args(c, G, ldg, c->arr_p, n)) return FA_ERR_ARG;
  // the other gradients hold these rows entirely or not at all (same piece boundaries for all)
  uint64_t resident = 0;
  for (int j = 0; j < c->arr_p; ++j) {
    if (j == i) continue;
    if (c->arr_rows[j] >= row1) resident |= (uint64_t)1 << j;
    else if (c->arr_rows[j] > row0) return FA_ERR_ARG;
  }
  // partial rows go to the Gram pass's partial buffer (at least 256 doubles per compute unit)
  int max_parts = c->gram_max_blocks * 256 / FA_ROW_JB;
  if (max_parts > 1024) max_parts = 1024;
  const unsigned char* first = reinterpret_cast<const unsigned char*>(G) + row0 * es;
  if (fa_launch_gram_row(first, ldg, c->arr_p, nrows, c->cfg.dtype, i, resident, c->partials,
                         max_parts, c->Kd, c->stream) != hipSuccess)
    return FA_ERR_DEVICE;
  c->arr_rows[i] = row1;
  if (row1 == n) c->arrived |= (uint64_t)1 << i;
  return FA_OK;
}

extern "C" fa_status fa_gram_update(fa_ctx* c, const void* G, int64_t ldg, int i) {
  if (!c || c->arr_p < 1) return FA_ERR_ARG;
  return fa_gram_update_rows(c, G, ldg, i, 0, c->arr_n);     // the whole gradient at once
}

extern "C" fa_status fa_aggregate_arrived(fa_ctx* c, const void* G, int64_t ldg, int m,
                                          double lambda, int iters, double tol, float* out) {
  if (!c || c->arr_p < 1) return FA_ERR_ARG;
  const int p = c->arr_p;
  const int64_t n = c->arr_n;
  const uint64_t all = p == 64 ? ~(uint64_t)0 : (((uint64_t)1 << p) - 1);
  if (c->arrived != all) return FA_ERR_ARG;                   // a gradient is still missing
  if (!check_matrix_args(c, G, ldg, p, n) || !out || ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (!check_solver_args(p, m, lambda, iters, tol)) return FA_ERR_ARG;
  hipStream_t st = c->stream;
  c->ev_recorded = 0;
  if (fa_launch_irls(c->Kd, p, m, lambda, iters, tol, c->cfg.clamp_delta, c->cfg.rank_tol,
                     c->cfg.pair_tol, c->cfg.exponent_a, c->cd, c->info_d, c->gws, c->cfg.solver,
                     c->cfg.wide_spin_budget, nullptr, st, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_combine(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out,
                        c->combine_max_blocks, st, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  c->last_nparts = 0;
  c->has_solution = 1;
  c->last_p = p;
  c->last_m = m;
  c->arr_p = 0;                                                // the round is over
  return FA_OK;
}

extern "C" fa_status fa_gram_async(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n) {
  if (!check_matrix_args(c, G, ldg, p, n)) return FA_ERR_ARG;
  int nparts = 0;
  if (fa_launch_gram(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cfg.gram, c->gram_max_blocks,
                     c->partials, c->Kd, c->flag_d, &nparts, c->stream, nullptr, nullptr) !=
      hipSuccess)
    return FA_ERR_DEVICE;
  return FA_OK;
}

extern "C" fa_status fa_irls(fa_ctx* c, const double* K_host, int p, int m, double lambda,
                             int iters, double tol) {
  if (!c || !K_host || p < 1 || p > c->cfg.p_max) return FA_ERR_ARG;
  if (!check_solver_args(p, m, lambda, iters, tol)) return FA_ERR_ARG;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
  if (hipMemcpy(c->Kd, K_host, sizeof(double) * p * p, hipMemcpyHostToDevice) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_irls(c->Kd, p, m, lambda, iters, tol, c->cfg.clamp_delta, c->cfg.rank_tol,
                     c->cfg.pair_tol, c->cfg.exponent_a, c->cd, c->info_d, c->gws, c->cfg.solver, c->cfg.wide_spin_budget, nullptr, c->stream,
                     nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  c->has_solution = 1;
  c->last_p = p;
  c->last_m = m;
  return FA_OK;
}

extern "C" fa_status fa_combine(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n,
                                const double* c_host, float* out) {
  if (!check_matrix_args(c, G, ldg, p, n) || !c_host || !out || ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
  if (hipMemcpy(c->cd, c_host, sizeof(double) * p, hipMemcpyHostToDevice) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_combine(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out, c->combine_max_blocks,
                        c->stream, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  return FA_OK;
}

extern "C" fa_status fa_basis(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n, int m,
                              float* Y, int64_t ldy) {
  if (!check_matrix_args(c, G, ldg, p, n) || !Y || ((uintptr_t)Y & 15u) != 0) return FA_ERR_ARG;
  // Y has room for m columns: it must be the m the coefficients in the context were made for
  if (!c->has_solution || c->last_p != p || c->last_m != m) return FA_ERR_ARG;
  if (ldy < n || ((ldy * 4) % 16 != 0 && m > 1)) return FA_ERR_ARG;
  // column a of Y = G * A[:, a]; A is row-major p x m inside the device-side record
  const double* A = reinterpret_cast<const double*>(reinterpret_cast<const char*>(c->info_d) +
                                                    offsetof(fa_info, A));
  // G is read once per eight columns of Y, whatever its layout
  if (fa_launch_combine_multi(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, A, m, Y, ldy,
                              c->combine_max_blocks, c->stream) != hipSuccess)
    return FA_ERR_DEVICE;
  return FA_OK;
}

extern "C" fa_status fa_aggregate_grouped(fa_ctx* c, const void* G, int64_t ldg, int q, int64_t n,
                                          const int* sizes_host, int nworkers, int m,
                                          double lambda, int iters, double tol, float* out) {
  if (!check_matrix_args(c, G, ldg, q, n) || !out || ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (!check_solver_args(q, m, lambda, iters, tol)) return FA_ERR_ARG;
  if (!sizes_host || nworkers < 1 || nworkers > q) return FA_ERR_ARG;
  int tot = 0;
  for (int i = 0; i < nworkers; ++i) {
    if (sizes_host[i] < 1 || sizes_host[i] > q) return FA_ERR_ARG;
    tot += sizes_host[i];
  }
  if (tot != q) return FA_ERR_ARG;
  hipStream_t st = c->stream;
  c->ev_recorded = 0;
  if (hipMemcpyAsync(c->sizes_d, sizes_host, sizeof(int) * nworkers, hipMemcpyHostToDevice, st) !=
      hipSuccess)
    return FA_ERR_DEVICE;
  int nparts = 0;
  if (fa_launch_gram(G, ldg, q, n, c->cfg.dtype, c->cfg.layout, c->cfg.gram, c->gram_max_blocks,
                     c->partials, c->Kd, c->flag_d, &nparts, st, nullptr, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_irls_grouped(c->Kd, q, nworkers, c->sizes_d, m, lambda, iters, tol,
                             c->cfg.clamp_delta, c->cfg.rank_tol, c->cfg.pair_tol,
                             c->cfg.exponent_a, c->cd, c->info_d, c->gws, c->cfg.solver,
                             c->cfg.wide_spin_budget, st) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_combine(G, ldg, q, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out,
                        c->combine_max_blocks, st, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  // the host array may be reused as soon as this returns
  if (hipStreamSynchronize(st) != hipSuccess) return FA_ERR_DEVICE;
  c->last_nparts = nparts;
  c->has_solution = 1;
  c->last_p = q;
  c->last_m = m;
  return FA_OK;
}

extern "C" fa_status fa_multikrum(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n, int f,
                                  int q, float* out, double* scores_host, int* selected_host) {
  if (!check_matrix_args(c, G, ldg, p, n) || !out || ((uintptr_t)out & 15u) != 0)
    return FA_ERR_ARG;
  if (f < 0 || p - f - 2 < 1 || q < 1 || q > p) return FA_ERR_ARG;
  hipStream_t st = c->stream;
  c->ev_recorded = 0;
  c->has_solution = 0;                       // no basis belongs to this result
  int nparts = 0;
  if (fa_launch_gram(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cfg.gram, c->gram_max_blocks,
                     c->partials, c->Kd, c->flag_d, &nparts, st, nullptr, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  // scores in the solvers' workspace, the selection in the block-width buffer
  if (fa_launch_krum(c->Kd, p, f, q, c->cd, c->gws, c->sizes_d, st) != hipSuccess)
    return FA_ERR_DEVICE;
  if (fa_launch_combine(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out,
                        c->combine_max_blocks, st, nullptr) != hipSuccess)
    return FA_ERR_DEVICE;
  c->last_nparts = nparts;
  if (scores_host || selected_host) {
    if (scores_host && hipMemcpyAsync(scores_host, c->gws, sizeof(double) * p,
                                      hipMemcpyDeviceToHost, st) != hipSuccess)
      return FA_ERR_DEVICE;
    if (selected_host && hipMemcpyAsync(selected_host, c->sizes_d, sizeof(int) * p,
                                        hipMemcpyDeviceToHost, st) != hipSuccess)
      return FA_ERR_DEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return FA_ERR_DEVICE;
  }
  return FA_OK;
}

extern "C" fa_status fa_check_basis(fa_ctx* c, const void* G, int64_t ldg, int p, int64_t n,
                                    const float* Y, int64_t ldy, int m, double* YtY_host,
                                    double* YtG_host) {
  if (!check_matrix_args(c, G, ldg, p, n) || !Y || ((uintptr_t)Y & 15u) != 0) return FA_ERR_ARG;
  if (m < 1 || m > p || ldy < n || !YtY_host || !YtG_host) return FA_ERR_ARG;
  if (m > 1 && (ldy * 4) % 16 != 0) return FA_ERR_ARG;     // every column of Y 16-byte aligned
  const int TMr = (m + 15) / 16, TC = TMr + (p + 15) / 16;
  const int T = (c->cfg.p_max + 15) / 16;
  // the partial buffer holds gram_max_blocks * 2 T^2 tiles
  const int max_parts = (int)((int64_t)c->gram_max_blocks * 2 * T * T / (TMr * TC));
  const int ncols = 16 * TMr + p;
  static_assert(FA_GWS_DOUBLES >= FA_P_MAX * (FA_P_MAX + 16 * ((FA_P_MAX + 15) / 16)),
                "the solvers' workspace doubles as the result buffer of the check");
  if (fa_launch_cross(Y, ldy, m, G, ldg, p, n, c->cfg.dtype, c->cfg.layout, max_parts,
                      c->partials, c->gws, c->stream) != hipSuccess)
    return FA_ERR_DEVICE;
  double* W = c->check_h;      // m <= FA_P_MAX rows of ncols <= 2 FA_P_MAX
  if (hipMemcpyAsync(W, c->gws, (size_t)m * ncols * sizeof(double), hipMemcpyDeviceToHost,
                     c->stream) != hipSuccess)
    return FA_ERR_DEVICE;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return FA_ERR_DEVICE;
  for (int a = 0; a < m; ++a) {
    for (int b = 0; b < m; ++b) YtY_host[a * m + b] = W[(size_t)a * ncols + b];
    for (int i = 0; i < p; ++i) YtG_host[a * p + i] = W[(size_t)a * ncols + 16 * TMr + i];
  }
  return FA_OK;
}

extern "C" fa_status fa_enqueue_kernel(fa_ctx* c, int which, const void* G, int64_t ldg, int p,
                                       int64_t n, int m, double lambda, int iters, double tol,
                                       float* out) {
  if (!c || which < 0 || which > 3) return FA_ERR_ARG;
  if (p < 1 || p > c->cfg.p_max) return FA_ERR_ARG;
  hipError_t e = hipSuccess;
  if (which == 0) {
    if (!check_matrix_args(c, G, ldg, p, n)) return FA_ERR_ARG;
    e = fa_launch_gram_partials(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cfg.gram, c->gram_max_blocks, c->partials,
                                &c->last_nparts, c->stream, nullptr);
  } else if (which == 1) {
    if (c->last_nparts < 1) return FA_ERR_ARG;
    e = fa_launch_gram_reduce(c->partials, c->last_nparts, p, c->Kd, nullptr, c->stream, nullptr);
  } else if (which == 2) {
    if (!check_solver_args(p, m, lambda, iters, tol)) return FA_ERR_ARG;
    e = fa_launch_irls(c->Kd, p, m, lambda, iters, tol, c->cfg.clamp_delta, c->cfg.rank_tol,
                       c->cfg.pair_tol, c->cfg.exponent_a, c->cd, c->info_d, c->gws, c->cfg.solver, c->cfg.wide_spin_budget, nullptr, c->stream,
                       nullptr);
    c->has_solution = 1; c->last_p = p; c->last_m = m;
  } else {
    if (!check_matrix_args(c, G, ldg, p, n) || !out || ((uintptr_t)out & 15u) != 0)
      return FA_ERR_ARG;
    e = fa_launch_combine(G, ldg, p, n, c->cfg.dtype, c->cfg.layout, c->cd, 1, out, c->combine_max_blocks,
                          c->stream, nullptr);
  }
  return e == hipSuccess ? FA_OK : FA_ERR_DEVICE;
}

extern "C" fa_status fa_set_profiling(fa_ctx* c, int enabled) {
  if (!c) return FA_ERR_ARG;
  c->profiling = enabled ? 1 : 0;
  c->ev_recorded = 0;
  return FA_OK;
}

extern "C" fa_status fa_get_timings(fa_ctx* c, float ms[4]) {
  if (!c || !ms) return FA_ERR_ARG;
  if (!c->ev_recorded) return FA_ERR_ARG;
  if (hipEventSynchronize(c->tm[3].stop) != hipSuccess) return FA_ERR_DEVICE;
  for (int k = 0; k < 4; ++k)
    if (hipEventElapsedTime(&ms[k], c->tm[k].start, c->tm[k].stop) != hipSuccess)
      return FA_ERR_DEVICE;
  return FA_OK;
}
