/*
 * fa.h -- C ABI of the Flag Aggregator hot path for AMD MI355X (gfx950).
 *
 * The library computes the parameter server's aggregation step of
 * "Flag Aggregator" (arXiv 2302.05865): given p worker gradients g_1..g_p in R^n
 * it finds an orthonormal Y (n x m) for the FA objective (Eq. 5 with the
 * data-dependent regulariser, Sec. 2.3 option (2)) by iteratively re-weighted
 * least squares (Alg. 1, step "IRLS"; Sec. 3 "Implementation Details") and
 * returns d = (1/p) Y Y^T G 1 (Alg. 1, "Obtain gradient direction").
 *
 * Everything n-sized runs in hand-written HIP kernels on the stream given at
 * creation.  All "device" pointers are plain HIP device addresses owned by the
 * caller; the library retains none of them after the call has completed on the
 * stream.  All "host" pointers are ordinary host memory.
 *
 * Storage of G ("worker-major"): gradient i is contiguous, element k of
 * gradient i is at  G + (i*ldg + k) * elem_size,  ldg >= n.  G must be 16-byte
 * aligned and ldg*elem_size a multiple of 16.  This is the paper's n x p
 * matrix G (columns = workers, Sec. 2.1) stored column by column, i.e. the
 * layout in which a parameter server receives p flat gradients (Alg. 1).
 *
 * Threading: a context is bound to one device and one stream and is not
 * thread-safe; distinct contexts are independent.
 */
#ifndef FA_H_
#define FA_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FA_P_MAX 64        /* largest number of workers p */
#define FA_ITERS_MAX 256   /* largest IRLS budget (length of the objective trace) */

typedef struct fa_ctx fa_ctx; /* opaque, library-owned */

typedef enum {
  FA_OK = 0,
  FA_ERR_ARG = 1,        /* bad argument; nothing was enqueued */
  FA_ERR_ALLOC = 2,      /* device/host allocation failed */
  FA_ERR_DEVICE = 3,     /* a HIP call failed */
  FA_ERR_NONFINITE = 4,  /* G holds NaN/Inf (detected on device from G^T G); out is NaN */
  FA_ERR_ZERO_INPUT = 5, /* every gradient is zero; out is zero */
  FA_ERR_TOO_LARGE = 6   /* fa_aggregate_static: p exceeds FA_STATIC_P_MAX, the size its fixed
                            device-resident workspace was built for; nothing was enqueued */
} fa_status;

typedef enum { FA_F32 = 0, FA_BF16 = 1 } fa_dtype; /* storage type of G */

/* Storage order of G.  FA_WORKER_MAJOR: gradient i contiguous (see above).  FA_ROW_MAJOR
 * ("interleaved", the n x p matrix of Sec. 2.1 stored row by row): element i of coordinate k
 * at G + (k*ldg + i) * elem_size with p <= ldg <= 16*ceil(p/16); G 16-byte aligned.  All
 * entry points accept it except fa_aggregate_restream. */
typedef enum { FA_WORKER_MAJOR = 0, FA_ROW_MAJOR = 1 } fa_layout;

/* Which kernel solves the p x p weighted-PCA problems of the IRLS (Alg. 1, step "IRLS").  All
 * compute the same iteration; they differ in how the m leading eigenvectors are found.
 * FA_SOLVER_AUTO: projector by matrix-core purification, no eigen-decomposition; a solve it
 *   cannot finish (eigenvalues m and m+1 tied) is redone by a Jacobi solver.
 * FA_SOLVER_JACOBI16: the p <= 16 Jacobi eigensolver (p > 16: as FA_SOLVER_AUTO).
 * FA_SOLVER_JACOBI: the any-p Jacobi eigensolver.
 * Every solver knows exponent_a. */
typedef enum { FA_SOLVER_AUTO = 0, FA_SOLVER_JACOBI16 = 1, FA_SOLVER_JACOBI = 2 } fa_solver;

/* How the Gram pass accumulates K = G^T G.
 * FA_GRAM_FP64: fp64 matrix-core accumulation of exact products (K good to ~1e-14 of
 *   sqrt(K_ii K_jj)).  HBM bound for fp32 storage at p <= 16; for bf16 storage and for p > 16
 *   the fp64 matrix core bounds the pass at under half of HBM speed.  Also what row-major
 *   storage and the re-streaming schedule always use.
 * FA_GRAM_BF16_MATRIX: bf16 storage, or fp32 storage at p > 16, worker-major: bf16 matrix
 *   core -- exact products of bf16 values (fp32 values are split exactly into three bf16
 *   pieces), 32 rows summed in fp32 by one matrix instruction, every such partial added in
 *   fp64.  K good to 2^-21 of sqrt(K_ii K_jj) at worst and to a few 1e-9 from a few thousand
 *   rows on (measured).  Its 32-row sums of products are fp32 and overflow for values beyond
 *   about 1e18; the fp64 pass therefore stands by behind it (always enqueued, returns at once
 *   unless K came out non-finite) and redoes K in that case, so finite input of any size is
 *   served, at the price of a second pass; products below about 1e-38 count as zero on this
 *   route.  Cases the kernel does not cover (fp32 storage at p <= 16, row-major) take the
 *   fp64 route.
 * FA_GRAM_AUTO: FA_GRAM_BF16_MATRIX from FA_GRAM_AUTO_MIN_ROWS rows on, where the pass is a
 *   visible share of the aggregation and the few 1e-9 stay well inside the parity gate;
 *   FA_GRAM_FP64 below, where the pass costs microseconds either way and a subspace with a
 *   small eigengap feels every digit of K. */
typedef enum { FA_GRAM_AUTO = 0, FA_GRAM_FP64 = 1, FA_GRAM_BF16_MATRIX = 2 } fa_gram_mode;
#define FA_GRAM_AUTO_MIN_ROWS (1 << 20)

typedef struct {
  int64_t n_max;      /* largest n this context will see (sizes the workspace) */
  int p_max;          /* largest p, 1..FA_P_MAX */
  int dtype;          /* fa_dtype */
  void* stream;       /* hipStream_t, borrowed; NULL = the default stream */
  double clamp_delta; /* weight floor: w = max(residual, delta)^(-1/2); default 1e-6 */
  double rank_tol;    /* eigenvalues of the normalised Gram below rank_tol*max are
                         treated as zero; default 1e-12 */
  double pair_tol;    /* a pair with D_ij^2 <= pair_tol*(|g_i|^2+|g_j|^2) counts as
                         D_ij = 0 and its term is dropped; default 1e-12 */
  double exponent_a;  /* the constant a >= 1 of the Taylor step in Sec. 2.2 ("Step 2"): every
                         term of the objective is (1 - v)^(1/a).  Default 2 = the Flag
                         Aggregator's square roots (Eq. 5).  Every p x p solver takes other
                         values (powers in place of the square roots; same passes over G). */
  int layout;         /* fa_layout of every G this context sees; default FA_WORKER_MAJOR */
  int solver;         /* fa_solver: which p x p solver runs the IRLS; default FA_SOLVER_AUTO */
  int wide_spin_budget; /* 16 < p <= 64 matrix-core solver: how many times a wavefront may poll
                         for a purification step's steering word before it gives up and the
                         Jacobi solver redoes the solve.  Default 1 << 22 (never reached in
                         practice); 0 = give up without polling, which makes every such solve
                         take the stand-by route (for testing it).  >= 0. */
  int gram;           /* fa_gram_mode; default FA_GRAM_AUTO */
} fa_config;

/* What the last fa_aggregate / fa_irls call on the context found (all fp64). */
typedef struct {
  int status;      /* fa_status of the device-side checks */
  int p, m;        /* as passed */
  int rank;        /* numerical rank of G */
  int iters_done;  /* IRLS solves performed (<= iters; fewer if tol stopped it) */
  int sweeps;      /* eigen-iteration count in total (diagnostic): purification steps on the
                      p <= 16 fast path, Jacobi sweeps otherwise */
  double eigengap; /* (mu_m - mu_{m+1}) / mu_1 of the last weighted PCA (inf if m >= rank) */
  double objective[FA_ITERS_MAX]; /* Eq. 5 value after each solve */
  double s[FA_P_MAX];  /* |g_i|^2 */
  double v[FA_P_MAX];  /* explained variance |Y^T g_i|^2/|g_i|^2 of each worker (Sec. 2.1) */
  double w[FA_P_MAX];  /* last IRLS weights of the data terms */
  double c[FA_P_MAX];  /* out = sum_i c[i] g_i */
  double A[FA_P_MAX * FA_P_MAX]; /* Y = G A; A[i*m + a], i < p, a < m (row-major p x m) */
  double K[FA_P_MAX * FA_P_MAX]; /* G^T G, row-major p x p */
} fa_info;

/* Fill *cfg with the defaults (n_max = 0, p_max = FA_P_MAX, FA_F32, NULL stream,
 * delta 1e-6, rank_tol 1e-12, pair_tol 1e-12, exponent_a 2, worker-major, FA_SOLVER_AUTO,
 * wide_spin_budget 1 << 22, FA_GRAM_AUTO). */
void fa_default_config(fa_config* cfg);

/* Allocate a context on the current HIP device: the per-block Gram partials
 * (sized from n_max, p_max) and the small p x p workspace.  Returns FA_ERR_ARG for
 * n_max < 1, p_max outside 1..FA_P_MAX, an unknown dtype, layout or solver, gram mode, a negative
 * wide_spin_budget, or tolerances / exponent out of range. */
fa_status fa_create(const fa_config* cfg, fa_ctx** out_ctx);

/* Free everything the context owns (synchronises its stream first).  NULL is ignored. */
void fa_destroy(fa_ctx* ctx);

/* Replace the stream later calls are enqueued on (hipStream_t, borrowed). */
fa_status fa_set_stream(fa_ctx* ctx, void* stream);

/*
 * The aggregation step (Eq. 5 solved by IRLS, then Alg. 1's direction):
 *   G      device, worker-major (see above), p gradients of n elements, read twice
 *   m      subspace dimension, 1 <= m <= p  (the paper uses ceil((p+1)/2))
 *   lambda weight of the pairwise regulariser, >= 0 (ordered pairs, factor lambda/(p-1))
 *   iters  number of weighted-PCA solves including the first, uniform one, 1..FA_ITERS_MAX
 *   tol    stop when successive objective values differ by less than tol; 0 = never
 *   out    device, n floats, caller-owned; receives d
 * Asynchronous on the context's stream; allocates nothing.  With profiling off the call is
 * kernel launches only (no copies, no memset nodes), so it may be recorded into a HIP graph
 * on a capturing stream; the same holds for fa_aggregate_restream and fa_aggregate_static
 * (whose first call on a device, the set-up, must come before the capture).  Argument errors
 * (including p > p_max, n > n_max, misaligned G/ldg, NULL pointers) return
 * FA_ERR_ARG synchronously.  Data errors are found on the device and reported by
 * fa_get_info: non-finite input fills out with NaN, all-zero input with zeros.
 */
fa_status fa_aggregate(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n, int m,
                       double lambda, int iters, double tol, float* out);

/*
 * The same aggregation under the re-streaming schedule, for measurement: every IRLS solve
 * passes over G twice, the way an implementation that re-does an n-sized decomposition per
 * iteration does (Sec. 3 "Implementation Details"; the cost discussed in Sec. 4).  Per solve:
 *   pass 1  weighted Gram matrix  G^T W G  with W = diag(w_i / |g_i|^2): G is streamed again
 *           and the weights are applied to the p x p sums, G^T W G = W^(1/2) (G^T G) W^(1/2)
 *           (applied to the columns inside the kernel they cost a fifth of the pass; plain
 *           G^T G for the first, uniform-weight solve),
 *   then one weighted PCA in p x p space (the pairwise terms of Eq. 5 are linear in G^T G),
 *   pass 2  projections Y^T g_i of all gradients on the new basis by streaming G (Y = G A is
 *           formed tile by tile in registers and never stored), from which the explained
 *           variances of Sec. 2.1, the residuals of Eq. 5 and the next weights are taken.
 * After `iters` solves the direction of Alg. 1 is written as in fa_aggregate.  The stop rule is
 * not available (tol = 0).  Results agree with fa_aggregate to rounding (about 1e-7: residuals
 * are formed as 1 - v from streamed projections); fa_get_info reports the p x p solver's own
 * record, fa_get_restream_info the streamed quantities.
 * HBM traffic: (2 iters + 1) n p elem_size + 4 n bytes, against 2 n p elem_size + 4 n of
 * fa_aggregate: this entry point exists to time the two per-iteration passes, not to be fast.
 */
fa_status fa_aggregate_restream(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n, int m,
                                double lambda, int iters, float* out);

/* After fa_aggregate_restream: waits for the stream; ms (may be NULL; needs
 * fa_set_profiling) receives the durations of the last solve's two passes in milliseconds
 * (ms[0] weighted Gram pass, ms[1] projection pass); v_streamed (NULL or FA_P_MAX doubles)
 * the explained variances measured by the last projection pass; objective_streamed (NULL or
 * FA_ITERS_MAX doubles) Eq. 5 after each solve, from streamed projections.  Host pointers. */
fa_status fa_get_restream_info(fa_ctx* ctx, float ms[2], double* v_streamed,
                               double* objective_streamed);

/* Wait for the context's stream and copy the record of the last solve to host memory. */
fa_status fa_get_info(fa_ctx* ctx, fa_info* host_out);

/*
 * Single steps of the path, exported so each kernel can be checked and timed alone.
 *
 * fa_gram: norms and pairwise inner products, K = G^T G (p x p, fp64; the quantities
 *   |g_i|^2 of Sec. 2.1 and D_ij^2 = K_ii + K_jj - 2 K_ij of Sec. 2.3).  Streams G
 *   once; synchronises and writes K row-major to host memory K_host (p*p doubles).
 * fa_gram_async: the same two kernels, enqueued only; K stays in the context's workspace
 *   (for timing the Gram pass alone, and as the first half of a caller-driven schedule).
 * fa_irls: the p x p part alone (normalisation, IRLS by repeated weighted PCA,
 *   coefficients) from a Gram matrix given in host memory; results via fa_get_info.
 * fa_combine: out = sum_i c[i] g_i with c (p doubles) given in host memory.  Streams G
 *   once.  Asynchronous.
 * fa_basis: Y = G A for the A of the last solve (Sec. 2.1's basis, materialised once):
 *   Y is device memory, m columns of n floats, column a at Y + a*ldy, ldy >= n.  m is the
 *   number of columns Y has room for and must equal the m of the last fa_aggregate /
 *   fa_aggregate_restream / fa_aggregate_grouped / fa_irls on the context, p its p
 *   (FA_ERR_ARG otherwise, nothing is written).  Asynchronous; the device-side status of that
 *   solve is not consulted: after a solve that fa_get_info reports as failed (non-finite or
 *   all-zero input) A is zero and so is Y.
 */
fa_status fa_gram(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n, double* K_host);
fa_status fa_gram_async(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n);
fa_status fa_irls(fa_ctx* ctx, const double* K_host, int p, int m, double lambda, int iters,
                  double tol);
fa_status fa_combine(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n,
                     const double* c_host, float* out);
fa_status fa_basis(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n, int m, float* Y,
                   int64_t ldy);

/*
 * The Gram pass spread over the arrival of the gradients (Alg. 1: in every round the parameter
 * server receives the gradients of the p workers; they come in one after another, and the
 * aggregation step need not wait for the last one to start on S1).
 *   fa_gram_begin   starts a round of p gradients of n elements: nothing has arrived, K = 0.
 *   fa_gram_update  gradient i is now in its place in G (worker-major storage as for
 *                   fa_aggregate: element k at G + (i*ldg + k) * elem_size).  One pass over
 *                   gradient i and the gradients that arrived before it extends K by row and
 *                   column i: K_ij = g_i . g_j, exact products added in fp64 (as accurate as the
 *                   fp64 Gram pass).  The places of gradients that have not arrived are not
 *                   read.  Asynchronous on the context's stream; a gradient may be announced
 *                   once per round, in any order.  Short for fa_gram_update_rows(i, 0, n).
 *   fa_gram_update_rows  the same for a gradient that lands piece by piece: elements
 *                   [row0, row0 + nrows) of gradient i are now in place.  One pass over those
 *                   rows of gradient i and of every gradient that already holds them adds their
 *                   share to row and column i of K (a pair's share of a piece is added when the
 *                   later of its two copies lands).  The pieces of one gradient are announced
 *                   in order (row0 = the end of the previous piece, 0 first); a piece starts
 *                   on a 16-byte boundary of the gradient (row0 * elem_size a multiple of 16);
 *                   all gradients are cut at the same places: FA_ERR_ARG if another gradient's
 *                   landed part ends inside the piece.  K is the fp64 Gram matrix to rounding
 *                   whatever the order of the pieces; its last bits depend on that order.
 *   fa_aggregate_arrived  once all p have arrived completely: the rest of fa_aggregate (S3-S6:
 *                   p x p IRLS on the K built so far, then out = G c), same arguments and
 *                   results; the Gram pass itself is not run again.  FA_ERR_ARG while anything
 *                   is missing.
 * When the last gradient lands whole, its own row of K is still to do: a pass that reads what
 * the one-shot Gram pass reads.  When it lands in pieces, only its last piece is: after the last
 * byte the server is a pass over (piece) x p elements away from the p x p solve, instead of a
 * pass over all of G.  In total the updates read p (p + 1) / 2 gradients instead of p: the price
 * of starting early, paid while the server would otherwise wait for the network.
 * Worker-major contexts only (a gradient arrives as one contiguous vector).
 */
fa_status fa_gram_begin(fa_ctx* ctx, int p, int64_t n);
fa_status fa_gram_update(fa_ctx* ctx, const void* G, int64_t ldg, int i);
fa_status fa_gram_update_rows(fa_ctx* ctx, const void* G, int64_t ldg, int i, int64_t row0,
                              int64_t nrows);
fa_status fa_aggregate_arrived(fa_ctx* ctx, const void* G, int64_t ldg, int m, double lambda,
                               int iters, double tol, float* out);

/*
 * Workers that send several gradients (Sec. 2.1; Sec. 2.2, the extension to g_i in
 * R^{n x k}; Appendix D): the q columns of G are
 * nworkers blocks of consecutive columns, block i of sizes_host[i] >= 1 columns (host memory,
 * they add up to q).  The value of worker i is tr(g_i^T Y Y^T g_i) / tr(g_i^T g_i); the IRLS
 * re-weights whole blocks; the pairwise term of Sec. 2.3 exists between blocks of equal width
 * (Frobenius distance), with the factor lambda / (nworkers - 1); the output counts every worker
 * once: out = (1/nworkers) Y Y^T sum_i mean_of_columns(g_i).  With every size 1 this is
 * fa_aggregate.  The other arguments, the layouts and the errors are fa_aggregate's (q takes
 * the place of p, also in m <= q and q <= p_max); fa_get_info then reports per column (v and w
 * of a column are its worker's).  Solvers: the matrix-core purification kernel with the any-p
 * kernel as stand-by (FA_SOLVER_AUTO), else the any-p kernel alone.  Synchronises the stream
 * before it returns, so sizes_host may be reused at once.
 */
fa_status fa_aggregate_grouped(fa_ctx* ctx, const void* G, int64_t ldg, int q, int64_t n,
                               const int* sizes_host, int nworkers, int m, double lambda,
                               int iters, double tol, float* out);

/*
 * Multi-Krum on the same two passes (the distance-based aggregator the paper compares with:
 * Sec. 3 "Baselines", Sec. 2.3 on aggregators built on pairwise distances; the rule is the
 * published one of Blanchard et al., 2017, which the paper cites).  The Gram pass gives
 * D_ij^2 = K_ii + K_jj - 2 K_ij; worker i is scored by the sum of its p - f - 2 smallest squared
 * distances to the other workers (f = Byzantine workers provided for, p - f - 2 >= 1); the q
 * workers with the smallest scores (ties: smaller index; 1 <= q <= p) are averaged by the
 * aggregate pass: out = (1/q) sum of the selected g_i.  scores_host (p doubles) and
 * selected_host (p ints, 0/1) are host memory and may be NULL; if either is given the call
 * synchronises the stream, otherwise it is asynchronous like fa_aggregate.  G, ldg, p, n, out
 * and the errors as for fa_aggregate.  No basis belongs to this result: fa_basis and
 * fa_get_info refer to the last fa_aggregate.
 */
fa_status fa_multikrum(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n, int f, int q,
                       float* out, double* scores_host, int* selected_host);

/*
 * Streamed check of a materialised basis (Sec. 2.1: Y has orthonormal columns, and the
 * explained variance of worker i is |Y^T g_i|^2 / |g_i|^2).  One pass over Y and G computes, in
 * fp64 on the device,
 *   YtY_host (m x m, row-major, host memory)  = Y^T Y   - the identity for a basis,
 *   YtG_host (m x p, row-major, host memory)  = Y^T G   - row a, column i: y_a . g_i.
 * Y is device memory as fa_basis writes it (m columns of n floats, column a at Y + a*ldy,
 * ldy >= n, every column 16-byte aligned: Y is, and for m > 1 so is ldy * 4); G, ldg, p, n as
 * for fa_aggregate, in the context's dtype and
 * layout.  Y need not come from fa_basis.  Synchronises the context's stream.  Uses the
 * context's workspace: the record of the last solve stays, its p x p scratch does not.
 * FA_ERR_ARG for bad shapes or pointers, FA_ERR_DEVICE if a launch or copy fails.
 */
fa_status fa_check_basis(fa_ctx* ctx, const void* G, int64_t ldg, int p, int64_t n,
                         const float* Y, int64_t ldy, int m, double* YtY_host, double* YtG_host);

/*
 * Per-kernel timing of fa_aggregate with HIP events on the context's stream.
 * fa_set_profiling(ctx, 1) makes every later fa_aggregate attach a begin and an end event
 * to each of its kernel dispatches (the events carry the kernel's own timestamps; nothing
 * extra is enqueued between the kernels); fa_get_timings synchronises and returns the last
 * call's kernel durations in milliseconds: ms[0] Gram pass, ms[1] partial reduction,
 * ms[2] p x p IRLS, ms[3] aggregate pass.  For 16 < p <= 64 the p x p part is two launches (the
 * matrix-core solver, then the Jacobi kernel that redoes a solve the first gave up and
 * otherwise returns at once); ms[2] runs from the begin of the first to the end of the second.
 * Where the Gram pass runs on the bf16 matrix core, ms[0] and ms[1] are that pass and its
 * reduction; the fp64 pass standing by behind them (three launches that return at once unless
 * the first overflowed) is not in any of the four figures.
 */
fa_status fa_set_profiling(fa_ctx* ctx, int enabled);
fa_status fa_get_timings(fa_ctx* ctx, float ms[4]);

/*
 * Enqueue ONE kernel of the path on the context's stream, with no synchronisation and no
 * host copies, so that a caller can time it alone (many launches between two events):
 *   which = 0  Gram pass (S1)            reads G, writes the context's partial Grams
 *   which = 1  partial reduction (S2)    partial Grams of the last Gram pass -> K
 *   which = 2  p x p IRLS (S3-S5)        K in the context -> coefficients c in the context
 *   which = 3  aggregate pass (S6)       reads G and the context's c, writes out
 * Arguments a kernel does not use are ignored (G may be NULL for 1 and 2, out for 0-2).
 * The kernels read what earlier calls on the same context left in its workspace.
 */
fa_status fa_enqueue_kernel(fa_ctx* ctx, int which, const void* G, int64_t ldg, int p, int64_t n,
                            int m, double lambda, int iters, double tol, float* out);

/*
 * fa_aggregate for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No context: the workspace (per-compute-unit partial
 * Gram matrices, K, the p x p solvers' scratch, the coefficients; FA_STATIC_SCRATCH_BYTES in
 * all) is a fixed array in the library's device image, one copy on every GPU the library runs
 * on, held until the process ends.  The call makes no hipMalloc / hipFree and uses no
 * allocating routine; the first call on a device looks the array's address up and sets kernel
 * launch attributes (neither allocates).
 *   G, ldg, p, n, m, lambda, iters, tol, out  as for fa_aggregate (worker-major storage only)
 *   dtype    fa_dtype of G
 *   stream   hipStream_t the work is enqueued on (NULL = the default stream), borrowed
 * Tolerances, exponent and solver are the defaults of fa_default_config.  Runs on the current
 * device; asynchronous.  Results are those of fa_aggregate, bit for bit, on a GPU of at most
 * 256 compute units.  Data errors show in out only (NaN for non-finite input, zeros for
 * all-zero input): there is no record to query.
 * Limits: p <= FA_STATIC_P_MAX, else FA_ERR_TOO_LARGE (n is not limited: nothing in the
 * workspace grows with n).  Other bad arguments: FA_ERR_ARG.  Nothing is enqueued on error.
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and must be serialised by the caller; calls on different GPUs
 * are independent.
 */
#define FA_STATIC_P_MAX 64
#define FA_STATIC_SCRATCH_BYTES (6u << 20)
fa_status fa_aggregate_static(const void* G, int64_t ldg, int p, int64_t n, int dtype, int m,
                              double lambda, int iters, double tol, float* out, void* stream);

const char* fa_status_string(fa_status s);
const char* fa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FA_H_ */
