// State that lets a caller drive the IRLS of the p x p solver one launch at a time (used by
// the re-streaming schedule, which passes over G again between the solves).  Plain C data in
// device memory; the same layout is read and written by all three solver paths.
#ifndef FA_RESUME_H_
#define FA_RESUME_H_

#include "fa.h"

typedef struct {
  int it0;          /* solves already done; 0 = start from uniform weights (PCA) */
  int scaled;       /* the Gram matrix handed to the solver is diag(u) K diag(u) */
  double prev_obj;  /* objective after solve it0 - 1 (for the stop rule) */
  double w[FA_P_MAX];               /* data-term weights for the next solve */
  double uinv[FA_P_MAX];            /* 1/u_i of the Gram matrix given (1 where u_i = 0) */
  double u[FA_P_MAX];               /* column scales for the next weighted Gram pass */
  double cp[FA_P_MAX * FA_P_MAX];   /* pair part of C for the next solve, row-major, ld = p:
                                       -2 lambda/(p-1) w_ij / D_ij^2, zero on the diagonal */
  double v_streamed[FA_P_MAX];          /* explained variances measured by streaming G */
  double obj_streamed[FA_ITERS_MAX];    /* Eq. 5 from the streamed projections, per solve */
} fa_resume;

#endif
