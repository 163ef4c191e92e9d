/*
 * nadmm.h -- C ABI of the MI355X (gfx950) library for one ADMM worker's local
 * x-update of Newton-ADMM: inexact Newton-CG on L2-regularised multinomial
 * (softmax) logistic regression.
 *
 * Local objective (x-update of the ADMM iteration, Section 2.3; cross-entropy
 * with C-1 free weight vectors, Section 2.1):
 *
 *   Fhat(X) = s * sum_i l_i(X) + lambda/2 ||X||^2 + rho/2 ||X - z + y/rho||^2
 *   l_i(X)  = log(1 + sum_c exp<a_i,x_c>) - sum_c 1(b_i = c) <a_i,x_c>
 *
 * lambda = 0 gives the paper's x-update exactly (there the regulariser lives in
 * the z-update).  Sign of y: the paper writes ||z - x + y/rho||^2; pass -y to
 * obtain that convention.
 *
 * General rules for every entry point
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The
 *     caller owns all memory; the library never allocates or frees device
 *     memory.  Outputs must not alias inputs unless stated.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  Calls return after enqueueing; results land in
 *     device memory in stream order.  Only nadmm_local_newton with a non-NULL
 *     h_stats synchronises the stream.
 *   - Layout of A: row-major n x p float32, row stride lda >= p elements, row i
 *     is sample a_i.  Labels: int32 in 0..C-1; class C-1 is the reference
 *     class with logit 0 (the paper's class C).  Label values and finiteness
 *     of A are not checked (out-of-range labels are treated as the reference
 *     class; no out-of-bounds access results).
 *   - Layout of X, V, g, H*V, z, y, p: row-major p x (C-1) float32 with leading
 *     dimension C-1; column c is the paper's x_{c+1}.  The paper's stacked
 *     vector [x_1; ...; x_{C-1}] is the column-major flattening of the same
 *     matrix; every vector operation used is independent of that order.
 *   - d_ws is a scratch workspace of at least nadmm_workspace_bytes() bytes,
 *     256-byte aligned.  Calls sharing a workspace must be stream-ordered.
 *   - Return value: NADMM_OK (0) or a negative nadmm_status.  Arguments are
 *     validated on the host before anything is enqueued.
 */
#ifndef NADMM_H
#define NADMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nadmm_status {
  NADMM_OK = 0,
  NADMM_EINVAL = -1,       /* null required pointer, n<1, p<1, C<2, lda<p, rho<=0, lambda<0,
                              beta or gamma outside (0,1), negative iteration limits */
  NADMM_EWORKSPACE = -2,   /* workspace missing, misaligned or too small */
  NADMM_EUNSUPPORTED = -3, /* shape outside the compiled range (C-1 > 32, max_ls > 62, ...) */
  NADMM_EHIP = -4          /* a HIP call or kernel launch failed */
} nadmm_status;

#define NADMM_MAX_FREE_CLASSES 32   /* largest supported C-1 */
#define NADMM_MAX_LS 62             /* largest supported max_ls */
#define NADMM_TRACE_LEN 64          /* Newton iterations recorded in nadmm_stats */

/* Borrowed views of one worker's data share and penalty parameters. */
typedef struct nadmm_problem {
  const float*   d_A;       /* n x p, row-major, device */
  int64_t        n;         /* samples */
  int32_t        p;         /* features */
  int64_t        lda;       /* row stride of A in elements, >= p */
  const int32_t* d_labels;  /* n labels, device; may be NULL for nadmm_hessvec / nadmm_cg_solve */
  int32_t        C;         /* classes, >= 2; X has C-1 columns */
  float          loss_scale;/* s: 1 = plain sum over samples (Section 2.1), 1/n = mean */
  float          lambda;    /* >= 0 */
  float          rho;       /* > 0 */
  const float*   d_z;       /* p x (C-1), device; NULL = zeros */
  const float*   d_y;       /* p x (C-1), device; NULL = zeros */
} nadmm_problem;

/* Parameters of Algorithms 2 and 3 and of the CG iteration (Section 2.4). */
typedef struct nadmm_params {
  int32_t max_newton;      /* Newton iterations (Algorithm 3) */
  int32_t max_cg;          /* CG iterations per Newton iteration */
  int32_t max_ls;          /* i_max of Algorithm 2 */
  float   cg_tol;          /* theta of eq. (inexact); 0 = run max_cg iterations */
  float   grad_tol;        /* epsilon of Algorithm 3; 0 = run max_newton iterations */
  float   armijo_beta;     /* beta of eq. (armijo), in (0,1) */
  float   backtrack_gamma; /* gamma of Algorithm 2, in (0,1) */
} nadmm_params;

/* Filled by nadmm_local_newton (host memory). */
typedef struct nadmm_stats {
  int32_t newton_iters;    /* iterations that took a step */
  int32_t cg_iters_total;
  int32_t ls_evals_total;  /* objective evaluations counted as Algorithm 2 would make them */
  int32_t armijo_failed;   /* iterations whose line search ended by the i_max break */
  double  loss_initial;    /* Fhat at the starting point */
  double  loss_final;      /* Fhat at the returned X */
  double  grad_norm_final; /* norm of the last gradient that was formed */
  float   alpha[NADMM_TRACE_LEN];     /* step size per iteration (first NADMM_TRACE_LEN) */
  int32_t cg_iters[NADMM_TRACE_LEN];
  double  loss[NADMM_TRACE_LEN];      /* Fhat at the start of each iteration */
  double  grad_norm[NADMM_TRACE_LEN]; /* ||g|| at the start of each iteration */
} nadmm_stats;

int         nadmm_version(void);
const char* nadmm_status_string(int code);

/* Text of the last HIP error seen by the calling thread's most recent failing call ("" if none). */
const char* nadmm_last_hip_error(void);

/*
 * Bytes of device workspace that every entry point below accepts for this
 * problem and these parameters (params may be NULL: defaults for the
 * stand-alone calls).  Host-only; returns 0 if the problem is invalid.
 */
size_t nadmm_workspace_bytes(const nadmm_problem* prob, const nadmm_params* params);

/*
 * Objective and gradient at X (Sections 2.1 and 2.2; gradient of eq. Newton_G):
 *   *d_loss = Fhat(X)  (float64; per-row terms M_i + log(alpha_i) - Z_{i,b_i}
 *             evaluated in float32 with the log-sum-exp shift, summed in float64)
 *   d_grad  = s A^T (P - Y) + lambda X + rho (X - z) + y; NULL = objective only.
 */
int nadmm_loss_grad(const nadmm_problem* prob, const float* d_X, double* d_loss, float* d_grad,
                    void* d_ws, size_t ws_bytes, void* stream);

/*
 * Hessian-vector product without forming the Hessian (Section 2.6):
 *   W = A V, P = softmax probabilities of the free classes at X,
 *   D = P o W - P o rowsum(P o W),  d_HV = s A^T D + (lambda + rho) V.
 */
int nadmm_hessvec(const nadmm_problem* prob, const float* d_X, const float* d_V, float* d_HV,
                  void* d_ws, size_t ws_bytes, void* stream);

/*
 * Conjugate gradients on H(X) p = -g with early stopping (eq. inexact):
 * starts from p = 0, stops when ||H p + g|| <= tol ||g|| or after max_iter
 * iterations, returns the last iterate in d_p.  *d_iters (int32) and *d_relres
 * (float32, ||r||/||g|| by the recurrence) may be NULL.
 */
int nadmm_cg_solve(const nadmm_problem* prob, const float* d_X, const float* d_g, float* d_p,
                   int max_iter, float tol, int32_t* d_iters, float* d_relres,
                   void* d_ws, size_t ws_bytes, void* stream);

/*
 * Backtracking Armijo line search, Algorithm 2: the first alpha in
 * {1, gamma, gamma^2, ...} with Fhat(X + alpha p) <= Fhat(X) + alpha beta <p,g>;
 * at most max_ls + 1 reductions (the pseudo-code's i > i_max test), after which
 * alpha = gamma^(max_ls+1) is returned with *d_armijo_ok = 0.
 * loss_at_X: Fhat(X) if known, NaN to have it computed.
 * Outputs (device): *d_alpha float32, *d_loss_new float64 = Fhat(X + alpha p),
 * *d_armijo_ok int32.  X is not modified.
 */
int nadmm_line_search(const nadmm_problem* prob, const float* d_X, const float* d_p, const float* d_g,
                      double loss_at_X, float beta, float gamma, int max_ls,
                      float* d_alpha, double* d_loss_new, int32_t* d_armijo_ok,
                      void* d_ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 3: inexact Newton iteration on the local subproblem.  d_X holds the
 * warm start on entry (Algorithm 1 passes x_i^k) and x_i^{k+1} on return.
 * h_stats (host) may be NULL; if not, the stream is synchronised before return.
 */
int nadmm_local_newton(const nadmm_problem* prob, float* d_X, const nadmm_params* params,
                       nadmm_stats* h_stats, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Kernel selection, for tests and benchmarks (process-wide, not thread-safe):
 *   0 = automatic (default), 1 = two-pass fp32 vector kernels (any shape),
 *   2 = fused single-pass matrix-core kernel (row stride a multiple of 4, A 16-byte aligned,
 *       C-1 <= 16, p <= 960), 3 = thin-data single-pass kernel (p <= 32, p % 4 == 0,
 *       C-1 <= 3, lda == p), 4 = column-sliced two-sweep matrix-core kernels (the automatic
 *       choice where 2 and 3 do not apply: row stride a multiple of 4, A 16-byte aligned,
 *       C-1 <= 32).  A forced path that does not support the problem makes the
 *       compute calls return NADMM_EUNSUPPORTED.
 * Returns the previous value, or NADMM_EINVAL.
 */
int nadmm_set_kernel_path(int path);

/* Which path (1 to 4) is taken for this problem under the current setting; host-only. */
int nadmm_query_kernel_path(const nadmm_problem* prob);

#ifdef __cplusplus
}
#endif
#endif /* NADMM_H */
