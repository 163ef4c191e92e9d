/*
 * nadmm.h -- C ABI of the MI355X (gfx950) library for one ADMM worker's local
 * x-update of Newton-ADMM: inexact Newton-CG on L2-regularised multinomial
 * (softmax) logistic regression; at the end, the ADMM outer solver with the
 * workers simulated on the one device.
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
 *     is sample a_i; or sparse storage, see nadmm_sparse.  The matrix-core kernels read rows in
 *     16-byte pieces.  With lda a multiple of 4 and d_A 16-byte aligned the pieces are aligned ones and d_A must be
 *     readable for (n-1) lda + 4 ceil(p/4) elements: up to three elements past the last sample when p is not a
 *     multiple of 4 (an n x lda allocation always is; what those elements hold does not matter).  Which kernels run
 *     depends on shape, stride and alignment:
 *       p <= 960 and C-1 <= 16: the single-pass matrix-core kernel, 55-60 % of the HBM roofline with aligned rows;
 *       wider rows or up to 32 free classes: the two-sweep matrix-core kernels (about 30 %);
 *       any other row stride (lda >= p) and a d_A that is only 4-byte aligned take variants of the same kernels that
 *         read nothing past column p-1 of a row and are 15-35 % slower (measured: Hessian-vector product at
 *         60000 x 785, C = 10: 57 us against 42 us at 60000 x 784, a local solve 5.3 against 5.1 ms; at 50000 x 3073:
 *         301 against 245 us; at 250000 x 2001, C = 20: 1.02 against 0.89 ms);
 *       rows of fewer than 48 columns that are not 16-byte aligned (and any A that is not 4-byte aligned): the
 *         two-pass float32 vector kernels, correct for every shape; on narrow rows they are the faster choice
 *         (1375000 x 29: 152 us per Hessian-vector product against 260 us), on wide rows 10 to 20 times slower
 *         than the matrix-core kernels (2-4 % of the roofline).
 *     nadmm_query_kernel_path() tells which path a problem takes.  Labels: int32 in 0..C-1; class C-1 is the reference
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
                              beta or gamma outside (0,1), negative iteration limits, nnz<0 */
  NADMM_EWORKSPACE = -2,   /* workspace missing, misaligned or too small */
  NADMM_EUNSUPPORTED = -3, /* shape outside the compiled range (C-1 > 32, max_ls > 62, n > 2^36 (sparse: 2^31 - 1), p (C-1) > 2^28) */
  NADMM_EHIP = -4,         /* a HIP call or kernel launch failed */
  NADMM_ESCRATCH = -5      /* nadmm_hessvec_static: the problem needs more scratch than the built-in buffer holds */
} nadmm_status;

#define NADMM_MAX_FREE_CLASSES 32   /* largest supported C-1 */
#define NADMM_MAX_LS 62             /* largest supported max_ls */
#define NADMM_TRACE_LEN 64          /* Newton iterations recorded in nadmm_stats */

/*
 * A in sparse storage (the paper reports on sparse as well as dense data sets, Section 1; its largest one,
 * E18 of Table 1, has 279,998 features).  Two views of the same n x p matrix, both on the device and
 * owned by the caller: compressed by rows for A V and A X, compressed by columns for A^T D (each
 * output row of either product is then summed by one workgroup in a fixed order, without atomics).
 *   row view:    entries k in [row_ptr[i], row_ptr[i+1]) belong to row i, at column col_idx[k], value val[k]
 *   column view: entries k in [col_ptr[j], col_ptr[j+1]) belong to column j, at row row_idx[k], value val_t[k]
 * Pointer arrays start at 0, do not decrease and end at nnz.  Entries of a row (column) may come in
 * any order; an entry repeated at one position counts as the sum.  The arrays are not checked: an
 * index outside its range is clamped into it and a pointer beyond nnz is cut off there (no
 * out-of-bounds access results, the values computed are then meaningless); the two views are not
 * compared with each other.  All arrays 4-byte (pointers: 8-byte) aligned; n <= 2^31 - 1.
 */
typedef struct nadmm_sparse {
  int64_t        nnz;        /* stored entries, >= 0 */
  const int64_t* d_row_ptr;  /* n + 1 */
  const int32_t* d_col_idx;  /* nnz */
  const float*   d_val;      /* nnz */
  const int64_t* d_col_ptr;  /* p + 1 */
  const int32_t* d_row_idx;  /* nnz */
  const float*   d_val_t;    /* nnz */
} nadmm_sparse;

/* Borrowed views of one worker's data share and penalty parameters. */
typedef struct nadmm_problem {
  const float*   d_A;       /* n x p, row-major, device (ignored if `sparse` is given) */
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
  const nadmm_sparse* sparse; /* HOST pointer, read during the call only; NULL = A is the dense array d_A.
                                 If given, d_A and lda are ignored. */
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

/* 100 * major + minor; 102: sparse storage of A, residual balancing (struct layouts changed since 100);
 * 103: nadmm_hessvec_static; 104: nadmm_workspace_bytes / nadmm_admm_workspace_bytes take the parameters into account */
int         nadmm_version(void);
const char* nadmm_status_string(int code);

/* Text of the last HIP error seen by the calling thread's most recent failing call ("" if none). */
const char* nadmm_last_hip_error(void);

/*
 * Bytes of device workspace that every entry point below accepts for this
 * problem and these parameters (params may be NULL: defaults for the
 * stand-alone calls).  Host-only; returns 0 if the problem is invalid.
 * With params the size can include room for max_cg (<= 32) arrays of n (C-1) floats (dense A on the
 * single-pass matrix-core path, 3 max_cg (C-1) <= p): see nadmm_local_newton.  The size without
 * params is a prefix of it and is accepted by every entry point as well.
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
 * nadmm_hessvec for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and
 * same results as nadmm_hessvec, but the scratch memory (rows of D, per-workgroup partial sums, the
 * sparse path's logits, packed operand and windows) is a buffer built into
 * the library: NADMM_STATIC_SCRATCH_BYTES = 32 MiB of device memory that every GPU the library runs on
 * holds until the process ends.  The call allocates and frees nothing and does not synchronise.
 *   - A problem that needs more (nadmm_hessvec_static_bytes(prob) > nadmm_static_scratch_bytes(); e.g.
 *     500000 x 2000, C = 20 with dense A: 49 MB) is rejected with NADMM_ESCRATCH before anything is enqueued.
 *     The headline shape 60000 x 784, C = 10 needs 18 MB (the size covers every kernel path that
 *     nadmm_set_kernel_path could select for the shape), 50000 x 3072, C = 10 needs 8.5 MB,
 *     250000 x 2000, C = 20 needs 30.5 MB.
 *   - Every call on one GPU shares that GPU's buffer, whatever the stream or thread: calls that overlap
 *     in time on one GPU race.  Order them on one stream (or with events).  Nothing in the buffer has to
 *     survive between calls and nothing has to start at zero.
 *   - The device that is current at the call is the one whose buffer is used; d_* pointers must belong to it.
 */
#define NADMM_STATIC_SCRATCH_BYTES (32u << 20)
size_t nadmm_static_scratch_bytes(void);                          /* size of the built-in buffer (host-only) */
size_t nadmm_hessvec_static_bytes(const nadmm_problem* prob);     /* what this problem would need; 0 if invalid */
int nadmm_hessvec_static(const nadmm_problem* prob, const float* d_X, const float* d_V, float* d_HV, void* stream);

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
 * Passes over A per Newton iteration: one for the gradient, one per CG iteration, one for the logits A p of
 * the step that the line search (Algorithm 2) evaluates all its candidates from.  If ws_bytes is at least
 * nadmm_workspace_bytes(prob, params) for these params and that includes the arrays named there, the last
 * pass is left out: the CG iterate is p = sum_k alpha_k d_k, every CG pass has A d_k in hand and stores
 * it, and A p is put together from those.  A smaller (but sufficient) workspace takes the pass; the results
 * agree to rounding.
 * Accuracy near a minimiser: there the gradient is a small difference of large sums, and its absolute error is that of
 * the products with A.  Measured on 1237 x 45, C = 5 (sum scaling, ||g|| = 585 at the start): the matrix-core paths stall at
 * ||g|| of 2e-4 .. 4e-4 (about 1e-6 of the starting norm), the fp32 vector path (kernel path 1) reaches 2e-5.  A grad_tol
 * below that level is never met; the iteration then runs its max_newton iterations.
 */
int nadmm_local_newton(const nadmm_problem* prob, float* d_X, const nadmm_params* params,
                       nadmm_stats* h_stats, void* d_ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ADMM outer solver with N workers simulated on one GPU (Algorithm 1 with fixed or residual-balanced penalty parameters;
 * Section 2.3: x-, z-, y-updates, closed-form z-update for g(z) = lambda/2 ||z||^2; Section 2.3.1:
 * residuals and stopping).  The workers' local solves of one outer iteration are independent; they are spread over a few
 * library-owned streams (forked from and joined to the caller's stream with events, created on the first call of a host
 * thread and kept), every worker on its own part of the workspace, so that they overlap on the one device.
 *
 * Multipliers are kept in the sign convention of nadmm_problem.d_y: u_i = -y_i of the paper, so
 *   z   = sum_i (rho_i x_i + u_i) / (lambda + sum_i rho_i)
 *   u_i = u_i + rho_i (x_i - z)
 *   r_i = z - x_i,  d_i = -rho_i (z - z_prev)
 * Stopping compares the stacked norms ||r||, ||d|| with
 *   eps_pri  = sqrt(N) eps_abs + eps_rel max{ sqrt(sum_i ||x_i||^2), sqrt(N) ||z|| }
 *   eps_dual = sqrt(d) eps_abs + eps_rel sqrt(sum_i ||u_i||^2)
 * (the printed tolerances with every squared norm read as the norm).
 *
 * Adaptive penalty: Section 2.3 names residual balancing as the customary rule and uses a spectral rule
 * whose formulas are in a cited work only; penalty_rule = 1 is residual balancing in its published form
 * (Boyd et al. 2011, the paper's reference for it), applied to all workers by one common factor c on the
 * given rho_i: after an iteration with ||r|| > mu ||d||, c <- tau c; with ||d|| > mu ||r||, c <- c / tau.
 * The multipliers are kept unscaled, so a change of penalty leaves them as they are.
 * ------------------------------------------------------------------------------------------------ */
#define NADMM_MAX_WORKERS 64

typedef struct nadmm_admm_params {
  int32_t      max_outer;   /* ADMM iterations */
  float        eps_abs;     /* both tolerances 0: run max_outer iterations */
  float        eps_rel;
  nadmm_params local;       /* Algorithm 3, run on every worker in every iteration */
  int32_t      penalty_rule;/* 0: the penalties rho_i stay as given; 1: residual balancing (below) */
  float        rb_mu;       /* rule 1: imbalance that triggers a change, >= 1 (customary 10) */
  float        rb_tau;      /* rule 1: factor of a change, > 1 (customary 2) */
} nadmm_admm_params;

typedef struct nadmm_admm_stats {
  int32_t outer_iters;      /* iterations performed */
  int32_t converged;        /* 1 if the residual test stopped the iteration */
  double  r_norm, d_norm, eps_pri, eps_dual;     /* of the last iteration */
  double  r_trace[NADMM_TRACE_LEN];              /* per iteration (first NADMM_TRACE_LEN) */
  double  d_trace[NADMM_TRACE_LEN];
  double  rho_scale;                             /* common factor on the rho_i after the last iteration */
  double  rho_scale_trace[NADMM_TRACE_LEN];      /* factor in force during each iteration */
} nadmm_admm_stats;

/*
 * Workspace for nadmm_admm_solve / nadmm_admm_consensus: the local workspaces of the N
 * workers (sized for params->local as nadmm_workspace_bytes sizes them; params may be NULL) plus the
 * consensus state.  h_workers: host array of N problem descriptions (shards of the
 * rows of A; same p and C).  Returns 0 on invalid arguments.
 */
size_t nadmm_admm_workspace_bytes(const nadmm_problem* h_workers, int32_t N, const nadmm_admm_params* params);

/*
 * One consensus step (z-, y-update, residuals, tolerances) on device-resident iterates:
 * d_x N x d (row i = x_i), d_u N x d (multipliers, updated in place), d_z d (z_prev in, z out),
 * h_rho host array of N penalties.  d_out (device, 4 doubles): ||r||, ||d||, eps_pri, eps_dual.
 * d_ws: at least nadmm_admm_workspace_bytes() (or 64 KiB if only this call is used), 256-byte aligned.
 */
int nadmm_admm_consensus(int32_t N, int64_t d, const float* d_x, float* d_u, float* d_z, const float* h_rho,
                         float lambda, float eps_abs, float eps_rel, double* d_out,
                         void* d_ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 1.  h_workers[i]: shard i (d_A, n, p, lda, d_labels, C, loss_scale, rho = rho_i; its lambda,
 * d_z, d_y are ignored: the local subproblems have no regulariser and use d_z, d_u below).
 * d_x: N x d, x_i^0 on entry, x_i on return.  d_u: N x d (out; zero-initialised by the call), d_z: d (out;
 * zero-initialised).  Everything is ordered after the work already on `stream` and before work enqueued on it later.
 * With both tolerances 0 nothing synchronises.  With a residual test the call waits for the stream after every fourth
 * outer iteration and stops enqueueing once the test has fired (under stream capture it cannot wait: all max_outer
 * iterations are enqueued and those after the stop are no-ops).  h_stats (host) may be NULL; if not, the stream is
 * synchronised before return.
 */
int nadmm_admm_solve(const nadmm_problem* h_workers, int32_t N, float lambda, float* d_x, float* d_u, float* d_z,
                     const nadmm_admm_params* params, nadmm_admm_stats* h_stats,
                     void* d_ws, size_t ws_bytes, void* stream);

/*
 * Kernel selection, for tests and benchmarks; kept per host thread (it applies to the calls that the same
 * thread makes afterwards, workspace sizes included), so the library has no state shared between threads:
 *   0 = automatic (default), 1 = two-pass fp32 vector kernels (any shape),
 *   2 = fused single-pass matrix-core kernel (C-1 <= 16, p <= 960; any row stride, A 4-byte aligned;
 *       p >= 4 unless the rows are 16-byte aligned), 3 = thin-data single-pass kernel (p <= 32, p % 4 == 0,
 *       C-1 <= 3, lda == p), 4 = column-sliced two-sweep matrix-core kernels (the automatic
 *       choice where 2 and 3 do not apply: C-1 <= 32; any row stride, A 4-byte aligned; p >= 4 unless
 *       the rows are 16-byte aligned), 5 = sparse-storage kernels (the only path for a problem with `sparse` set,
 *       and only for those).  A forced path that does not support the problem makes the
 *       compute calls return NADMM_EUNSUPPORTED.
 * Returns the previous value, or NADMM_EINVAL.
 */
int nadmm_set_kernel_path(int path);

/* Which path (1 to 5) is taken for this problem under the current setting; host-only. */
int nadmm_query_kernel_path(const nadmm_problem* prob);

#ifdef __cplusplus
}
#endif
#endif /* NADMM_H */
