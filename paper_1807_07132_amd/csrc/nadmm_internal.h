// Internal declarations shared by the translation units of libnadmm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "nadmm.h"

namespace nadmm {

// Raises a kernel's dynamic-LDS limit to the 160 KB of a gfx950 compute unit, once per device
// (the attribute belongs to the kernel's code object on the current device).
inline hipError_t ensure_lds_limit(const void* kernel, uint64_t* done_mask) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = (uint64_t)1 << (dev & 63);
  if ((*done_mask & bit) == 0) {
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    *done_mask |= bit;
  }
  return hipSuccess;
}

constexpr int kWave = 64;
constexpr int kMaxCand = NADMM_MAX_LS + 2;  // candidate step sizes 1, gamma, ..., gamma^(max_ls+1)
constexpr int kCandSlots = kMaxCand + 1;    // + one slot for alpha = 0 (objective at X itself)

// CG state after some number of updates, kept twice: a kernel that applies a pending update reads one copy and
// its workgroup 0 writes the other, so that no workgroup reads what another one of the same kernel writes.
struct CgSlot {
  double rr;        // ||r||^2 of the current residual
  int32_t active;   // 0 once CG has stopped (tolerance met, no positive curvature, or nothing to solve)
  int32_t iters;    // updates applied
  int32_t cur;      // which of the two sets of the vectors r, d, p is current
  int32_t pad_;
};

// Device-resident scalars of the Newton / CG / line-search drivers.  Lives at
// the start of the workspace; written only by single-workgroup tail kernels.
// Iterations of one CG solve whose directional logits A d_k the fused path may keep, so that the line search gets
// A p = sum_k alpha_k A d_k without another pass over A.
constexpr int kCgHist = 32;

struct DevState {
  double loss;      // Fhat at the current X
  double gg;        // ||g||^2 at the current X
  double rr;        // CG: ||r||^2 of the current residual
  double gg_cg;     // CG: ||g||^2 of the right-hand side
  double loss_new;  // line search: Fhat(X + alpha p)
  double loss_initial;
  float alpha;      // line search result
  int32_t newton_active;
  int32_t cg_active;
  int32_t cg_iters;
  int32_t armijo_ok;
  int32_t ls_evals;
  int32_t cg_go;    // two-kernel CG update: the first kernel's verdict (active and positive curvature)
  int32_t cg_ok;    //   0 if the first kernel met non-positive curvature
  float cg_alpha;   //   step length of this CG iteration
  int32_t pad_[3];
  double rr_prev;   //   ||r||^2 before this CG iteration
  CgSlot cgs[2];    // deferred CG update (fused single-pass path): see CgPend
  float cg_alphas[kCgHist];  // deferred CG update: step length of every iteration taken (p = sum_k alpha_k d_k)
  nadmm_stats stats;  // copied to the host at the end of nadmm_local_newton
};

// 16 bytes of a row of A that need only start on a 4-byte boundary: the load type of the matrix-core kernels' variants
// for rows that are not 16-byte aligned (any row stride, A 4-byte aligned).
struct __attribute__((packed, aligned(4))) Quad {
  float x, y, z, w;
};

// Row-pass (forward) work description, shared by the two-pass and the fused kernels.
//   kind 0  Hessian-vector rows:  D = P o W - P o rowsum(P o W)         (Section 2.6)
//   kind 1  gradient rows:        R = P - Y, row losses                  (Sections 2.1, 2.2)
//   kind 2  row losses only
//   kind 3  logits only:          Z0 = A B0 and / or Z1 = A B1
enum RowKind { kRowsHv = 0, kRowsGrad = 1, kRowsLoss = 2, kRowsLogits = 3 };

struct RowArgs {
  const float* A;
  int64_t n;
  int32_t p;
  int64_t lda;
  int32_t NC;          // C-1
  const float* B0;     // p x NC, operand of the logits Z = A B0 (X); NULL if P comes from Pin
  const float* B1;     // p x NC, operand of the directional logits W = A B1 (V or p); may be NULL
  const int32_t* labels;
  const float* Pin;    // n x NC cached probabilities (kind 0 with B0 == NULL)
  float* rows_out;     // n x NC: D (kind 0) or R (kind 1); may be NULL
  float* Pout;         // n x NC: probabilities, optional
  float* Z0out;        // n x NC: logits A B0, optional
  float* Z1out;        // n x NC: logits A B1, optional
  double* loss_part;   // per-workgroup partial sums of row losses (kinds 1, 2)
  int32_t kind;
  const int32_t* flag; // if non-NULL and *flag == 0 the kernel does nothing
};

// A CG update (Section 2.4) that has not been applied yet, handed to the kernel that needs its result: the
// next Hessian-vector sweep needs the new direction d, the sweep after the last CG iteration the iterate p.
// Every workgroup of that kernel applies the update for itself from q = H d and the partial sums of <d, q>
// (identical arithmetic in every workgroup, so all of them agree bit for bit, also on whether CG stops);
// workgroup 0 writes the new vectors to the other set and the new state to the other CgSlot.
struct CgPend {
  DevState* st;          // NULL: no deferred update (operands come from RowArgs as usual)
  int32_t slot_in;       // st->cgs[slot_in] is read, st->cgs[slot_in ^ 1] written
  int32_t final_p;       // 0: the kernel wants d (Hessian-vector product), 1: it wants p (end of CG)
  float* r[2];
  float* d[2];
  float* p[2];
  const float* q;        // H d of the update
  const double* dot_part;
  int32_t ndot;
  float tol;
  float* p_final;        // final_p: workgroup 0 leaves the iterate here and copies the state to the scalars of DevState
  int64_t dlen;
};

// Column-pass (transpose product) description: partial[k] = (rows of chunk k of A)^T rows_in
struct ColArgs {
  const float* A;
  int64_t n;
  int32_t p;
  int64_t lda;
  int32_t NC;
  const float* rows_in;  // n x NC
  float* partial;        // nparts x (p*NC)
  int32_t rows_per_chunk;
  const int32_t* flag;
};

struct Shape {
  int64_t n;
  int32_t p;
  int32_t NC;
  int64_t d;  // p * NC
};

// ---- launchers, generic two-pass path (nadmm_generic.hip) ----
int generic_row_blocks(int64_t n);
void generic_col_grid(const Shape& s, int* nslabs, int* nchunks, int* rows_per_chunk);
hipError_t launch_generic_rows(const RowArgs& a, hipStream_t st);
hipError_t launch_generic_cols(const ColArgs& a, int nslabs, int nchunks, hipStream_t st);
// rows stage on per-slice partial logits zw[slice][row][Z|W][C-1] (Z only if B0, W only if B1 is given);
// partial losses per block of generic_row_blocks()
hipError_t launch_logit_rows(const RowArgs& a, const float* zw, int nslices, hipStream_t st);

// ---- vector / tail kernels (nadmm_vec.hip) ----
struct NewtonHeadArgs {
  DevState* st;
  const double* loss_part;
  int32_t nblocks;
  float scale, lambda, rho;
  const float* X;
  const float* z;
  const float* y;
  const float* g;
  float* pdir;
  float* r;
  float* dvec;
  int64_t d;
  int32_t iter;        // Newton iteration index
  float grad_tol;
  int32_t newton_mode; // 1: part of Algorithm 3 (stats, grad_tol); 0: plain CG initialisation from g
  const double* pen_part;  // optional (with gg_part): partial sums left by the reduction that formed g, which
  const double* gg_part;   //   has then also written p = 0, r = d = -g
  int32_t npart;
  const float* rho_scale;  // optional device scalar factor on rho
};

struct ReduceArgs {
  const float* partial;
  int32_t nparts;
  int64_t d;
  float scale;            // s
  int32_t kind;           // 0: out = s*sum + (lambda+rho) V ; 1: out = s*sum + lambda X + rho (X - z) + y
  const float* V;         // kind 0
  const float* X;         // kind 1
  const float* z;
  const float* y;
  float lambda, rho;
  const float* rho_scale; // optional device scalar: the penalty is rho * *rho_scale (adaptive penalty of the outer solver)
  float* out;
  const float* V_alt;     // kind 0, optional with cur: V is V_alt if *cur != 0 (the two vector sets of a deferred CG update)
  const int32_t* cur;
  double* dot_part;       // kind 0, optional: per-workgroup sums of out[e] * V[e], reduce_out_blocks(d) entries
  double* pen_part;       // kind 1, optional: per-workgroup sums of the penalty terms lambda/2 x^2 + rho/2 (x - z + y/rho)^2
  double* gg_part;        // kind 1, optional: per-workgroup sums of out[e]^2
  float* cg_p;            // kind 1, optional: CG start from the gradient just formed, p = 0, r = d = -out
  float* cg_r;
  float* cg_d;
  const int32_t* flag;
  // kind 1, optional (d <= kReduceFinishMax): one more workgroup finishes the objective beside the reduction,
  // *lf_loss_out = s * sum(lf_loss_part[0 .. lf_nblocks)) + penalty terms of X (from X, z, y themselves)
  const double* lf_loss_part;
  int32_t lf_nblocks;
  double* lf_loss_out;
  // kind 0, optional (d <= kReduceFinishMax): that workgroup does the work of newton_head_kernel instead (the first
  // Hessian-vector product of a CG solve needs nothing of it: its direction is the -g that the gradient's reduction left)
  int32_t has_head;
  NewtonHeadArgs head;
};
constexpr int64_t kReduceFinishMax = 16384;
int reduce_out_blocks(int64_t d);
hipError_t launch_reduce_out(const ReduceArgs& a, hipStream_t st);

struct LossFinishArgs {
  const double* loss_part;
  int32_t nblocks;
  float scale, lambda, rho;
  const float* X;
  const float* z;
  const float* y;
  int64_t d;
  const double* pen_part;  // optional: penalty terms already summed per workgroup by the reduction (npart entries)
  int32_t npart;
  double* loss_out;  // device scalar
  const float* rho_scale;  // optional device scalar factor on rho
};
hipError_t launch_loss_finish(const LossFinishArgs& a, hipStream_t st);

hipError_t launch_newton_head(const NewtonHeadArgs& a, hipStream_t st);

struct CgUpdateArgs {
  DevState* st;
  float* pdir;
  float* r;
  float* dvec;
  const float* q;
  const double* dot_part;  // partial sums of <d, q> left by the reduction that formed q
  int32_t ndot;
  double* rr_part;         // cg_update_blocks(d) partial sums of the new ||r||^2 (two-kernel form, long vectors)
  int64_t d;
  float tol;
};
int cg_update_blocks(int64_t d);
// Small problems (d <= 1024 and at most 64 partial sums per thread): the reduction of the partial sums
// of A^T D, the linear term and the whole CG update in one single-workgroup kernel.
bool cg_fused_tail_supported(int64_t d, int nparts);
hipError_t launch_cg_reduce_update(const ReduceArgs& r, const CgUpdateArgs& a, hipStream_t st);
hipError_t launch_cg_update(const CgUpdateArgs& a, hipStream_t st);

struct CgFinishArgs {
  const DevState* st;
  const float* pdir;
  float* p_out;
  int64_t d;
  int32_t* iters_out;
  float* relres_out;
};
hipError_t launch_cg_finish(const CgFinishArgs& a, hipStream_t st);

struct LsEvalArgs {
  const float* Zx;
  const float* Zp;         // A p; or NULL: A p = sum_{k < st->cg_iters} st->cg_alphas[k] * hist[k * hist_stride + .]
  const float* hist;       // the directional logits A d_k that the CG sweeps left, n x NC each
  int64_t hist_stride;     // elements between two of them
  int32_t nbuf;            // buffers there are (<= kCgHist): the most iterations a solve takes
  int32_t has_pend;        // the last CG update is still pending (pend): workgroup 0 applies it, the others take its
                           // step length from the same scalars; launched with one workgroup more
  CgPend pend;
  const DevState* st;
  const int32_t* labels;
  int64_t n;
  int32_t NC;
  int32_t ncand;           // number of step sizes in alphas[] that are evaluated
  float alphas[kCandSlots];
  double* lpart;           // [candidate slot][workgroup], ls_eval_blocks(n) workgroups
  const int32_t* flag;
};
int ls_eval_blocks(int64_t n);
bool ls_eval_takes_pending(int64_t n);
hipError_t launch_ls_eval(const LsEvalArgs& a, hipStream_t st);

struct LsTailArgs {
  DevState* st;
  const double* lpart;
  int32_t nblocks;
  int32_t ncand;          // candidates of Algorithm 2 (max_ls + 2)
  int32_t zero_slot;      // index in alphas[] of alpha = 0, or -1 if loss_at_X is given
  float alphas[kCandSlots];
  double loss_at_X;       // used if zero_slot < 0 and !use_state_loss
  int32_t use_state_loss; // take Fhat(X) from st->loss
  float scale, lambda, rho, beta;
  const float* X;
  const float* z;
  const float* y;
  const float* pdir;
  const float* g;
  int64_t d;
  float* X_apply;         // if non-NULL: X_apply += alpha * pdir (Newton update)
  float* alpha_out;       // optional device outputs of the stand-alone call
  double* loss_new_out;
  int32_t* ok_out;
  int32_t iter;           // Newton iteration index or -1
  const int32_t* flag;
  const float* rho_scale; // optional device scalar factor on rho
  double* qpart;          // scratch of 2 reduce_out_blocks(d) doubles (long vectors: the sums over d are formed by
                          // several workgroups and pass through it); NULL = single-workgroup form at any length
};
hipError_t launch_ls_tail(const LsTailArgs& a, hipStream_t st);

// outer_flag, if non-NULL, is copied into newton_active: a stopped outer iteration turns the local solve into no-ops
hipError_t launch_state_init(DevState* st, const int32_t* outer_flag, hipStream_t stream);

// ---- ADMM outer solver (nadmm_admm.hip) ----
struct AdmmState {
  int32_t active;     // 0 once the residual test has stopped the iteration
  float rho_scale;    // common factor on every worker's penalty (residual balancing); written by the finishing
                      // kernel of a consensus step, read by the kernels launched after it
  nadmm_admm_stats stats;
};
struct AdmmConsensusArgs {
  AdmmState* st;           // may be NULL (stand-alone consensus step)
  const float* x;          // N x d
  float* u;                // N x d
  float* z;                // d
  int32_t N;
  int64_t d;
  float rho[NADMM_MAX_WORKERS];
  float lambda, eps_abs, eps_rel;
  int32_t penalty_rule;    // 0 fixed, 1 residual balancing
  float rb_mu, rb_tau;
  double* part;            // admm_blocks(d) x 5 partial sums
  double* out;             // optional: r_norm, d_norm, eps_pri, eps_dual
  int32_t iter;
};
int admm_blocks(int64_t d);
hipError_t launch_admm_init(AdmmState* st, float* u, float* z, int32_t N, int64_t d, hipStream_t stream);
hipError_t launch_admm_consensus(const AdmmConsensusArgs& a, hipStream_t stream);

// ---- fused single-pass path (nadmm_fused.hip) ----
bool fused_supported(const Shape& s, int64_t lda, const void* A);
int fused_num_partials(const Shape& s);
// Runs the rows pass and (if partial != NULL) the transpose product in one sweep
// over A; leaves per-workgroup partial sums of A^T rows in `partial`
// (nparts = fused_num_partials() blocks of d floats) and per-workgroup partial
// losses in a.loss_part[0 .. nparts).
hipError_t launch_fused(const RowArgs& a, float* partial, int nparts, hipStream_t st, const CgPend* cg = nullptr);
// the pending update alone (one workgroup): end of a stand-alone CG solve
hipError_t launch_cg_pending_finish(const CgPend& c, hipStream_t st);

// ---- thin-data single-pass path (nadmm_thin.hip): p <= 32, p % 4 == 0, C-1 <= 3, lda == p ----
bool thin_supported(const Shape& s, int64_t lda, const void* A);
int thin_num_partials(const Shape& s);
// cg, prev (both or neither): the sweep first applies the pending CG update, forming q = H d from the previous sweep's
// partial sums prev->partial (prev also carries scale, lambda, rho of the linear terms); see ThinArgs in nadmm_thin.hip
hipError_t launch_thin(const RowArgs& a, float* partial, int nparts, hipStream_t st, const CgPend* cg = nullptr,
                       const ReduceArgs* prev = nullptr);

// ---- column-sliced two-sweep matrix-core path (nadmm_sliced.hip): any p, C-1 <= 32, lda % 4 == 0 ----
bool sliced_supported(const Shape& s, int64_t lda, const void* A);
void sliced_grid(const Shape& s, int* nslices, int* steps_per_slice, int* row_groups);
// sweep 1 and the rows stage in one kernel (the logits never leave the compute unit); partial row losses: one per
// workgroup, sliced_loss_blocks() of them
int sliced_loss_blocks(const Shape& s);
hipError_t launch_sliced_logits(const RowArgs& a, hipStream_t st);
hipError_t launch_sliced_cols(const RowArgs& a, const float* rows_in, float* partial, hipStream_t st);

// ---- sparse storage of A (nadmm_sparse.hip) ----
// compressed rows of an nrows x ncols matrix; used for A (row view) and for A^T (column view of A)
struct SparseView {
  const int64_t* ptr;  // nrows + 1
  const int32_t* idx;  // nnz, in 0..ncols-1
  const float* val;    // nnz
  int64_t nrows;
  int32_t ncols;
  int64_t nnz;
};
// out = S B for a packed dense operand B: ncols rows of nops blocks of 4 sparse_group(NC) floats (zero
// padded); row r of the product goes to out[r * ldo + ooff + op * NC + c], op < nops, c < NC
struct SpmmArgs {
  SparseView S;
  const float* B;
  float* out;
  int32_t NC, nq, nops;  // nq = ceil(NC / 4) quads of a block hold data
  int32_t ldo, ooff;
  const int32_t* win;  // first row of each window of equal cost, nwin + 1 entries (launch_sparse_plan)
  int32_t nwin;
  const int32_t* flag;
};
int sparse_group(int NC);
int sparse_windows(int64_t nrows, int64_t nnz);
hipError_t launch_sparse_plan(const SparseView& S, int32_t* win, int nwin, hipStream_t st);
// dst[r] = [src0[r] | src1[r]] with every block padded to 4 sparse_group(NC) floats; one of src0, src1 may be NULL
hipError_t launch_sparse_pack(const float* src0, const float* src1, int64_t rows, int NC, float* dst,
                              const int32_t* flag, hipStream_t st);
hipError_t launch_spmm(const SpmmArgs& a, hipStream_t st);

}  // namespace nadmm
