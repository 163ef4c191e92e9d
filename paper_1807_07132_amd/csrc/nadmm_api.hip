// C ABI of libnadmm: argument validation, workspace layout and the host-side
// drivers that enqueue the kernels of one local x-update (Algorithm 3 with the CG
// of Section 2.4 and the line search of Algorithm 2).  Nothing here synchronises
// the device except the final copy of the statistics.
#include <cmath>
#include <cstring>
#include <mutex>
#include <string>

#include "nadmm_internal.h"

// Built-in workspace of nadmm_hessvec_static: every device that loads the library holds its own copy until the
// process ends.  Host code never passes this name to a kernel; it asks the runtime for the copy's address on the
// current device (scratch_on_current_device) and uses that pointer.
static __device__ __align__(256) unsigned char scratch[NADMM_STATIC_SCRATCH_BYTES];

namespace nadmm {
namespace {

thread_local int g_path = 0;  // kernel path forced by the calling thread (0 = automatic)
thread_local std::string g_last_hip_error;

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout {
  Shape s;
  size_t state, g, pdir, r, dvec, q;
  size_t pdir2, r2, dvec2, pfinal;  // second vector set and final iterate of the deferred CG update (fused path)
  size_t drows, pcache, zx, zp;
  size_t partial, partial2, loss_part, lpart, dotpart, rrpart, headpart, zw;
  size_t pack, win_rows, win_cols;  // sparse storage: packed dense operand, windows of the two views
  size_t total;       // with the history of directional logits (hist_bufs of them), which comes last
  size_t total_base;  // without it
  size_t hist;
  int hist_bufs;
  int gen_row_blocks, gen_slabs, gen_chunks, gen_rpc;
  int fused_parts, thin_parts, sliced_parts, sliced_loss;
  bool fused_ok, thin_ok, sliced_ok;
  bool mc_auto;  // the matrix-core paths are also the automatic choice (see kAnyStrideMinP)
  bool sparse;
  int nwin_rows, nwin_cols;
  const float* rho_scale;  // device scalar factor on rho (outer solver with an adaptive penalty), or NULL
};

// Rows that are not 16-byte aligned take the matrix-core kernels' any-stride variants automatically only from this many
// columns on: with fewer, most waves of those kernels have no column step and the vector kernels are faster (measured
// per Hessian-vector product: 1375000 x 29: 260 against 152 us, 200000 x 13: 47 against 37 us, 100000 x 70: 29 against 75 us).
constexpr int kAnyStrideMinP = 48;

int validate_problem(const nadmm_problem* p, bool need_labels) {
  if (p == nullptr) return NADMM_EINVAL;
  if (p->n < 1 || p->p < 1 || p->C < 2) return NADMM_EINVAL;
  if (p->sparse != nullptr) {
    const nadmm_sparse* sp = p->sparse;
    if (sp->nnz < 0 || sp->d_row_ptr == nullptr || sp->d_col_ptr == nullptr) return NADMM_EINVAL;
    if (sp->nnz > 0 && (sp->d_col_idx == nullptr || sp->d_val == nullptr || sp->d_row_idx == nullptr ||
                        sp->d_val_t == nullptr))
      return NADMM_EINVAL;
    if (p->n > (int64_t)INT32_MAX) return NADMM_EUNSUPPORTED;  // row indices are 32-bit
  } else if (p->d_A == nullptr || p->lda < (int64_t)p->p) {
    return NADMM_EINVAL;
  }
  if (!(p->rho > 0.f) || !(p->lambda >= 0.f) || !std::isfinite(p->rho) || !std::isfinite(p->lambda)) return NADMM_EINVAL;
  if (!std::isfinite(p->loss_scale)) return NADMM_EINVAL;
  if (need_labels && p->d_labels == nullptr) return NADMM_EINVAL;
  if (p->C - 1 > NADMM_MAX_FREE_CLASSES) return NADMM_EUNSUPPORTED;
  if ((int64_t)p->p * (p->C - 1) > ((int64_t)1 << 28)) return NADMM_EUNSUPPORTED;
  if (p->n > ((int64_t)1 << 36)) return NADMM_EUNSUPPORTED;  // rows per workgroup are kept in 32 bits
  return NADMM_OK;
}

// hv_only: only the regions that a stand-alone Hessian-vector product touches (rows of D, partial sums, partial
// logits, the sparse path's packed operand and windows); the other offsets are then not to be used.
// wg_cap > 0: at most that many workgroups for the fused single-pass kernels (several workers' solves running side by
// side share the compute units; each then keeps the long row ranges per workgroup that amortise a launch).
// max_cg > 0: room for the directional logits A d_k of that many CG iterations, if the fused single-pass path is the
// one a solve would take and keeping them is cheaper than the pass over A they replace (see local_newton_enqueue).
void make_layout(const nadmm_problem* p, Layout* L, bool hv_only = false, int wg_cap = 0, int max_cg = 0) {
  Shape s;
  s.n = p->n;
  s.p = p->p;
  s.NC = p->C - 1;
  s.d = (int64_t)s.p * s.NC;
  L->s = s;
  L->rho_scale = nullptr;
  L->sparse = p->sparse != nullptr;
  L->gen_row_blocks = generic_row_blocks(s.n);
  generic_col_grid(s, &L->gen_slabs, &L->gen_chunks, &L->gen_rpc);
  if (L->sparse) L->gen_chunks = 1;  // the column view gives every element of A^T D whole
  L->mc_auto = L->sparse || (((p->lda & 3) == 0 && (reinterpret_cast<uintptr_t>(p->d_A) & 15) == 0) || s.p >= kAnyStrideMinP);
  L->fused_ok = !L->sparse && fused_supported(s, p->lda, p->d_A);
  L->fused_parts = L->fused_ok ? fused_num_partials(s) : 0;
  if (wg_cap > 0 && L->fused_parts > wg_cap) L->fused_parts = wg_cap;
  L->thin_ok = !L->sparse && thin_supported(s, p->lda, p->d_A);
  L->thin_parts = L->thin_ok ? thin_num_partials(s) : 0;
  const size_t vec = hv_only ? 0 : align256((size_t)s.d * sizeof(float));
  const size_t rows = align256((size_t)s.n * s.NC * sizeof(float));
  const size_t rows_solver = hv_only ? 0 : rows;
  size_t off = 0;
  L->state = off; off += hv_only ? 0 : align256(sizeof(DevState));
  L->g = off; off += vec;
  L->pdir = off; off += vec;
  L->r = off; off += vec;
  L->dvec = off; off += vec;
  L->q = off; off += vec;
  const bool two_sets = L->fused_ok || L->thin_ok;  // the paths with a deferred CG update
  L->pdir2 = off; off += two_sets ? vec : 0;
  L->r2 = off; off += two_sets ? vec : 0;
  L->dvec2 = off; off += two_sets ? vec : 0;
  L->pfinal = off; off += two_sets ? vec : 0;
  L->drows = off; off += rows;
  L->pcache = off; off += rows_solver;
  L->zx = off; off += rows_solver;
  L->zp = off; off += rows_solver;
  L->sliced_ok = !L->sparse && sliced_supported(s, p->lda, p->d_A);
  L->sliced_parts = 0;
  L->sliced_loss = 0;
  if (L->sliced_ok) {
    int sps = 0, S2 = 0;
    sliced_grid(s, &S2, &sps, &L->sliced_parts);  // partial sums per row group
    L->sliced_loss = sliced_loss_blocks(s);       // partial row losses per workgroup of sweep 1
  }
  int parts = L->gen_chunks > L->fused_parts ? L->gen_chunks : L->fused_parts;
  if (L->sliced_parts > parts) parts = L->sliced_parts;
  if (L->thin_parts > parts) parts = L->thin_parts;
  L->partial = off; off += align256((size_t)parts * s.d * sizeof(float));
  // thin-data path: the sweeps of a CG solve write their partial sums to two buffers in turn (each reads the previous one's)
  L->partial2 = off; off += (L->thin_ok && !hv_only) ? align256((size_t)L->thin_parts * s.d * sizeof(float)) : 0;
  int lblocks = L->gen_row_blocks > L->fused_parts ? L->gen_row_blocks : L->fused_parts;
  if (L->thin_parts > lblocks) lblocks = L->thin_parts;
  if (L->sliced_loss > lblocks) lblocks = L->sliced_loss;
  L->loss_part = off; off += hv_only ? 0 : align256((size_t)lblocks * sizeof(double));
  L->lpart = off; off += hv_only ? 0 : align256((size_t)ls_eval_blocks(s.n) * kCandSlots * sizeof(double));
  L->dotpart = off; off += hv_only ? 0 : align256((size_t)2 * reduce_out_blocks(s.d) * sizeof(double));  // two sums per workgroup
  L->rrpart = off; off += hv_only ? 0 : align256((size_t)cg_update_blocks(s.d) * sizeof(double));
  // partial sums of the penalty terms and of ||g||^2 that a Newton iteration's gradient leaves for its head (apart from dotpart:
  // the head may run beside the first reduction of the CG solve, which writes that)
  L->headpart = off; off += hv_only ? 0 : align256((size_t)2 * reduce_out_blocks(s.d) * sizeof(double));
  // the logits [Z | W] of the sparse path
  L->zw = off; off += align256(L->sparse ? (size_t)s.n * 2 * s.NC * sizeof(float) : 0);
  L->pack = off;
  L->win_rows = off;
  L->win_cols = off;
  L->nwin_rows = L->nwin_cols = 0;
  if (L->sparse) {
    const size_t npad = (size_t)4 * sparse_group(s.NC);
    const size_t a = (size_t)s.p * 2 * npad, b = (size_t)s.n * npad;  // [X | V] or D, rows padded
    off += align256((a > b ? a : b) * sizeof(float));
    L->nwin_rows = sparse_windows(s.n, p->sparse->nnz);
    L->nwin_cols = sparse_windows(s.p, p->sparse->nnz);
    L->win_rows = off; off += align256((size_t)(L->nwin_rows + 1) * sizeof(int32_t));
    L->win_cols = off; off += align256((size_t)(L->nwin_cols + 1) * sizeof(int32_t));
  }
  L->total_base = off;
  // 2 max_cg n (C-1) floats written and read instead of n p floats read: taken with a margin
  const bool fused_default = L->fused_ok && (g_path == 2 || (g_path == 0 && !L->thin_ok && L->mc_auto));
  L->hist_bufs = (!hv_only && fused_default && max_cg >= 1 && max_cg <= kCgHist && (int64_t)3 * max_cg * s.NC <= s.p) ? max_cg : 0;
  L->hist = off; off += (size_t)L->hist_bufs * rows;
  L->total = off;
}

int check_ws(const Layout& L, void* ws, size_t bytes) {
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || bytes < L.total) return NADMM_EWORKSPACE;
  return NADMM_OK;
}

template <typename T>
inline T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

int hip_fail(hipError_t e) {
  g_last_hip_error = hipGetErrorString(e);
  return NADMM_EHIP;
}

#define NADMM_HIP(expr)                          \
  do {                                           \
    hipError_t e_ = (expr);                      \
    if (e_ != hipSuccess) return hip_fail(e_);   \
  } while (0)

// Address of the built-in scratch array on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int scratch_on_current_device(void** out) {
  int dev = -1;
  NADMM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return NADMM_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    NADMM_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr || ((uintptr_t)ptr & 255) != 0) return NADMM_EWORKSPACE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return NADMM_OK;
}

// 1 = two-pass vector kernels, 2 = fused single pass (matrix cores), 3 = thin-data single pass,
// 4 = column-sliced two-sweep matrix-core path, 5 = sparse storage
int choose_path(const Layout& L, int* path) {
  if (L.sparse) {
    if (g_path != 0 && g_path != 5) return NADMM_EUNSUPPORTED;
    *path = 5;
    return NADMM_OK;
  }
  if (g_path == 5) return NADMM_EUNSUPPORTED;
  if (g_path == 1) { *path = 1; return NADMM_OK; }
  if (g_path == 2) {
    if (!L.fused_ok) return NADMM_EUNSUPPORTED;
    *path = 2;
    return NADMM_OK;
  }
  if (g_path == 3) {
    if (!L.thin_ok) return NADMM_EUNSUPPORTED;
    *path = 3;
    return NADMM_OK;
  }
  if (g_path == 4) {
    if (!L.sliced_ok) return NADMM_EUNSUPPORTED;
    *path = 4;
    return NADMM_OK;
  }
  *path = L.thin_ok ? 3 : (L.fused_ok && L.mc_auto ? 2 : (L.sliced_ok && L.mc_auto ? 4 : 1));
  return NADMM_OK;
}

int loss_blocks(const Layout& L, int path) {
  return path == 3 ? L.thin_parts : (path == 2 ? L.fused_parts : (path == 4 ? L.sliced_loss : L.gen_row_blocks));
}

SparseView row_view(const nadmm_problem* prob) {
  const nadmm_sparse* sp = prob->sparse;
  return SparseView{sp->d_row_ptr, sp->d_col_idx, sp->d_val, prob->n, prob->p, sp->nnz};
}
SparseView col_view(const nadmm_problem* prob) {
  const nadmm_sparse* sp = prob->sparse;
  return SparseView{sp->d_col_ptr, sp->d_row_idx, sp->d_val_t, (int64_t)prob->p, (int32_t)prob->n, sp->nnz};
}

// Sparse storage: the windows of equal cost of both views, once per entry-point call (they depend on the
// pointer arrays only, but the workspace is the caller's between calls).
int sparse_plan(const nadmm_problem* prob, const Layout& L, void* ws, hipStream_t st) {
  NADMM_HIP(launch_sparse_plan(row_view(prob), at<int32_t>(ws, L.win_rows), L.nwin_rows, st));
  NADMM_HIP(launch_sparse_plan(col_view(prob), at<int32_t>(ws, L.win_cols), L.nwin_cols, st));
  return NADMM_OK;
}

// One sweep over A: rows pass, and (if with_cols) partial sums of A^T rows_out.
// cg: the sweep applies a pending CG update first (fused and thin-data kernels); on the thin-data path prev names the
// previous sweep's partial sums, which that kernel adds up itself, and partial_out where this sweep's go.
int sweep(const nadmm_problem* prob, const Layout& L, int path, void* ws, RowArgs ra, bool with_cols,
          int* nparts, hipStream_t st, const CgPend* cg = nullptr, const ReduceArgs* prev = nullptr,
          float* partial_out = nullptr) {
  if (cg != nullptr && path != 2 && path != 3) return NADMM_EINVAL;
  if ((prev != nullptr || partial_out != nullptr) && path != 3) return NADMM_EINVAL;
  ra.A = prob->d_A;
  ra.n = prob->n;
  ra.p = prob->p;
  ra.lda = prob->lda;
  ra.NC = L.s.NC;
  if (path == 5) {
    SpmmArgs sa;
    sa.NC = L.s.NC;
    sa.nq = (L.s.NC + 3) / 4;
    sa.flag = ra.flag;
    sa.B = at<float>(ws, L.pack);
    if (ra.B0 != nullptr || ra.B1 != nullptr) {  // [Z | W] = A [X | V]
      const bool both = ra.B0 != nullptr && ra.B1 != nullptr;
      sa.S = row_view(prob);
      sa.out = at<float>(ws, L.zw);
      sa.win = at<int32_t>(ws, L.win_rows);
      sa.nwin = L.nwin_rows;
      sa.ldo = (both ? 2 : 1) * L.s.NC;
      if (both && sparse_group(L.s.NC) > 4) {
        // a row of X and a row of V do not share a 128-byte cache line: two products of one operand each
        // fetch a line per stored entry and are faster than one product that fetches two
        sa.nops = 1;
        NADMM_HIP(launch_sparse_pack(ra.B0, nullptr, prob->p, L.s.NC, at<float>(ws, L.pack), ra.flag, st));
        sa.ooff = 0;
        NADMM_HIP(launch_spmm(sa, st));
        NADMM_HIP(launch_sparse_pack(ra.B1, nullptr, prob->p, L.s.NC, at<float>(ws, L.pack), ra.flag, st));
        sa.ooff = L.s.NC;
        NADMM_HIP(launch_spmm(sa, st));
      } else {
        NADMM_HIP(launch_sparse_pack(ra.B0, ra.B1, prob->p, L.s.NC, at<float>(ws, L.pack), ra.flag, st));
        sa.nops = both ? 2 : 1;
        sa.ooff = 0;
        NADMM_HIP(launch_spmm(sa, st));
      }
    }
    NADMM_HIP(launch_logit_rows(ra, at<float>(ws, L.zw), 1, st));
    if (with_cols) {  // A^T D from the column view
      NADMM_HIP(launch_sparse_pack(ra.rows_out, nullptr, prob->n, L.s.NC, at<float>(ws, L.pack), ra.flag, st));
      sa.S = col_view(prob);
      sa.out = at<float>(ws, L.partial);
      sa.nops = 1;
      sa.ldo = L.s.NC;
      sa.ooff = 0;
      sa.win = at<int32_t>(ws, L.win_cols);
      sa.nwin = L.nwin_cols;
      NADMM_HIP(launch_spmm(sa, st));
      *nparts = 1;
    }
    return NADMM_OK;
  }
  if (path == 2) {
    NADMM_HIP(launch_fused(ra, with_cols ? at<float>(ws, L.partial) : nullptr, L.fused_parts, st, cg));
    *nparts = L.fused_parts;
    return NADMM_OK;
  }
  if (path == 3) {
    float* pout = partial_out != nullptr ? partial_out : at<float>(ws, L.partial);
    NADMM_HIP(launch_thin(ra, with_cols ? pout : nullptr, L.thin_parts, st, cg, prev));
    *nparts = L.thin_parts;
    return NADMM_OK;
  }
  if (path == 4) {
    NADMM_HIP(launch_sliced_logits(ra, st));
    if (with_cols) {
      NADMM_HIP(launch_sliced_cols(ra, ra.rows_out, at<float>(ws, L.partial), st));
      *nparts = L.sliced_parts;
    }
    return NADMM_OK;
  }
  NADMM_HIP(launch_generic_rows(ra, st));
  if (with_cols) {
    ColArgs ca;
    ca.A = prob->d_A;
    ca.n = prob->n;
    ca.p = prob->p;
    ca.lda = prob->lda;
    ca.NC = L.s.NC;
    ca.rows_in = ra.rows_out;
    ca.partial = at<float>(ws, L.partial);
    ca.rows_per_chunk = L.gen_rpc;
    ca.flag = ra.flag;
    NADMM_HIP(launch_generic_cols(ca, L.gen_slabs, L.gen_chunks, st));
    *nparts = L.gen_chunks;
  }
  return NADMM_OK;
}

RowArgs blank_rows() {
  RowArgs ra;
  std::memset(&ra, 0, sizeof(ra));
  return ra;
}

ReduceArgs reduce_args(const nadmm_problem* prob, const Layout& L, void* ws, int nparts, int kind, const float* XorV,
                       float* out, double* dot_part, const int32_t* flag) {
  ReduceArgs r;
  std::memset(&r, 0, sizeof(r));
  r.partial = at<float>(ws, L.partial);
  r.nparts = nparts;
  r.d = L.s.d;
  r.scale = prob->loss_scale;
  r.kind = kind;
  r.V = XorV;
  r.X = XorV;
  r.z = prob->d_z;
  r.y = prob->d_y;
  r.lambda = prob->lambda;
  r.rho = prob->rho;
  r.rho_scale = L.rho_scale;
  r.out = out;
  r.dot_part = dot_part;
  r.flag = flag;
  return r;
}

int reduce(const nadmm_problem* prob, const Layout& L, void* ws, int nparts, int kind, const float* XorV,
           float* out, double* dot_part, const int32_t* flag, hipStream_t st) {
  NADMM_HIP(launch_reduce_out(reduce_args(prob, L, ws, nparts, kind, XorV, out, dot_part, flag), st));
  return NADMM_OK;
}

// q = H(X) v.  With X == NULL the probabilities cached in the workspace are used.  With out == NULL only
// the partial sums of A^T D are formed (*nparts_out of them) and the caller finishes q.
int hv_apply(const nadmm_problem* prob, const Layout& L, int path, void* ws, const float* X, bool write_pcache,
             const float* v, float* out, double* dot_part, const int32_t* flag, int* nparts_out, hipStream_t st,
             const CgPend* cg = nullptr, const int32_t* red_flag = nullptr, const int32_t* cur = nullptr,
             const float* v_alt = nullptr, float* w_rows = nullptr, const NewtonHeadArgs* head = nullptr) {
  RowArgs ra = blank_rows();
  ra.kind = kRowsHv;
  ra.Z1out = w_rows;  // fused single-pass path only: the directional logits A v, n x (C-1)
  ra.B0 = X;
  ra.B1 = v;
  ra.Pin = X ? nullptr : at<float>(ws, L.pcache);
  ra.Pout = (X && write_pcache) ? at<float>(ws, L.pcache) : nullptr;
  ra.rows_out = at<float>(ws, L.drows);
  ra.flag = flag;
  int nparts = 0;
  int rc = sweep(prob, L, path, ws, ra, true, &nparts, st, cg);
  if (rc != NADMM_OK) return rc;
  if (nparts_out) *nparts_out = nparts;
  if (out == nullptr) return NADMM_OK;
  // deferred CG update: the reduction reads the activity flag and the current vector set that the sweep's
  // workgroup 0 has just written
  ReduceArgs r = reduce_args(prob, L, ws, nparts, 0, v, out, dot_part, red_flag != nullptr ? red_flag : flag);
  r.cur = cur;
  r.V_alt = v_alt;
  if (head != nullptr) {
    r.has_head = 1;
    r.head = *head;
  }
  NADMM_HIP(launch_reduce_out(r, st));
  return NADMM_OK;
}

// The deferred form of the CG update (fused single-pass path): see CgPend.
bool cg_deferred(int path) { return path == 2; }

CgPend cg_pend(const Layout& L, void* ws, DevState* ds, int slot_in, bool final_p, float tol) {
  CgPend c;
  std::memset(&c, 0, sizeof(c));
  c.st = ds;
  c.slot_in = slot_in;
  c.final_p = final_p ? 1 : 0;
  c.r[0] = at<float>(ws, L.r); c.r[1] = at<float>(ws, L.r2);
  c.d[0] = at<float>(ws, L.dvec); c.d[1] = at<float>(ws, L.dvec2);
  c.p[0] = at<float>(ws, L.pdir); c.p[1] = at<float>(ws, L.pdir2);
  c.q = at<float>(ws, L.q);
  c.dot_part = at<double>(ws, L.dotpart);
  c.ndot = reduce_out_blocks(L.s.d);
  c.tol = tol;
  c.p_final = at<float>(ws, L.pfinal);
  c.dlen = L.s.d;
  return c;
}

// Thin-data path inside a Newton iteration: the CG update is deferred as on the fused path, and the reduction of the partial
// sums with it: sweep k writes partial buffer k & 1 and first applies update k - 1 from buffer (k - 1) & 1.
bool thin_deferred(int path) { return path == 3; }
float* thin_partial(const Layout& L, void* ws, int k) { return at<float>(ws, (k & 1) ? L.partial2 : L.partial); }
ReduceArgs thin_prev(const nadmm_problem* prob, const Layout& L, void* ws, int k_prev) {
  ReduceArgs r = reduce_args(prob, L, ws, L.thin_parts, 0, nullptr, nullptr, nullptr, nullptr);
  r.partial = thin_partial(L, ws, k_prev);
  return r;
}

// CG iteration k after the initialisation: q = H d, then the update of p, r, d (Section 2.4).  On the fused path
// the update is deferred: iteration k's sweep first applies the update of iteration k - 1 (every workgroup for
// itself), and the update of the last iteration is applied by whatever consumes the iterate (cg_pend(final_p)).
// w_rows (deferred form only): where the sweep leaves A d_k, or NULL.
// head (deferred form, k == 0): the work of newton_head_kernel is done by a workgroup of this iteration's reduction; the sweep
// and the reduction then go by the Newton iteration's flag as the previous head left it (the first direction is the -g that
// the gradient's reduction wrote; if this head finds the iteration finished, one sweep was made for nothing).
int cg_iteration(const nadmm_problem* prob, const Layout& L, int path, void* ws, DevState* ds, const float* X,
                 bool write_pcache, float tol, int k, hipStream_t st, float* w_rows = nullptr,
                 const NewtonHeadArgs* head = nullptr, bool thin_def = false) {
  float* dvec = at<float>(ws, L.dvec);
  float* q = at<float>(ws, L.q);
  if (thin_def) {  // cached probabilities, no reduction kernel: see thin_deferred
    if (!thin_deferred(path) || X != nullptr) return NADMM_EINVAL;
    RowArgs ra = blank_rows();
    ra.kind = kRowsHv;
    ra.B1 = dvec;  // k == 0: the first direction; later the kernel takes the direction from the update it applies
    ra.Pin = at<float>(ws, L.pcache);
    ra.rows_out = at<float>(ws, L.drows);
    int nparts = 0;
    if (k == 0) {
      ra.flag = &ds->cgs[0].active;
      return sweep(prob, L, path, ws, ra, true, &nparts, st, nullptr, nullptr, thin_partial(L, ws, 0));
    }
    const CgPend c = cg_pend(L, ws, ds, (k - 1) & 1, false, tol);
    const ReduceArgs prev = thin_prev(prob, L, ws, k - 1);
    return sweep(prob, L, path, ws, ra, true, &nparts, st, &c, &prev, thin_partial(L, ws, k));
  }
  if (cg_deferred(path)) {
    double* dot = at<double>(ws, L.dotpart);
    if (k == 0)  // nothing pending: d is the first direction, state slot 0 as the initialisation left it
      return hv_apply(prob, L, path, ws, X, write_pcache, dvec, q, dot, head != nullptr ? &ds->newton_active : &ds->cgs[0].active,
                      nullptr, st, nullptr, nullptr, nullptr, nullptr, w_rows, head);
    const CgPend c = cg_pend(L, ws, ds, (k - 1) & 1, false, tol);
    return hv_apply(prob, L, path, ws, nullptr, false, dvec, q, dot, nullptr, nullptr, st, &c, &ds->cgs[k & 1].active,
                    &ds->cgs[k & 1].cur, at<float>(ws, L.dvec2), w_rows);
  }
  CgUpdateArgs cu;
  cu.st = ds;
  cu.pdir = at<float>(ws, L.pdir);
  cu.r = at<float>(ws, L.r);
  cu.dvec = dvec;
  cu.q = q;
  cu.dot_part = at<double>(ws, L.dotpart);
  cu.ndot = reduce_out_blocks(L.s.d);
  cu.rr_part = at<double>(ws, L.rrpart);
  cu.d = L.s.d;
  cu.tol = tol;
  const int parts = path == 3 ? L.thin_parts : (path == 2 ? L.fused_parts : (path == 4 ? L.sliced_parts : L.gen_chunks));
  if (cg_fused_tail_supported(L.s.d, parts)) {
    int nparts = 0;
    int rc = hv_apply(prob, L, path, ws, X, write_pcache, dvec, nullptr, nullptr, &ds->cg_active, &nparts, st);
    if (rc != NADMM_OK) return rc;
    NADMM_HIP(launch_cg_reduce_update(reduce_args(prob, L, ws, nparts, 0, dvec, q, nullptr, &ds->cg_active), cu, st));
    return NADMM_OK;
  }
  int rc = hv_apply(prob, L, path, ws, X, write_pcache, dvec, q, at<double>(ws, L.dotpart), &ds->cg_active, nullptr, st);
  if (rc != NADMM_OK) return rc;
  NADMM_HIP(launch_cg_update(cu, st));
  return NADMM_OK;
}

void fill_alphas(float* alphas, int ncand, float gamma) {
  double a = 1.0;
  for (int k = 0; k < ncand; ++k) {
    alphas[k] = (float)a;
    a *= (double)gamma;
  }
}

int validate_ls(float beta, float gamma, int max_ls) {
  if (!(beta > 0.f && beta < 1.f) || !(gamma > 0.f && gamma < 1.f) || max_ls < 0) return NADMM_EINVAL;
  if (max_ls > NADMM_MAX_LS) return NADMM_EUNSUPPORTED;
  return NADMM_OK;
}

}  // namespace
}  // namespace nadmm

using namespace nadmm;

static int validate_params(const nadmm_params* params) {
  if (params == nullptr) return NADMM_EINVAL;
  if (params->max_newton < 0 || params->max_cg < 0 || !(params->cg_tol >= 0.f) || !(params->grad_tol >= 0.f))
    return NADMM_EINVAL;
  return validate_ls(params->armijo_beta, params->backtrack_gamma, params->max_ls);
}

// Enqueues Algorithm 3 (arguments already validated).  outer_flag: see launch_state_init.
// use_hist: the workspace holds L.hist_bufs >= max_cg buffers for the directional logits of the CG sweeps.  The step p is
// sum_k alpha_k d_k over the iterations taken, so A p = sum_k alpha_k (A d_k), and every sweep has A d_k in hand: it
// stores it (n (C-1) floats), and the line search puts A p together from them instead of a further pass over A.
static int local_newton_enqueue(const nadmm_problem* prob, float* d_X, const nadmm_params* params, const Layout& L,
                                int path, void* d_ws, const int32_t* outer_flag, hipStream_t st, bool use_hist = false) {
  int rc = NADMM_OK;
  DevState* ds = at<DevState>(d_ws, L.state);
  float* g = at<float>(d_ws, L.g);
  float* pdir = at<float>(d_ws, L.pdir);
  float* r = at<float>(d_ws, L.r);
  float* dvec = at<float>(d_ws, L.dvec);

  if (path == 5 && (rc = sparse_plan(prob, L, d_ws, st)) != NADMM_OK) return rc;
  NADMM_HIP(launch_state_init(ds, outer_flag, st));
  const int ncand = params->max_ls + 2;

  for (int t = 0; t < params->max_newton; ++t) {
    // gradient and objective at X; caches the probabilities and the logits A X
    RowArgs ra = blank_rows();
    ra.kind = kRowsGrad;
    ra.B0 = d_X;
    ra.labels = prob->d_labels;
    ra.rows_out = at<float>(d_ws, L.drows);
    ra.Pout = at<float>(d_ws, L.pcache);
    ra.Z0out = at<float>(d_ws, L.zx);
    ra.loss_part = at<double>(d_ws, L.loss_part);
    ra.flag = &ds->newton_active;
    int nparts = 0;
    if ((rc = sweep(prob, L, path, d_ws, ra, true, &nparts, st)) != NADMM_OK) return rc;
    {
      // gradient; the same kernel leaves the partial sums of the penalty terms and of ||g||^2 and starts CG (p = 0, r = d = -g)
      ReduceArgs rg = reduce_args(prob, L, d_ws, nparts, 1, d_X, g, nullptr, &ds->newton_active);
      rg.pen_part = at<double>(d_ws, L.headpart);
      rg.gg_part = rg.pen_part + reduce_out_blocks(L.s.d);
      rg.cg_p = pdir;
      rg.cg_r = r;
      rg.cg_d = dvec;
      NADMM_HIP(launch_reduce_out(rg, st));
    }

    NewtonHeadArgs nh;
    std::memset(&nh, 0, sizeof(nh));
    nh.st = ds;
    nh.loss_part = at<double>(d_ws, L.loss_part);
    nh.nblocks = loss_blocks(L, path);
    nh.scale = prob->loss_scale;
    nh.lambda = prob->lambda;
    nh.rho = prob->rho;
    nh.X = d_X;
    nh.z = prob->d_z;
    nh.y = prob->d_y;
    nh.g = g;
    nh.pdir = pdir;
    nh.r = r;
    nh.dvec = dvec;
    nh.d = L.s.d;
    nh.iter = t;
    nh.grad_tol = params->grad_tol;
    nh.newton_mode = 1;
    nh.pen_part = at<double>(d_ws, L.headpart);
    nh.gg_part = nh.pen_part + reduce_out_blocks(L.s.d);
    nh.npart = reduce_out_blocks(L.s.d);
    nh.rho_scale = L.rho_scale;
    // on the fused path the head is one more workgroup of the first CG iteration's reduction instead of a launch of its own
    const bool head_in_reduce = cg_deferred(path) && params->max_cg >= 1 && L.s.d <= kReduceFinishMax;
    if (!head_in_reduce) NADMM_HIP(launch_newton_head(nh, st));

    // CG on H p = -g with the probabilities of this iterate
    const bool thin_def = thin_deferred(path) && params->max_cg >= 1;
    const bool hist = use_hist && cg_deferred(path) && params->max_cg >= 1 && params->max_cg <= L.hist_bufs;
    const size_t hist_stride = align256((size_t)L.s.n * L.s.NC * sizeof(float)) / sizeof(float);
    for (int k = 0; k < params->max_cg; ++k) {
      float* w_rows = hist ? at<float>(d_ws, L.hist) + (size_t)k * hist_stride : nullptr;
      if ((rc = cg_iteration(prob, L, path, d_ws, ds, nullptr, false, params->cg_tol, k, st, w_rows,
                             (k == 0 && head_in_reduce) ? &nh : nullptr, thin_def)) != NADMM_OK)
        return rc;
    }

    // Armijo backtracking on Z(alpha) = A X + alpha A p, then X += alpha p.  With the deferred CG update the sweep
    // that forms A p applies the last update first and leaves p in its own buffer.
    const bool pend = (cg_deferred(path) || thin_def) && params->max_cg > 0;
    float* pstep = pend ? at<float>(d_ws, L.pfinal) : pdir;
    RowArgs rz = blank_rows();
    rz.kind = kRowsLogits;
    rz.B1 = pstep;
    rz.Z1out = at<float>(d_ws, L.zp);
    rz.flag = &ds->newton_active;
    const bool eval_finishes = hist && ls_eval_takes_pending(prob->n);  // the row kernel of the line search applies the last update
    if (hist) {  // A p comes from the history; the last update alone, unless the line search's row kernel takes it along
      if (!eval_finishes)
        NADMM_HIP(launch_cg_pending_finish(cg_pend(L, d_ws, ds, (params->max_cg - 1) & 1, true, params->cg_tol), st));
    } else if (pend) {
      const CgPend c = cg_pend(L, d_ws, ds, (params->max_cg - 1) & 1, true, params->cg_tol);
      if (thin_def) {  // the last sweep's partial sums are added up by this pass as well
        const ReduceArgs prev = thin_prev(prob, L, d_ws, params->max_cg - 1);
        if ((rc = sweep(prob, L, path, d_ws, rz, false, &nparts, st, &c, &prev)) != NADMM_OK) return rc;
      } else if ((rc = sweep(prob, L, path, d_ws, rz, false, &nparts, st, &c)) != NADMM_OK) {
        return rc;
      }
    } else if ((rc = sweep(prob, L, path, d_ws, rz, false, &nparts, st)) != NADMM_OK) {
      return rc;
    }

    LsEvalArgs le;
    std::memset(&le, 0, sizeof(le));
    le.Zx = at<float>(d_ws, L.zx);
    le.Zp = hist ? nullptr : at<float>(d_ws, L.zp);
    le.hist = hist ? at<float>(d_ws, L.hist) : nullptr;
    le.hist_stride = (int64_t)hist_stride;
    le.nbuf = hist ? params->max_cg : 0;
    if (eval_finishes) {
      le.has_pend = 1;
      le.pend = cg_pend(L, d_ws, ds, (params->max_cg - 1) & 1, true, params->cg_tol);
    }
    le.st = ds;
    le.labels = prob->d_labels;
    le.n = prob->n;
    le.NC = L.s.NC;
    fill_alphas(le.alphas, ncand, params->backtrack_gamma);
    le.ncand = ncand;
    le.lpart = at<double>(d_ws, L.lpart);
    le.flag = &ds->newton_active;
    NADMM_HIP(launch_ls_eval(le, st));

    LsTailArgs lt;
    std::memset(&lt, 0, sizeof(lt));
    lt.st = ds;
    lt.lpart = le.lpart;
    lt.nblocks = ls_eval_blocks(prob->n);
    lt.ncand = ncand;
    lt.zero_slot = -1;
    std::memcpy(lt.alphas, le.alphas, sizeof(lt.alphas));
    lt.use_state_loss = 1;
    lt.scale = prob->loss_scale;
    lt.lambda = prob->lambda;
    lt.rho = prob->rho;
    lt.beta = params->armijo_beta;
    lt.X = d_X;
    lt.z = prob->d_z;
    lt.y = prob->d_y;
    lt.pdir = pstep;
    lt.g = g;
    lt.d = L.s.d;
    lt.X_apply = d_X;
    lt.iter = t;
    lt.flag = &ds->newton_active;
    lt.rho_scale = L.rho_scale;
    lt.qpart = at<double>(d_ws, L.dotpart);
    NADMM_HIP(launch_ls_tail(lt, st));
  }

  return NADMM_OK;
}

struct AdmmLayout {
  size_t state, part, total;
  size_t local[NADMM_MAX_WORKERS];  // one local workspace per worker: their solves run side by side
  int wg_cap;
};

constexpr int kAdmmStreams = 4;  // streams the workers' solves are spread over: the caller's and three internal ones
                                 // (a process has four hardware queues by default; a fifth stream would share one)

static int admm_wg_cap(int32_t N) {
  const int lanes = N < kAdmmStreams ? N : kAdmmStreams;
  return lanes > 1 ? 256 / lanes : 0;
}

static int admm_layout(const nadmm_problem* w, int32_t N, AdmmLayout* AL, int64_t* d_out, int max_cg = 0) {
  if (w == nullptr || N < 1 || N > NADMM_MAX_WORKERS) return NADMM_EINVAL;
  AL->wg_cap = admm_wg_cap(N);
  const int64_t d0 = (int64_t)w[0].p * (w[0].C - 1);
  size_t off = 0;
  AL->state = off; off += align256(sizeof(AdmmState));
  for (int i = 0; i < N; ++i) {
    int rc = validate_problem(&w[i], true);
    if (rc != NADMM_OK) return rc;
    if (w[i].p != w[0].p || w[i].C != w[0].C) return NADMM_EINVAL;
  }
  AL->part = off; off += align256((size_t)admm_blocks(d0) * 5 * sizeof(double));
  for (int i = 0; i < N; ++i) {
    Layout L;
    make_layout(&w[i], &L, false, AL->wg_cap, max_cg);
    AL->local[i] = off;
    off += align256(L.total);
  }
  AL->total = off;
  if (d_out) *d_out = d0;
  return NADMM_OK;
}

// Streams and events of the outer solver, per host thread and device, created on first use and kept.
struct AdmmLanes {
  hipStream_t stream[kAdmmStreams];
  hipEvent_t fork;
  hipEvent_t join[kAdmmStreams];
  bool ready;
};

static int admm_lanes(AdmmLanes** out) {
  thread_local AdmmLanes lanes[kMaxDevices] = {};
  int dev = -1;
  NADMM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return NADMM_EUNSUPPORTED;
  AdmmLanes* l = &lanes[dev];
  if (!l->ready) {
    for (int i = 1; i < kAdmmStreams; ++i) {  // lane 0 is the caller's stream
      NADMM_HIP(hipStreamCreateWithFlags(&l->stream[i], hipStreamNonBlocking));  // default priority
      NADMM_HIP(hipEventCreateWithFlags(&l->join[i], hipEventDisableTiming));
    }
    NADMM_HIP(hipEventCreateWithFlags(&l->fork, hipEventDisableTiming));
    l->ready = true;
  }
  *out = l;
  return NADMM_OK;
}

extern "C" {

int nadmm_version(void) { return 104; }

const char* nadmm_status_string(int code) {
  switch (code) {
    case NADMM_OK: return "ok";
    case NADMM_EINVAL: return "invalid argument";
    case NADMM_EWORKSPACE: return "workspace missing, misaligned or too small";
    case NADMM_EUNSUPPORTED: return "shape or parameter outside the supported range";
    case NADMM_EHIP: return "HIP runtime error";
    case NADMM_ESCRATCH: return "problem needs more scratch memory than the library's built-in buffer holds";
    default: return "unknown status";
  }
}

const char* nadmm_last_hip_error(void) { return g_last_hip_error.c_str(); }

int nadmm_set_kernel_path(int path) {
  if (path < 0 || path > 5) return NADMM_EINVAL;
  const int prev = g_path;
  g_path = path;
  return prev;
}

int nadmm_query_kernel_path(const nadmm_problem* prob) {
  int rc = validate_problem(prob, false);
  if (rc != NADMM_OK) return rc;
  Layout L;
  make_layout(prob, &L);
  int path = 0;
  rc = choose_path(L, &path);
  return rc != NADMM_OK ? rc : path;
}

size_t nadmm_workspace_bytes(const nadmm_problem* prob, const nadmm_params* params) {
  if (validate_problem(prob, false) != NADMM_OK) return 0;
  Layout L;
  make_layout(prob, &L, false, 0, params != nullptr ? params->max_cg : 0);
  return L.total;
}

int nadmm_loss_grad(const nadmm_problem* prob, const float* d_X, double* d_loss, float* d_grad, void* d_ws,
                    size_t ws_bytes, void* stream) {
  int rc = validate_problem(prob, true);
  if (rc != NADMM_OK) return rc;
  if (d_X == nullptr || d_loss == nullptr) return NADMM_EINVAL;
  Layout L;
  make_layout(prob, &L);
  if ((rc = check_ws(L, d_ws, ws_bytes)) != NADMM_OK) return rc;
  int path = 0;
  if ((rc = choose_path(L, &path)) != NADMM_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (path == 5 && (rc = sparse_plan(prob, L, d_ws, st)) != NADMM_OK) return rc;

  RowArgs ra = blank_rows();
  ra.kind = d_grad ? kRowsGrad : kRowsLoss;
  ra.B0 = d_X;
  ra.labels = prob->d_labels;
  ra.rows_out = d_grad ? at<float>(d_ws, L.drows) : nullptr;
  ra.loss_part = at<double>(d_ws, L.loss_part);
  int nparts = 0;
  if ((rc = sweep(prob, L, path, d_ws, ra, d_grad != nullptr, &nparts, st)) != NADMM_OK) return rc;
  if (d_grad) {
    ReduceArgs rg = reduce_args(prob, L, d_ws, nparts, 1, d_X, d_grad, nullptr, nullptr);
    if (L.s.d <= kReduceFinishMax) {  // short vectors: the objective is finished by a workgroup of the same launch
      rg.lf_loss_part = at<double>(d_ws, L.loss_part);
      rg.lf_nblocks = loss_blocks(L, path);
      rg.lf_loss_out = d_loss;
      NADMM_HIP(launch_reduce_out(rg, st));
      return NADMM_OK;
    }
    rg.pen_part = at<double>(d_ws, L.dotpart);  // penalty terms, summed per workgroup on the way
    NADMM_HIP(launch_reduce_out(rg, st));
  }

  LossFinishArgs lf;
  lf.loss_part = at<double>(d_ws, L.loss_part);
  lf.nblocks = loss_blocks(L, path);
  lf.scale = prob->loss_scale;
  lf.lambda = prob->lambda;
  lf.rho = prob->rho;
  lf.X = d_X;
  lf.z = prob->d_z;
  lf.y = prob->d_y;
  lf.d = L.s.d;
  lf.pen_part = d_grad ? at<double>(d_ws, L.dotpart) : nullptr;
  lf.npart = reduce_out_blocks(L.s.d);
  lf.loss_out = d_loss;
  lf.rho_scale = nullptr;
  NADMM_HIP(launch_loss_finish(lf, st));
  return NADMM_OK;
}

int nadmm_hessvec(const nadmm_problem* prob, const float* d_X, const float* d_V, float* d_HV, void* d_ws,
                  size_t ws_bytes, void* stream) {
  int rc = validate_problem(prob, false);
  if (rc != NADMM_OK) return rc;
  if (d_X == nullptr || d_V == nullptr || d_HV == nullptr) return NADMM_EINVAL;
  Layout L;
  make_layout(prob, &L);
  if ((rc = check_ws(L, d_ws, ws_bytes)) != NADMM_OK) return rc;
  int path = 0;
  if ((rc = choose_path(L, &path)) != NADMM_OK) return rc;
  if (path == 5 && (rc = sparse_plan(prob, L, d_ws, (hipStream_t)stream)) != NADMM_OK) return rc;
  return hv_apply(prob, L, path, d_ws, d_X, false, d_V, d_HV, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

size_t nadmm_static_scratch_bytes(void) { return NADMM_STATIC_SCRATCH_BYTES; }

size_t nadmm_hessvec_static_bytes(const nadmm_problem* prob) {
  if (validate_problem(prob, false) != NADMM_OK) return 0;
  Layout L;
  make_layout(prob, &L, true);
  return L.total;
}

int nadmm_hessvec_static(const nadmm_problem* prob, const float* d_X, const float* d_V, float* d_HV, void* stream) {
  int rc = validate_problem(prob, false);
  if (rc != NADMM_OK) return rc;
  if (d_X == nullptr || d_V == nullptr || d_HV == nullptr) return NADMM_EINVAL;
  Layout L;
  make_layout(prob, &L, true);
  if (L.total > (size_t)NADMM_STATIC_SCRATCH_BYTES) return NADMM_ESCRATCH;  // before any device call: host-testable
  int path = 0;
  if ((rc = choose_path(L, &path)) != NADMM_OK) return rc;
  void* ws = nullptr;
  if ((rc = scratch_on_current_device(&ws)) != NADMM_OK) return rc;
  if (path == 5 && (rc = sparse_plan(prob, L, ws, (hipStream_t)stream)) != NADMM_OK) return rc;
  return hv_apply(prob, L, path, ws, d_X, false, d_V, d_HV, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

int nadmm_cg_solve(const nadmm_problem* prob, const float* d_X, const float* d_g, float* d_p, int max_iter,
                   float tol, int32_t* d_iters, float* d_relres, void* d_ws, size_t ws_bytes, void* stream) {
  int rc = validate_problem(prob, false);
  if (rc != NADMM_OK) return rc;
  if (d_X == nullptr || d_g == nullptr || d_p == nullptr || max_iter < 0 || !(tol >= 0.f)) return NADMM_EINVAL;
  Layout L;
  make_layout(prob, &L);
  if ((rc = check_ws(L, d_ws, ws_bytes)) != NADMM_OK) return rc;
  int path = 0;
  if ((rc = choose_path(L, &path)) != NADMM_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  DevState* ds = at<DevState>(d_ws, L.state);
  if (path == 5 && (rc = sparse_plan(prob, L, d_ws, st)) != NADMM_OK) return rc;

  NADMM_HIP(launch_state_init(ds, nullptr, st));
  NewtonHeadArgs nh;
  std::memset(&nh, 0, sizeof(nh));
  nh.st = ds;
  nh.g = d_g;
  nh.pdir = at<float>(d_ws, L.pdir);
  nh.r = at<float>(d_ws, L.r);
  nh.dvec = at<float>(d_ws, L.dvec);
  nh.d = L.s.d;
  nh.newton_mode = 0;
  NADMM_HIP(launch_newton_head(nh, st));

  for (int k = 0; k < max_iter; ++k) {
    if ((rc = cg_iteration(prob, L, path, d_ws, ds, k == 0 ? d_X : nullptr, true, tol, k, st)) != NADMM_OK) return rc;
  }
  const bool pend = cg_deferred(path) && max_iter > 0;
  if (pend) NADMM_HIP(launch_cg_pending_finish(cg_pend(L, d_ws, ds, (max_iter - 1) & 1, true, tol), st));
  CgFinishArgs cf;
  cf.st = ds;
  cf.pdir = pend ? at<float>(d_ws, L.pfinal) : at<float>(d_ws, L.pdir);
  cf.p_out = d_p;
  cf.d = L.s.d;
  cf.iters_out = d_iters;
  cf.relres_out = d_relres;
  NADMM_HIP(launch_cg_finish(cf, st));
  return NADMM_OK;
}

int nadmm_line_search(const nadmm_problem* prob, const float* d_X, const float* d_p, const float* d_g,
                      double loss_at_X, float beta, float gamma, int max_ls, float* d_alpha, double* d_loss_new,
                      int32_t* d_armijo_ok, void* d_ws, size_t ws_bytes, void* stream) {
  int rc = validate_problem(prob, true);
  if (rc != NADMM_OK) return rc;
  if (d_X == nullptr || d_p == nullptr || d_g == nullptr || d_alpha == nullptr) return NADMM_EINVAL;
  if ((rc = validate_ls(beta, gamma, max_ls)) != NADMM_OK) return rc;
  Layout L;
  make_layout(prob, &L);
  if ((rc = check_ws(L, d_ws, ws_bytes)) != NADMM_OK) return rc;
  int path = 0;
  if ((rc = choose_path(L, &path)) != NADMM_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  DevState* ds = at<DevState>(d_ws, L.state);
  if (path == 5 && (rc = sparse_plan(prob, L, d_ws, st)) != NADMM_OK) return rc;
  NADMM_HIP(launch_state_init(ds, nullptr, st));

  RowArgs ra = blank_rows();
  ra.kind = kRowsLogits;
  ra.B0 = d_X;
  ra.B1 = d_p;
  ra.Z0out = at<float>(d_ws, L.zx);
  ra.Z1out = at<float>(d_ws, L.zp);
  int nparts = 0;
  if ((rc = sweep(prob, L, path, d_ws, ra, false, &nparts, st)) != NADMM_OK) return rc;

  const int ncand = max_ls + 2;
  const bool need_f0 = std::isnan(loss_at_X);
  LsEvalArgs le;
  std::memset(&le, 0, sizeof(le));
  le.Zx = at<float>(d_ws, L.zx);
  le.Zp = at<float>(d_ws, L.zp);
  le.labels = prob->d_labels;
  le.n = prob->n;
  le.NC = L.s.NC;
  fill_alphas(le.alphas, ncand, gamma);
  le.alphas[ncand] = 0.f;
  le.ncand = ncand + (need_f0 ? 1 : 0);
  le.lpart = at<double>(d_ws, L.lpart);
  NADMM_HIP(launch_ls_eval(le, st));

  LsTailArgs lt;
  std::memset(&lt, 0, sizeof(lt));
  lt.st = ds;
  lt.lpart = le.lpart;
  lt.nblocks = ls_eval_blocks(prob->n);
  lt.ncand = ncand;
  lt.zero_slot = need_f0 ? ncand : -1;
  std::memcpy(lt.alphas, le.alphas, sizeof(lt.alphas));
  lt.loss_at_X = loss_at_X;
  lt.use_state_loss = 0;
  lt.scale = prob->loss_scale;
  lt.lambda = prob->lambda;
  lt.rho = prob->rho;
  lt.beta = beta;
  lt.X = d_X;
  lt.z = prob->d_z;
  lt.y = prob->d_y;
  lt.pdir = d_p;
  lt.g = d_g;
  lt.d = L.s.d;
  lt.X_apply = nullptr;
  lt.alpha_out = d_alpha;
  lt.loss_new_out = d_loss_new;
  lt.ok_out = d_armijo_ok;
  lt.iter = -1;
  lt.qpart = at<double>(d_ws, L.dotpart);
  NADMM_HIP(launch_ls_tail(lt, st));
  return NADMM_OK;
}

int nadmm_local_newton(const nadmm_problem* prob, float* d_X, const nadmm_params* params, nadmm_stats* h_stats,
                       void* d_ws, size_t ws_bytes, void* stream) {
  int rc = validate_problem(prob, true);
  if (rc != NADMM_OK) return rc;
  if (d_X == nullptr) return NADMM_EINVAL;
  if ((rc = validate_params(params)) != NADMM_OK) return rc;
  Layout L;
  make_layout(prob, &L, false, 0, params->max_cg);
  // the history of directional logits is used if the workspace has room for it (it has if it was sized for these
  // parameters); a workspace sized without parameters still does, with one more pass over A per Newton iteration
  const bool use_hist = L.hist_bufs > 0 && ws_bytes >= L.total;
  if (!use_hist) L.total = L.total_base;
  if ((rc = check_ws(L, d_ws, ws_bytes)) != NADMM_OK) return rc;
  int path = 0;
  if ((rc = choose_path(L, &path)) != NADMM_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = local_newton_enqueue(prob, d_X, params, L, path, d_ws, nullptr, st, use_hist)) != NADMM_OK) return rc;
  DevState* ds = at<DevState>(d_ws, L.state);
  if (h_stats != nullptr) {
    NADMM_HIP(hipMemcpyAsync(h_stats, &ds->stats, sizeof(nadmm_stats), hipMemcpyDeviceToHost, st));
    NADMM_HIP(hipStreamSynchronize(st));
  }
  return NADMM_OK;
}


// ---- ADMM outer solver (Algorithm 1) ----
size_t nadmm_admm_workspace_bytes(const nadmm_problem* h_workers, int32_t N, const nadmm_admm_params* params) {
  AdmmLayout AL;
  if (admm_layout(h_workers, N, &AL, nullptr, params != nullptr ? params->local.max_cg : 0) != NADMM_OK) return 0;
  return AL.total;
}

int nadmm_admm_consensus(int32_t N, int64_t d, const float* d_x, float* d_u, float* d_z, const float* h_rho,
                         float lambda, float eps_abs, float eps_rel, double* d_out,
                         void* d_ws, size_t ws_bytes, void* stream) {
  if (N < 1 || N > NADMM_MAX_WORKERS || d < 1 || d_x == nullptr || d_u == nullptr || d_z == nullptr || h_rho == nullptr)
    return NADMM_EINVAL;
  if (!(lambda >= 0.f) || !(eps_abs >= 0.f) || !(eps_rel >= 0.f)) return NADMM_EINVAL;
  const size_t need = align256((size_t)admm_blocks(d) * 5 * sizeof(double));
  if (d_ws == nullptr || ((uintptr_t)d_ws & 255) != 0 || ws_bytes < need) return NADMM_EWORKSPACE;
  AdmmConsensusArgs a;
  std::memset(&a, 0, sizeof(a));
  a.x = d_x; a.u = d_u; a.z = d_z; a.N = N; a.d = d;
  for (int i = 0; i < N; ++i) {
    if (!(h_rho[i] > 0.f) || !std::isfinite(h_rho[i])) return NADMM_EINVAL;
    a.rho[i] = h_rho[i];
  }
  a.lambda = lambda; a.eps_abs = eps_abs; a.eps_rel = eps_rel;
  a.part = static_cast<double*>(d_ws);
  a.out = d_out;
  NADMM_HIP(launch_admm_consensus(a, (hipStream_t)stream));
  return NADMM_OK;
}

int nadmm_admm_solve(const nadmm_problem* h_workers, int32_t N, float lambda, float* d_x, float* d_u, float* d_z,
                     const nadmm_admm_params* params, nadmm_admm_stats* h_stats,
                     void* d_ws, size_t ws_bytes, void* stream) {
  AdmmLayout AL;
  int64_t d = 0;
  int rc = admm_layout(h_workers, N, &AL, &d, params != nullptr ? params->local.max_cg : 0);
  if (rc != NADMM_OK) return rc;
  if (d_x == nullptr || d_u == nullptr || d_z == nullptr || params == nullptr) return NADMM_EINVAL;
  // room for the workers' histories of directional logits (see nadmm_local_newton), else the layout without them
  bool use_hist = ws_bytes >= AL.total;
  if (!use_hist && (rc = admm_layout(h_workers, N, &AL, &d, 0)) != NADMM_OK) return rc;
  if (params->max_outer < 0 || !(lambda >= 0.f) || !std::isfinite(lambda) || !(params->eps_abs >= 0.f) ||
      !(params->eps_rel >= 0.f))
    return NADMM_EINVAL;
  if (params->penalty_rule != 0 && params->penalty_rule != 1) return NADMM_EINVAL;
  if (params->penalty_rule == 1 && (!(params->rb_mu >= 1.f) || !(params->rb_tau > 1.f) || !std::isfinite(params->rb_mu) ||
                                    !std::isfinite(params->rb_tau)))
    return NADMM_EINVAL;
  if ((rc = validate_params(&params->local)) != NADMM_OK) return rc;
  if (d_ws == nullptr || ((uintptr_t)d_ws & 255) != 0 || ws_bytes < AL.total) return NADMM_EWORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  AdmmState* as = at<AdmmState>(d_ws, AL.state);

  // per-worker subproblems: no local regulariser, consensus variable and multipliers of this call
  nadmm_problem wk[NADMM_MAX_WORKERS];
  Layout Ls[NADMM_MAX_WORKERS];
  int paths[NADMM_MAX_WORKERS];
  AdmmConsensusArgs ca;
  std::memset(&ca, 0, sizeof(ca));
  for (int i = 0; i < N; ++i) {
    wk[i] = h_workers[i];
    wk[i].lambda = 0.f;
    wk[i].d_z = d_z;
    wk[i].d_y = d_u + (size_t)i * d;
    make_layout(&wk[i], &Ls[i], false, AL.wg_cap, use_hist ? params->local.max_cg : 0);
    Ls[i].rho_scale = &as->rho_scale;
    if ((rc = choose_path(Ls[i], &paths[i])) != NADMM_OK) return rc;
    ca.rho[i] = wk[i].rho;
  }
  ca.st = as; ca.x = d_x; ca.u = d_u; ca.z = d_z; ca.N = N; ca.d = d;
  ca.lambda = lambda; ca.eps_abs = params->eps_abs; ca.eps_rel = params->eps_rel;
  ca.penalty_rule = params->penalty_rule; ca.rb_mu = params->rb_mu; ca.rb_tau = params->rb_tau;
  ca.part = at<double>(d_ws, AL.part);

  // The workers' local solves of one outer iteration are independent: they are spread over a few internal streams
  // (forked from and joined to the caller's stream with events, each worker on its own workspace), so that their
  // launch latencies and tails overlap; the consensus step runs on the caller's stream after the join.
  AdmmLanes* lanes = nullptr;
  const int nlanes = N < kAdmmStreams ? N : kAdmmStreams;
  if (nlanes > 1 && (rc = admm_lanes(&lanes)) != NADMM_OK) return rc;
  // With a residual test the host looks at the stopping flag every few iterations instead of enqueueing max_outer
  // iterations of no-ops (not while the stream is being captured into a graph, where it cannot wait).
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  NADMM_HIP(hipStreamIsCapturing(st, &cap));
  const bool poll = (params->eps_abs > 0.f || params->eps_rel > 0.f) && cap == hipStreamCaptureStatusNone;
  constexpr int kPollEvery = 4;

  NADMM_HIP(launch_admm_init(as, d_u, d_z, N, d, st));
  for (int k = 0; k < params->max_outer; ++k) {
    if (nlanes > 1) {
      NADMM_HIP(hipEventRecord(lanes->fork, st));
      for (int l = 1; l < nlanes; ++l) NADMM_HIP(hipStreamWaitEvent(lanes->stream[l], lanes->fork, 0));
    }
    for (int i = 0; i < N; ++i) {
      hipStream_t si = (nlanes > 1 && i % nlanes != 0) ? lanes->stream[i % nlanes] : st;
      rc = local_newton_enqueue(&wk[i], d_x + (size_t)i * d, &params->local, Ls[i], paths[i], at<char>(d_ws, AL.local[i]),
                                &as->active, si, use_hist && Ls[i].hist_bufs > 0);
      if (rc != NADMM_OK) return rc;
    }
    if (nlanes > 1) {
      for (int l = 1; l < nlanes; ++l) {
        NADMM_HIP(hipEventRecord(lanes->join[l], lanes->stream[l]));
        NADMM_HIP(hipStreamWaitEvent(st, lanes->join[l], 0));
      }
    }
    ca.iter = k;
    NADMM_HIP(launch_admm_consensus(ca, st));
    if (poll && (k + 1) % kPollEvery == 0 && k + 1 < params->max_outer) {
      int32_t active = 1;
      NADMM_HIP(hipMemcpyAsync(&active, &as->active, sizeof(active), hipMemcpyDeviceToHost, st));
      NADMM_HIP(hipStreamSynchronize(st));
      if (active == 0) break;
    }
  }
  if (h_stats != nullptr) {
    NADMM_HIP(hipMemcpyAsync(h_stats, &as->stats, sizeof(nadmm_admm_stats), hipMemcpyDeviceToHost, st));
    NADMM_HIP(hipStreamSynchronize(st));
  }
  return NADMM_OK;
}

}  // extern "C"
