// Small kernels on vectors of length d = p (C-1) and on the n x (C-1) logit caches:
// fixed-order reduction of per-workgroup partials, the scalar work of CG
// (Section 2.4), the Armijo backtracking of Algorithm 2 on cached logits, and
// the bookkeeping of Algorithm 3.  All scalars stay in device memory; the
// single-workgroup "tail" kernels sum in a fixed order, so results are
// reproducible bit for bit.
#include "nadmm_internal.h"
#include "nadmm_cgstep.h"
#include "nadmm_mfma.h"

namespace nadmm {
namespace {

constexpr int kTail = 1024;

// Sum over the wave in every lane: rotations inside rows of 16 lanes and the four row totals in a fixed order (a tree of
// cross-lane shuffles of a double is twelve trips through the LDS pipe, one after the other).
__device__ __forceinline__ double wave_sum(double v) { return mfma_detail::wave64_sum(v); }

// Sum over the whole workgroup (fixed order); result valid in every thread.
__device__ __forceinline__ double block_sum(double v, double* sm /* >= 17 doubles */) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nw = (blockDim.x + 63) >> 6;
  __syncthreads();  // previous users of sm are done
  if (lane == 0) sm[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < nw; ++w) t += sm[w];
  return t;
}

// The objective finished by one workgroup of 256 threads that runs beside the reduction of a gradient's partial sums
// (ReduceArgs.lf_*): the row losses' partial sums are complete, the penalty terms come from X, z, y themselves.
// All of a piece's loads (32 elements per vector and thread) are requested before the first is used.
__device__ __forceinline__ void reduce_loss_finish_role(const ReduceArgs& a) {
  __shared__ double smd[17];
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;
  constexpr int PER = 32;
  const double inv_rho = 1.0 / (double)rho_;
  // no load under a condition: a missing z or y reads X instead and counts with factor 0
  const float* __restrict__ zp = a.z != nullptr ? a.z : a.X;
  const float* __restrict__ yp = a.y != nullptr ? a.y : a.X;
  const double zf = a.z != nullptr ? 1.0 : 0.0, yf = a.y != nullptr ? inv_rho : 0.0;
  double acc = 0.0;
  auto term = [&](float xf, float zv, float yv) {
    const double x = xf;
    const double uu = x - zf * (double)zv + yf * (double)yv;
    return 0.5 * (double)a.lambda * x * x + 0.5 * (double)rho_ * uu * uu;
  };
  int64_t done = 0;  // elements handled by the 16-byte path
  if ((((uintptr_t)a.X | (uintptr_t)zp | (uintptr_t)yp) & 15) == 0) {  // uniform
    constexpr int PQ = PER / 4;
    const int64_t n4 = a.d >> 2;
    for (int64_t base = threadIdx.x; base < n4; base += (int64_t)PQ * 256) {
      float4 xq[PQ], zq[PQ], yq[PQ];
#pragma unroll
      for (int u = 0; u < PQ; ++u) {
        const int64_t k = base + (int64_t)u * 256;
        const int64_t kc = k < n4 ? k : n4 - 1;
        xq[u] = reinterpret_cast<const float4*>(a.X)[kc];
        zq[u] = reinterpret_cast<const float4*>(zp)[kc];
        yq[u] = reinterpret_cast<const float4*>(yp)[kc];
      }
#pragma unroll
      for (int u = 0; u < PQ; ++u)
        if (base + (int64_t)u * 256 < n4)
          acc += (term(xq[u].x, zq[u].x, yq[u].x) + term(xq[u].y, zq[u].y, yq[u].y)) +
                 (term(xq[u].z, zq[u].z, yq[u].z) + term(xq[u].w, zq[u].w, yq[u].w));
    }
    done = n4 << 2;
  }
  for (int64_t base = done + threadIdx.x; base < a.d; base += (int64_t)PER * 256) {
    float xv[PER], zv[PER], yv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int64_t e = base + (int64_t)u * 256;
      const int64_t ec = e < a.d ? e : a.d - 1;
      xv[u] = a.X[ec];
      zv[u] = zp[ec];
      yv[u] = yp[ec];
    }
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if (base + (int64_t)u * 256 < a.d) acc += term(xv[u], zv[u], yv[u]);
  }
  double data = 0.0;
  for (int k = threadIdx.x; k < a.lf_nblocks; k += 256) data += a.lf_loss_part[k];
  const double pen = block_sum(acc, smd);
  data = block_sum(data, smd);
  if (threadIdx.x == 0) *a.lf_loss_out = (double)a.scale * data + pen;
}

// out[e] = s * sum_k partial[k][e] + linear terms.  A workgroup covers 32 elements; its 8
// thread groups each sum every 8th partial (independent loads in flight), then the 8 group sums
// are added in a fixed order, so the result does not depend on scheduling.
__device__ __forceinline__ void newton_head_body(const NewtonHeadArgs& a);  // defined below

// FINISH: launched with one workgroup more, which finishes the objective after a gradient pass or does the work of
// newton_head_kernel beside the first reduction of a CG solve (an instantiation of its own: that workgroup's registers
// would cost the plain kernel its occupancy on long vectors).
template <bool FINISH>
__global__ __launch_bounds__(256) void reduce_out_kernel(const ReduceArgs a) {
  if (FINISH && blockIdx.x == gridDim.x - 1) {  // the workgroup beyond the last 32 elements
    if (a.has_head != 0) newton_head_body(a.head);  // looks at the state's own activity flag
    else if (a.flag == nullptr || *a.flag != 0) reduce_loss_finish_role(a);
    return;
  }
  __shared__ float sm[8][32];
  const int el = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int64_t e = (int64_t)blockIdx.x * 32 + el;
  const bool ok = e < a.d;
  const int64_t ec = ok ? e : a.d - 1;
  // Every load is requested before the first result is needed: the vectors of the linear terms (clamped index, all
  // threads, so that no load sits under a condition), then the partials; only then the activity flag is looked at.
  float lin0 = 0.f, lin1 = 0.f, lin2 = 0.f;
  if (a.kind == 0) {
    lin0 = a.V[ec];
    lin1 = a.V_alt != nullptr ? a.V_alt[ec] : 0.f;
  } else {
    lin0 = a.X[ec];
    lin1 = a.z != nullptr ? a.z[ec] : 0.f;
    lin2 = a.y != nullptr ? a.y[ec] : 0.f;
  }
  const float* __restrict__ pp = a.partial + ec;
  float sum = 0.f;
  int k = grp;
  float v[16];
  const bool first_batch = k + 8 * 15 < a.nparts;  // uniform: the same for all 8 thread groups
  if (first_batch) {
#pragma unroll
    for (int t = 0; t < 16; ++t) v[t] = pp[(size_t)(k + 8 * t) * a.d];
  }
  if (a.flag != nullptr && *a.flag == 0) return;
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  if (first_batch) {
#pragma unroll
    for (int t = 0; t < 16; ++t) sum += v[t];
    k += 8 * 16;
  }
  for (; k + 8 * 15 < a.nparts; k += 8 * 16) {  // 16 independent loads in flight, summed in order
#pragma unroll
    for (int t = 0; t < 16; ++t) v[t] = pp[(size_t)(k + 8 * t) * a.d];
#pragma unroll
    for (int t = 0; t < 16; ++t) sum += v[t];
  }
  for (; k < a.nparts; k += 8) sum += pp[(size_t)k * a.d];
  sm[grp][el] = sum;
  __syncthreads();
  if (grp != 0) return;
#pragma unroll
  for (int g = 1; g < 8; ++g) sum += sm[g][el];
  float out = a.scale * sum;
  double prod = 0.0, pen = 0.0;
  if (ok) {
    if (a.kind == 0) {
      const float vv = (a.cur != nullptr && *a.cur != 0) ? lin1 : lin0;
      out = fmaf(a.lambda + rho_, vv, out);
      prod = (double)out * (double)vv;
    } else {
      const float x = lin0, zz = lin1, yy = lin2;
      out += a.lambda * x + rho_ * (x - zz) + yy;
      const double xd = x, u = xd - (double)zz + (double)yy / (double)rho_;
      pen = 0.5 * (double)a.lambda * xd * xd + 0.5 * (double)rho_ * u * u;
      prod = (double)out * (double)out;
      if (a.cg_p != nullptr) {
        a.cg_p[e] = 0.f;
        a.cg_r[e] = -out;
        a.cg_d[e] = -out;
      }
    }
    a.out[e] = out;
  }
  // the 32 values of this workgroup, summed in a fixed order by lane 0
  double* first = a.kind == 0 ? a.dot_part : a.gg_part;
  if (first != nullptr) {
    prod = mfma_detail::half32_sum(prod);
    if (el == 0) first[blockIdx.x] = prod;
  }
  if (a.kind != 0 && a.pen_part != nullptr) {
    pen = mfma_detail::half32_sum(pen);
    if (el == 0) a.pen_part[blockIdx.x] = pen;
  }
}

// The same reduction for long vectors (d > kWideFrom: sparse data with hundreds of thousands of features),
// where there are few partials per element and many elements: a workgroup covers kWideChunk consecutive
// elements, 8 per thread with all loads of a partial in flight together, and adds the partials in order.
constexpr int64_t kWideFrom = (int64_t)1 << 18;
constexpr int kWidePer = 8;
constexpr int kWideChunk = 256 * kWidePer;

__global__ __launch_bounds__(256) void reduce_out_wide_kernel(const ReduceArgs a) {
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ double sm[17];
  const int64_t base = (int64_t)blockIdx.x * kWideChunk + threadIdx.x;
  float sum[kWidePer];
#pragma unroll
  for (int u = 0; u < kWidePer; ++u) sum[u] = 0.f;
  for (int k = 0; k < a.nparts; ++k) {
    const float* __restrict__ pp = a.partial + (size_t)k * a.d;
    float v[kWidePer];
#pragma unroll
    for (int u = 0; u < kWidePer; ++u) {
      const int64_t e = base + u * 256;
      v[u] = e < a.d ? pp[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kWidePer; ++u) sum[u] += v[u];
  }
  float xv[kWidePer], zv[kWidePer], yv[kWidePer];
#pragma unroll
  for (int u = 0; u < kWidePer; ++u) {
    const int64_t e = base + u * 256;
    const bool ok = e < a.d;
    xv[u] = ok ? (a.kind == 0 ? a.V[e] : a.X[e]) : 0.f;
    zv[u] = (ok && a.kind != 0 && a.z) ? a.z[e] : 0.f;
    yv[u] = (ok && a.kind != 0 && a.y) ? a.y[e] : 0.f;
  }
  double prod = 0.0, pen = 0.0;
#pragma unroll
  for (int u = 0; u < kWidePer; ++u) {
    const int64_t e = base + u * 256;
    if (e >= a.d) continue;
    float out = a.scale * sum[u];
    if (a.kind == 0) {
      out = fmaf(a.lambda + rho_, xv[u], out);
      prod += (double)out * (double)xv[u];
    } else {
      const float x = xv[u];
      out += a.lambda * x + rho_ * (x - zv[u]) + yv[u];
      const double xd = x, uu = xd - (double)zv[u] + (double)yv[u] / (double)rho_;
      pen += 0.5 * (double)a.lambda * xd * xd + 0.5 * (double)rho_ * uu * uu;
      prod += (double)out * (double)out;
      if (a.cg_p != nullptr) {
        a.cg_p[e] = 0.f;
        a.cg_r[e] = -out;
        a.cg_d[e] = -out;
      }
    }
    a.out[e] = out;
  }
  double* first = a.kind == 0 ? a.dot_part : a.gg_part;
  if (first != nullptr) {
    prod = block_sum(prod, sm);
    if (threadIdx.x == 0) first[blockIdx.x] = prod;
  }
  if (a.kind != 0 && a.pen_part != nullptr) {
    pen = block_sum(pen, sm);
    if (threadIdx.x == 0) a.pen_part[blockIdx.x] = pen;
  }
}

// The single-workgroup tail kernels walk vectors of d elements.  Loads go out in blocks of kBlk per
// vector and thread before any of them is used, so that a pass costs a few memory round trips
// instead of one per element and thread.
constexpr int kBlk = 4;

// lambda/2 ||X||^2 + rho/2 ||X - z + y/rho||^2, summed over the workgroup
__device__ __forceinline__ double penalty_block(const float* X, const float* z, const float* y, int64_t d,
                                                float lambda, float rho, double* sm) {
  double acc = 0.0;
  const double inv_rho = 1.0 / (double)rho;
  for (int64_t e0 = threadIdx.x; e0 < d; e0 += (int64_t)kBlk * blockDim.x) {
    float xv[kBlk], zv[kBlk], yv[kBlk];
#pragma unroll
    for (int u = 0; u < kBlk; ++u) {
      const int64_t e = e0 + (int64_t)u * blockDim.x;
      const bool ok = e < d;
      xv[u] = ok ? X[e] : 0.f;
      zv[u] = (ok && z) ? z[e] : 0.f;
      yv[u] = (ok && y) ? y[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kBlk; ++u) {
      const double x = xv[u];
      const double uu = x - (double)zv[u] + (double)yv[u] * inv_rho;
      acc += 0.5 * (double)lambda * x * x + 0.5 * (double)rho * uu * uu;  // zero for the padding (x = z = y = 0)
    }
  }
  return block_sum(acc, sm);
}

__device__ __forceinline__ double partial_sum_block(const double* part, int n, double* sm) {
  double acc = 0.0;
  for (int k0 = threadIdx.x; k0 < n; k0 += kBlk * blockDim.x) {
    double v[kBlk];
#pragma unroll
    for (int u = 0; u < kBlk; ++u) {
      const int k = k0 + u * blockDim.x;
      v[u] = k < n ? part[k] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < kBlk; ++u) acc += v[u];
  }
  return block_sum(acc, sm);
}

__global__ __launch_bounds__(kTail) void loss_finish_kernel(const LossFinishArgs a) {
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  __shared__ double sm[17];
  const double data = partial_sum_block(a.loss_part, a.nblocks, sm);
  const double pen = a.pen_part ? partial_sum_block(a.pen_part, a.npart, sm)
                                : penalty_block(a.X, a.z, a.y, a.d, a.lambda, rho_, sm);
  if (threadIdx.x == 0) *a.loss_out = (double)a.scale * data + pen;
}

__global__ void state_init_kernel(DevState* st, const int32_t* outer_flag) {
  // one thread; zero the scalars and the statistics, raise the activity flags
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->loss = 0.0; st->gg = 0.0; st->rr = 0.0; st->gg_cg = 0.0; st->loss_new = 0.0; st->loss_initial = 0.0;
  st->alpha = 0.f;
  st->newton_active = outer_flag ? *outer_flag : 1; st->cg_active = st->newton_active; st->cg_iters = 0; st->armijo_ok = 1; st->ls_evals = 0;
  st->cg_go = 0; st->cg_ok = 1; st->cg_alpha = 0.f; st->rr_prev = 0.0;
  nadmm_stats* s = &st->stats;
  s->newton_iters = 0; s->cg_iters_total = 0; s->ls_evals_total = 0; s->armijo_failed = 0;
  s->loss_initial = 0.0; s->loss_final = 0.0; s->grad_norm_final = 0.0;
  for (int i = 0; i < NADMM_TRACE_LEN; ++i) {
    s->alpha[i] = 0.f; s->cg_iters[i] = 0; s->loss[i] = 0.0; s->grad_norm[i] = 0.0;
  }
}

// After a gradient evaluation: finish the objective, ||g||, the stopping test of
// Algorithm 3, and start CG from p = 0, r = d = -g.
// (a device function: it runs as a kernel of its own or as one workgroup of the reduction that follows the first
// Hessian-vector sweep of a CG solve, ReduceArgs.has_head; any workgroup size that is a multiple of 64)
__device__ __forceinline__ void newton_head_body(const NewtonHeadArgs& a) {
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  __shared__ double sm[17];
  DevState* st = a.st;
  if (a.newton_mode && st->newton_active == 0) {
    if (threadIdx.x == 0) st->cgs[0] = CgSlot{0.0, 0, 0, 0, 0};  // a stopped Newton iteration leaves CG inactive
    return;
  }

  double gg = 0.0;
  if (a.gg_part != nullptr) {
    gg = partial_sum_block(a.gg_part, a.npart, sm);  // the reduction has written p, r, d already
  } else {
    for (int64_t e0 = threadIdx.x; e0 < a.d; e0 += (int64_t)kBlk * blockDim.x) {
      float gv[kBlk];
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        const int64_t e = e0 + (int64_t)u * blockDim.x;
        gv[u] = e < a.d ? a.g[e] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        const int64_t e = e0 + (int64_t)u * blockDim.x;
        gg += (double)gv[u] * (double)gv[u];
        if (e < a.d) {
          a.pdir[e] = 0.f;
          a.r[e] = -gv[u];
          a.dvec[e] = -gv[u];
        }
      }
    }
    gg = block_sum(gg, sm);
  }

  double loss = 0.0;
  if (a.newton_mode) {
    const double data = partial_sum_block(a.loss_part, a.nblocks, sm);
    const double pen = a.pen_part ? partial_sum_block(a.pen_part, a.npart, sm)
                                  : penalty_block(a.X, a.z, a.y, a.d, a.lambda, rho_, sm);
    loss = (double)a.scale * data + pen;
  }
  if (threadIdx.x == 0) {
    st->gg = gg;
    st->rr = gg;
    st->gg_cg = gg;
    st->cg_iters = 0;
    st->cg_active = gg > 0.0 ? 1 : 0;
    int32_t cg_on = st->cg_active;
    if (a.newton_mode && (sqrt(gg) < (double)a.grad_tol || !(gg > 0.0))) cg_on = 0;
    st->cgs[0] = CgSlot{gg, cg_on, 0, 0, 0};
    if (a.newton_mode) {
      const double gn = sqrt(gg);
      st->loss = loss;
      nadmm_stats* s = &st->stats;
      if (a.iter == 0) { st->loss_initial = loss; s->loss_initial = loss; s->loss_final = loss; }
      s->grad_norm_final = gn;
      if (gn < (double)a.grad_tol || !(gg > 0.0)) {
        st->newton_active = 0;
        st->cg_active = 0;
      } else if (a.iter < NADMM_TRACE_LEN) {
        s->loss[a.iter] = loss;
        s->grad_norm[a.iter] = gn;
      }
    }
  }
}

__global__ __launch_bounds__(kTail) void newton_head_kernel(const NewtonHeadArgs a) { newton_head_body(a); }

// One CG iteration's vector work, given q = H d:  a = rr / <d,q>; p += a d; r -= a q;
// stop on ||r|| <= tol ||g|| (eq. inexact); else d = r + (rr'/rr) d.
// <d, q> arrives as partial sums from the reduction that formed q.  Every vector is then read once:
// pass 1 forms the new residual (kept in registers, d <= PER * 1024) and its norm, pass 2 updates the
// iterate and the direction.  Loads go out in blocks of 8 per vector and thread.  One workgroup: for
// short vectors a second launch would cost more than the serial work.
template <int PER>
__global__ __launch_bounds__(kTail) void cg_update_kernel(const CgUpdateArgs a) {
  __shared__ double sm[17];
  DevState* st = a.st;
  if (st->cg_active == 0) return;
  constexpr int U = 8;
  constexpr int N = PER > 0 ? PER : U;
  static_assert(N % U == 0, "blocks of 8");
  constexpr int kUnroll = PER > 0 ? PER / U : 1;
  const int nblk = PER > 0 ? PER / U : (int)((a.d + (int64_t)U * kTail - 1) / ((int64_t)U * kTail));
  const double dq = partial_sum_block(a.dot_part, a.ndot, sm);
  const double rr = st->rr;
  const double gg = st->gg_cg;
  if (!(dq > 0.0) || !isfinite(dq)) {  // no positive curvature: keep the current iterate
    __syncthreads();
    if (threadIdx.x == 0) st->cg_active = 0;
    return;
  }
  const float al = (float)(rr / dq);
  float rn[N];
  double rr_new = 0.0;
#pragma unroll kUnroll
  for (int b = 0; b < nblk; ++b) {
    float y[U], re[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t e = threadIdx.x + (int64_t)(b * U + u) * kTail;
      const bool ok = e < a.d;
      y[u] = ok ? a.q[e] : 0.f;
      re[u] = ok ? a.r[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t e = threadIdx.x + (int64_t)(b * U + u) * kTail;
      const float v = fmaf(-al, y[u], re[u]);
      rn[PER > 0 ? b * U + u : u] = v;
      if (e < a.d) a.r[e] = v;
      rr_new += (double)v * (double)v;
    }
  }
  rr_new = block_sum(rr_new, sm);
  const bool stop = sqrt(rr_new) <= (double)a.tol * sqrt(gg);
  const float be = (float)(rr_new / rr);
  // every thread re-reads only elements of r that it wrote itself
#pragma unroll kUnroll
  for (int b = 0; b < nblk; ++b) {
    float x[U], pe[U], re[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t e = threadIdx.x + (int64_t)(b * U + u) * kTail;
      const bool ok = e < a.d;
      x[u] = ok ? a.dvec[e] : 0.f;
      pe[u] = ok ? a.pdir[e] : 0.f;
      re[u] = PER > 0 ? rn[b * U + u] : (ok ? a.r[e] : 0.f);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t e = threadIdx.x + (int64_t)(b * U + u) * kTail;
      if (e < a.d) {
        a.pdir[e] = fmaf(al, x[u], pe[u]);
        if (!stop) a.dvec[e] = fmaf(be, x[u], re[u]);
      }
    }
  }
  if (threadIdx.x == 0) {
    st->rr = rr_new;
    st->cg_iters += 1;
    if (stop) st->cg_active = 0;
  }
}

// The same update for long vectors (d > 24576), spread over several workgroups in two kernels; the sum
// of the new ||r||^2 passes between them as per-workgroup partials, added in a fixed order.  Flags that
// one kernel reads are never written by the same kernel: the first one reads cg_active and leaves its
// verdict in cg_go, the second one reads cg_go and writes cg_active.
constexpr int kCgThreads = 256;
constexpr int kCgPerThread = 8;
constexpr int kCgChunk = kCgThreads * kCgPerThread;

__global__ __launch_bounds__(kCgThreads) void cg_residual_kernel(const CgUpdateArgs a) {
  __shared__ double sm[17];
  DevState* st = a.st;
  const bool active = st->cg_active != 0;
  const double dq = active ? partial_sum_block(a.dot_part, a.ndot, sm) : 0.0;
  const bool curv = dq > 0.0 && isfinite(dq);
  const double rr = st->rr;
  const float al = curv ? (float)(rr / dq) : 0.f;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st->cg_go = (active && curv) ? 1 : 0;
    st->cg_ok = (!active || curv) ? 1 : 0;
    st->cg_alpha = al;
    st->rr_prev = rr;
  }
  if (!active || !curv) return;
  double acc = 0.0;
  for (int64_t base = (int64_t)blockIdx.x * kCgChunk; base < a.d; base += (int64_t)gridDim.x * kCgChunk) {
    float y[kCgPerThread], re[kCgPerThread];
#pragma unroll
    for (int u = 0; u < kCgPerThread; ++u) {
      const int64_t e = base + threadIdx.x + u * kCgThreads;
      y[u] = e < a.d ? a.q[e] : 0.f;
      re[u] = e < a.d ? a.r[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kCgPerThread; ++u) {
      const int64_t e = base + threadIdx.x + u * kCgThreads;
      const float v = fmaf(-al, y[u], re[u]);
      if (e < a.d) a.r[e] = v;
      acc += (double)v * (double)v;
    }
  }
  acc = block_sum(acc, sm);
  if (threadIdx.x == 0) a.rr_part[blockIdx.x] = acc;
}

__global__ __launch_bounds__(kCgThreads) void cg_direction_kernel(const CgUpdateArgs a) {
  __shared__ double sm[17];
  DevState* st = a.st;
  if (st->cg_go == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0 && st->cg_ok == 0) st->cg_active = 0;  // no positive curvature
    return;
  }
  const float al = st->cg_alpha;
  const double rr = st->rr_prev;
  const double rr_new = partial_sum_block(a.rr_part, (int)gridDim.x, sm);
  const bool stop = sqrt(rr_new) <= (double)a.tol * sqrt(st->gg_cg);
  const float be = (float)(rr_new / rr);
  for (int64_t base = (int64_t)blockIdx.x * kCgChunk; base < a.d; base += (int64_t)gridDim.x * kCgChunk) {
    float x[kCgPerThread], pe[kCgPerThread], re[kCgPerThread];
#pragma unroll
    for (int u = 0; u < kCgPerThread; ++u) {
      const int64_t e = base + threadIdx.x + u * kCgThreads;
      x[u] = e < a.d ? a.dvec[e] : 0.f;
      pe[u] = e < a.d ? a.pdir[e] : 0.f;
      re[u] = e < a.d ? a.r[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kCgPerThread; ++u) {
      const int64_t e = base + threadIdx.x + u * kCgThreads;
      if (e < a.d) {
        a.pdir[e] = fmaf(al, x[u], pe[u]);
        if (!stop) a.dvec[e] = fmaf(be, x[u], re[u]);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st->rr = rr_new;
    st->cg_iters += 1;
    if (stop) st->cg_active = 0;
  }
}

// Small problems: q = s sum_k partial[k] + (lambda + rho) d and the CG update above in one kernel.
// Thread t sums the partials k = g, g + G, ... of element e = t mod d (g = t / d, G = 1024 / d groups),
// the G group sums are added in order.
__global__ __launch_bounds__(kTail) void cg_reduce_update_kernel(const ReduceArgs ra, const CgUpdateArgs a) {
  __shared__ double sm[17];
  __shared__ float gsum[kTail];
  DevState* st = a.st;
  const int d = (int)a.d;
  const int groups = kTail / d;
  const int t = threadIdx.x;
  const int e = t % d, g = t / d;
  // Everything the update reads is requested before the first value is needed (indices clamped, no load under a
  // condition): the scalars of the state, this thread's elements of the vectors, then the partials in runs of 16.
  const int active = st->cg_active;
  const double rr = st->rr;
  const double gg = st->gg_cg;
  const float rho_ = ra.rho_scale != nullptr ? ra.rho * *ra.rho_scale : ra.rho;  // outer solver: common factor on the penalty
  const bool mine = t < d;
  const int tc = mine ? t : d - 1;
  const float dv_in = a.dvec[tc], r_in = a.r[tc], p_in = a.pdir[tc];
  float sum = 0.f;
  {
    constexpr int U = 16;
    const float* __restrict__ pp = ra.partial + e;
    const int gc = g < groups ? g : groups - 1;
    for (int k = gc; k < ra.nparts; k += U * groups) {
      float v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = k + u * groups;
        v[u] = pp[(size_t)(idx < ra.nparts ? idx : ra.nparts - 1) * d];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) sum += (k + u * groups < ra.nparts) ? v[u] : 0.f;  // in the order of the partials
    }
  }
  if (active == 0) return;  // uniform
  gsum[t] = g < groups ? sum : 0.f;
  __syncthreads();
  float dv = 0.f, qv = 0.f;
  if (mine) {
    float s2 = 0.f;
    for (int g2 = 0; g2 < groups; ++g2) s2 += gsum[g2 * d + t];
    dv = dv_in;
    qv = fmaf(ra.lambda + rho_, dv, ra.scale * s2);
  }
  const double dq = block_sum((double)dv * (double)qv, sm);
  if (!(dq > 0.0) || !isfinite(dq)) {  // no positive curvature: keep the current iterate
    __syncthreads();
    if (t == 0) st->cg_active = 0;
    return;
  }
  const float al = (float)(rr / dq);
  const float rn = mine ? fmaf(-al, qv, r_in) : 0.f;
  const double rr_new = block_sum((double)rn * (double)rn, sm);
  const bool stop = sqrt(rr_new) <= (double)a.tol * sqrt(gg);
  const float be = (float)(rr_new / rr);
  if (mine) {
    a.r[t] = rn;
    a.pdir[t] = fmaf(al, dv, p_in);
    if (!stop) a.dvec[t] = fmaf(be, dv, rn);
  }
  if (t == 0) {
    st->rr = rr_new;
    st->cg_iters += 1;
    if (stop) st->cg_active = 0;
  }
}

// The pending update of a deferred CG iteration alone (end of a stand-alone CG solve); the iterate is formed in p_final.
constexpr int kPendThreads = 512;
constexpr int kPendPer = 8;   // quads per thread: the fused single-pass path has p (C-1) <= 960 * 16 <= 4 * 512 * 8
__global__ __launch_bounds__(kPendThreads) void cg_pending_finish_kernel(const CgPend c) {
  __shared__ double sm[kPendThreads / 64 + 1];
  cg_pending_update<kPendThreads, kPendPer>(c, true, c.p_final, sm, [] {});
}

__global__ __launch_bounds__(256) void cg_finish_kernel(const CgFinishArgs a) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < a.d; e += (int64_t)gridDim.x * blockDim.x)
    a.p_out[e] = a.pdir[e];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (a.iters_out) *a.iters_out = a.st->cg_iters;
    if (a.relres_out) *a.relres_out = a.st->gg_cg > 0.0 ? (float)sqrt(a.st->rr / a.st->gg_cg) : 0.f;
  }
}

// A p of one element of the cached-logit arrays from the directional logits of the CG iterations taken (LsEvalArgs).
__device__ __forceinline__ float zp_from_history(const LsEvalArgs& a, int nused, const float* al, size_t e) {
  float v = 0.f;
  for (int k = 0; k < nused; ++k) v = fmaf(al[k], a.hist[(size_t)k * a.hist_stride + e], v);
  return v;
}

// Row losses at Z = Zx + alpha Zp for all candidate step sizes (Sections 2.1, 2.2).  One thread per (row, candidate):
// a workgroup is 16 rows x 16 candidate slots, the 16 threads of a row read the same cached logits (one broadcast
// load per wave and address), and a row costs a thread one log-sum-exp instead of one per candidate, so that a compute
// unit holds many short threads instead of a few long ones.  More than 16 candidates take further passes.
// NK = 0: A p is given.  NK > 0: A p comes from up to NK history buffers (LsEvalArgs).  The 4 rows of a wave are 4 (C-1)
// consecutive elements of every buffer: lane l takes element l through all buffers (NK coalesced loads, each a line or
// two), and the threads of a row then fetch the C-1 sums of their row from those lanes.
// No load sits under a condition (indices are clamped instead: padded classes read class C-2 again, rows past the end
// the last row, buffers past the last one the last one), so that all of a row's loads are in flight together.
template <int NCP, int NK>
__global__ __launch_bounds__(256) void ls_eval_kernel(const LsEvalArgs a) {
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ double sm[4][16];
  const int NC = a.NC;
  const int slot = threadIdx.x & 15, rloc = threadIdx.x >> 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // With the last CG update still pending, workgroup 0 applies it (iterate, final scalars) while the others evaluate;
  // they take its step length from the same partial sums by the same arithmetic.
  const int role0 = (NK > 0 && a.has_pend != 0) ? 1 : 0;
  const int wg = blockIdx.x - role0, nwg = gridDim.x - role0;
  float hal[NK > 0 ? NK : 1];
  if (NK > 0) {
    __shared__ double smd[256 / 64 + 1];
    if (role0 != 0 && blockIdx.x == 0) {
      cg_pending_final_walk<256>(a.pend, smd);
      return;
    }
    int nprev = a.st->cg_iters;
    float al_last = 0.f;
    if (role0 != 0) {
      const CgPendScalars ps = cg_pending_scalars<256>(a.pend, smd);
      nprev = ps.in.iters;
      al_last = ps.al;  // 0 if the update does not take place
    }
    nprev = nprev < a.nbuf ? nprev : a.nbuf;
#pragma unroll
    for (int k = 0; k < NK; ++k)  // uniform
      hal[k] = k < nprev ? a.st->cg_alphas[k < kCgHist ? k : kCgHist - 1] : ((k == nprev && k < a.nbuf) ? al_last : 0.f);
  }
  const int64_t last = a.n * NC - 1;
  for (int k0 = 0; k0 < a.ncand; k0 += 16) {
    const bool live = k0 + slot < a.ncand;
    const float al = live ? a.alphas[k0 + slot] : 0.f;
    double acc = 0.0;
    for (int64_t g = (int64_t)wg * 16; g < a.n; g += (int64_t)nwg * 16) {  // the same trips for every thread
      const int64_t i = g + rloc;
      const bool valid = i < a.n;
      const size_t ro = (size_t)(valid ? i : a.n - 1) * NC;
      const int b = a.labels[valid ? i : a.n - 1];
      float zx[NCP], zp[NCP], h[NK > 0 ? NK : 1];
      if (NK > 0) {
        const int64_t e = (g + 4 * wave) * NC + lane;  // lanes past the 4 rows read on into the next rows: never used
        const float* src = a.hist + (e < last ? e : last);
#pragma unroll
        for (int k = 0; k < NK; ++k) h[k] = src[(size_t)(k < a.nbuf ? k : a.nbuf - 1) * a.hist_stride];
      }
#pragma unroll
      for (int c = 0; c < NCP; ++c) {
        const size_t e = ro + (c < NC ? c : NC - 1);
        zx[c] = a.Zx[e];
        if (NK == 0) zp[c] = a.Zp[e];
      }
      if (NK > 0) {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < NK; ++k) sum = hal[k] != 0.f ? fmaf(hal[k], h[k], sum) : sum;  // unused buffers hold anything
#pragma unroll
        for (int c = 0; c < NCP; ++c) {
          const int from = (rloc & 3) * NC + (c < NC ? c : NC - 1);  // < 4 (C-1) <= 64
          zp[c] = __int_as_float(__builtin_amdgcn_ds_bpermute(from << 2, __float_as_int(sum)));
        }
      }
      float zz[NCP];
      float M = 0.f, zb = 0.f;
#pragma unroll
      for (int c = 0; c < NCP; ++c) {
        zz[c] = fmaf(al, zp[c], zx[c]);
        M = c < NC ? fmaxf(M, zz[c]) : M;
        zb = (c < NC && c == b) ? zz[c] : zb;   // the reference class (label C-1) has logit 0
      }
      float alpha = expf(-M);
#pragma unroll
      for (int c = 0; c < NCP; ++c) alpha += c < NC ? expf(zz[c] - M) : 0.f;
      if (valid) acc += (double)M + (double)logf(alpha) - (double)zb;
    }
    // rows of this workgroup, in a fixed order: the 4 row lanes of a wave, then the 4 waves
    acc += __shfl_xor(acc, 16, 64);
    acc += __shfl_xor(acc, 32, 64);
    __syncthreads();  // the previous pass has read sm
    if (lane < 16) sm[wave][lane] = acc;
    __syncthreads();
    if (threadIdx.x < 16 && live)
      a.lpart[(size_t)(k0 + slot) * nwg + wg] = (sm[0][slot] + sm[1][slot]) + (sm[2][slot] + sm[3][slot]);
  }
}

// The same with one thread per row and all candidates in a loop (the cached logits are read once per 16 candidates):
// for many rows (n > kLsRowsPerThreadFrom) there are threads enough, and a thread per row reads the logits coalesced.
template <int NCP>
__global__ __launch_bounds__(256) void ls_eval_rows_kernel(const LsEvalArgs a) {
  if (a.flag != nullptr && *a.flag == 0) return;
  constexpr int G = 16;  // candidates per pass over the cached logits (the usual 12 take one pass)
  __shared__ double smk[G][4];
  __shared__ float cgal[kCgHist];
  const int NC = a.NC;
  const int64_t stride = (int64_t)gridDim.x * 256;
  const bool from_hist = a.Zp == nullptr;
  int nused = 0;
  if (from_hist) {
    nused = a.st->cg_iters < kCgHist ? a.st->cg_iters : kCgHist;
    if (threadIdx.x < kCgHist) cgal[threadIdx.x] = threadIdx.x < nused ? a.st->cg_alphas[threadIdx.x] : 0.f;
    __syncthreads();
  }
  for (int k0 = 0; k0 < a.ncand; k0 += G) {
    float al[G];
#pragma unroll
    for (int kk = 0; kk < G; ++kk) al[kk] = (k0 + kk < a.ncand) ? a.alphas[k0 + kk] : 0.f;
    double acc[G];
#pragma unroll
    for (int kk = 0; kk < G; ++kk) acc[kk] = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < a.n; i += stride) {
      float zx[NCP], zp[NCP];
      const size_t ro = (size_t)i * NC;
#pragma unroll
      for (int c = 0; c < NCP; ++c) {
        const size_t e = ro + (c < NC ? c : NC - 1);  // no load under a condition: padded classes read class C-2 again
        zx[c] = a.Zx[e];
        zp[c] = from_hist ? zp_from_history(a, nused, cgal, e) : a.Zp[e];
      }
      const int b = a.labels[i];
#pragma unroll
      for (int kk = 0; kk < G; ++kk) {
        if (k0 + kk < a.ncand) {  // uniform
          float M = 0.f, zb = 0.f;
          float zz[NCP];
#pragma unroll
          for (int c = 0; c < NCP; ++c) {
            zz[c] = fmaf(al[kk], zp[c], zx[c]);
            if (c < NC) {
              M = fmaxf(M, zz[c]);
              if (c == b) zb = zz[c];
            }
          }
          float alpha;
          if constexpr (NCP == 1) {
            // two classes: one of exp(-M) and exp(z - M) is exp(0), the other exp(-|z|): the same sum with one exponential
            alpha = 1.f + expf(-fabsf(zz[0]));
          } else {
            alpha = expf(-M);
#pragma unroll
            for (int c = 0; c < NCP; ++c)
              if (c < NC) alpha += expf(zz[c] - M);
          }
          acc[kk] += (double)M + (double)logf(alpha) - (double)zb;
        }
      }
    }
    // the candidates' sums over the workgroup share one pair of barriers: per wave first, then the four waves in order
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int kk = 0; kk < G; ++kk) {
      const double t = wave_sum(acc[kk]);
      if (lane == 0) smk[kk][wave] = t;
    }
    __syncthreads();
    if (threadIdx.x < G && k0 + (int)threadIdx.x < a.ncand) {
      const int kk = threadIdx.x;
      a.lpart[(size_t)(k0 + kk) * gridDim.x + blockIdx.x] = ((smk[kk][0] + smk[kk][1]) + smk[kk][2]) + smk[kk][3];
    }
    __syncthreads();  // the next pass writes smk again
  }
}

// Long vectors (d > kWideFrom): the sums over d that the line search needs, per workgroup, and the update
// X += alpha p as kernels of their own around the single-workgroup decision kernel below.
// qpart: [4][nq] partial sums of the penalty coefficients q0, q1, q2 and of the slope <p, g>.
__global__ __launch_bounds__(256) void ls_vec_part_kernel(const LsTailArgs a, int nq) {
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ double sm[17];
  double q0 = 0.0, q1 = 0.0, q2 = 0.0, sl = 0.0;
  const double inv_rho = 1.0 / (double)rho_;
  for (int64_t base = (int64_t)blockIdx.x * kWideChunk + threadIdx.x; base < a.d; base += (int64_t)gridDim.x * kWideChunk) {
    float xv[kWidePer], zv[kWidePer], yv[kWidePer], pvv[kWidePer], gv[kWidePer];
#pragma unroll
    for (int u = 0; u < kWidePer; ++u) {
      const int64_t e = base + u * 256;
      const bool ok = e < a.d;
      xv[u] = ok ? a.X[e] : 0.f;
      zv[u] = (ok && a.z) ? a.z[e] : 0.f;
      yv[u] = (ok && a.y) ? a.y[e] : 0.f;
      pvv[u] = ok ? a.pdir[e] : 0.f;
      gv[u] = ok ? a.g[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kWidePer; ++u) {  // the padding (all zero) adds nothing
      const double x = xv[u];
      const double uu = x - (double)zv[u] + (double)yv[u] * inv_rho;
      const double pv = pvv[u];
      q0 += 0.5 * (double)a.lambda * x * x + 0.5 * (double)rho_ * uu * uu;
      q1 += (double)a.lambda * x * pv + (double)rho_ * uu * pv;
      q2 += 0.5 * ((double)a.lambda + (double)rho_) * pv * pv;
      sl += pv * (double)gv[u];
    }
  }
  q0 = block_sum(q0, sm);
  q1 = block_sum(q1, sm);
  q2 = block_sum(q2, sm);
  sl = block_sum(sl, sm);
  if (threadIdx.x == 0) {
    a.qpart[blockIdx.x] = q0;
    a.qpart[nq + blockIdx.x] = q1;
    a.qpart[2 * nq + blockIdx.x] = q2;
    a.qpart[3 * nq + blockIdx.x] = sl;
  }
}

__global__ __launch_bounds__(256) void ls_apply_kernel(const DevState* st, const float* __restrict__ pdir,
                                                       float* __restrict__ X, int64_t d, const int32_t* flag) {
  if (flag != nullptr && *flag == 0) return;
  const float alpha = st->alpha;
  for (int64_t base = (int64_t)blockIdx.x * kWideChunk + threadIdx.x; base < d; base += (int64_t)gridDim.x * kWideChunk) {
    float pv[kWidePer], xv[kWidePer];
#pragma unroll
    for (int u = 0; u < kWidePer; ++u) {
      const int64_t e = base + u * 256;
      pv[u] = e < d ? pdir[e] : 0.f;
      xv[u] = e < d ? X[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kWidePer; ++u) {
      const int64_t e = base + u * 256;
      if (e < d) X[e] = fmaf(alpha, pv[u], xv[u]);
    }
  }
}

// Algorithm 2 on the candidate objective values; optionally applies X += alpha p.  nq > 0: the sums
// over d come as partial sums from ls_vec_part_kernel and X is updated by ls_apply_kernel.
__global__ __launch_bounds__(kTail) void ls_tail_kernel(const LsTailArgs a, int nq) {
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  __shared__ double sm[17];
  __shared__ double cand[kCandSlots];
  __shared__ float s_alpha;
  DevState* st = a.st;
  if (a.flag != nullptr && *a.flag == 0) return;

  const int nslots = a.ncand + (a.zero_slot >= 0 ? 1 : 0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int k = wave; k < nslots; k += kTail / 64) {
    double acc = 0.0;
    for (int b0 = lane; b0 < a.nblocks; b0 += 64 * kBlk) {
      double v[kBlk];
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        const int b = b0 + 64 * u;
        v[u] = b < a.nblocks ? a.lpart[(size_t)k * a.nblocks + b] : 0.0;
      }
#pragma unroll
      for (int u = 0; u < kBlk; ++u) acc += v[u];
    }
    acc = wave_sum(acc);
    if (lane == 0) cand[k] = acc;
  }
  // penalty along the line: q0 + alpha q1 + alpha^2 q2, and the slope <p, g>
  double q0 = 0.0, q1 = 0.0, q2 = 0.0, sl = 0.0;
  const double inv_rho = 1.0 / (double)rho_;
  for (int64_t e0 = threadIdx.x; nq == 0 && e0 < a.d; e0 += (int64_t)kBlk * blockDim.x) {
    float xv[kBlk], zv[kBlk], yv[kBlk], pvv[kBlk], gv[kBlk];
#pragma unroll
    for (int u = 0; u < kBlk; ++u) {
      const int64_t e = e0 + (int64_t)u * blockDim.x;
      const bool ok = e < a.d;
      xv[u] = ok ? a.X[e] : 0.f;
      zv[u] = (ok && a.z) ? a.z[e] : 0.f;
      yv[u] = (ok && a.y) ? a.y[e] : 0.f;
      pvv[u] = ok ? a.pdir[e] : 0.f;
      gv[u] = ok ? a.g[e] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kBlk; ++u) {  // the padding (all zero) adds nothing
      const double x = xv[u];
      const double uu = x - (double)zv[u] + (double)yv[u] * inv_rho;
      const double pv = pvv[u];
      q0 += 0.5 * (double)a.lambda * x * x + 0.5 * (double)rho_ * uu * uu;
      q1 += (double)a.lambda * x * pv + (double)rho_ * uu * pv;
      q2 += 0.5 * ((double)a.lambda + (double)rho_) * pv * pv;
      sl += pv * (double)gv[u];
    }
  }
  if (nq > 0) {
    q0 = partial_sum_block(a.qpart, nq, sm);
    q1 = partial_sum_block(a.qpart + nq, nq, sm);
    q2 = partial_sum_block(a.qpart + 2 * nq, nq, sm);
    sl = partial_sum_block(a.qpart + 3 * nq, nq, sm);
  } else {
    q0 = block_sum(q0, sm);
    q1 = block_sum(q1, sm);
    q2 = block_sum(q2, sm);
    sl = block_sum(sl, sm);
  }

  if (threadIdx.x == 0) {
    double f0;
    if (a.zero_slot >= 0) f0 = (double)a.scale * cand[a.zero_slot] + q0;
    else if (a.use_state_loss) f0 = st->loss;
    else f0 = a.loss_at_X;
    int k = 0, ok = 1;
    double fk = 0.0;
    for (;;) {
      const double al = (double)a.alphas[k];
      fk = (double)a.scale * cand[k] + q0 + al * q1 + al * al * q2;
      if (!(fk > f0 + al * (double)a.beta * sl)) break;       // Armijo holds (eq. armijo)
      if (k + 1 >= a.ncand) { ok = 0; break; }                 // the i > i_max break of Algorithm 2
      ++k;
    }
    const float alpha = a.alphas[k];
    s_alpha = alpha;
    st->alpha = alpha;
    st->loss_new = fk;
    st->armijo_ok = ok;
    st->ls_evals = k + 1;
    if (a.alpha_out) *a.alpha_out = alpha;
    if (a.loss_new_out) *a.loss_new_out = fk;
    if (a.ok_out) *a.ok_out = ok;
    if (a.iter >= 0) {
      nadmm_stats* s = &st->stats;
      s->newton_iters += 1;
      s->cg_iters_total += st->cg_iters;
      s->ls_evals_total += k + 1;
      s->armijo_failed += ok ? 0 : 1;
      s->loss_final = fk;
      if (a.iter < NADMM_TRACE_LEN) { s->alpha[a.iter] = alpha; s->cg_iters[a.iter] = st->cg_iters; }
    }
  }
  __syncthreads();
  if (a.X_apply != nullptr && nq == 0) {
    const float alpha = s_alpha;
    for (int64_t e0 = threadIdx.x; e0 < a.d; e0 += (int64_t)kBlk * blockDim.x) {
      float pvv[kBlk], xv[kBlk];
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        const int64_t e = e0 + (int64_t)u * blockDim.x;
        pvv[u] = e < a.d ? a.pdir[e] : 0.f;
        xv[u] = e < a.d ? a.X_apply[e] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        const int64_t e = e0 + (int64_t)u * blockDim.x;
        if (e < a.d) a.X_apply[e] = fmaf(alpha, pvv[u], xv[u]);
      }
    }
  }
}

// The same for short vectors (d <= PER * 1024, at most 1024 partial sums per candidate): every load of the kernel is
// issued before anything is used, so that it costs one memory round trip instead of one per stage, and the four sums
// over d share their barriers.  X_apply, if given, is X itself.
template <int PER>
__global__ __launch_bounds__(kTail) void ls_tail_fast_kernel(const LsTailArgs a) {
  const float rho_ = a.rho_scale != nullptr ? a.rho * *a.rho_scale : a.rho;  // outer solver: common factor on the penalty
  __shared__ double sm4[4][kTail / 64];
  __shared__ double cand[kCandSlots];
  __shared__ float s_alpha;
  DevState* st = a.st;
  if (a.flag != nullptr && *a.flag == 0) return;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int nslots = a.ncand + (a.zero_slot >= 0 ? 1 : 0);
  const int d = (int)a.d;
  // ---- loads ----
  const float* zsrc = a.z ? a.z : a.X;  // a missing z or y reads X instead and is then set to zero (no branch around loads)
  const float* ysrc = a.y ? a.y : a.X;
  float xv[PER], zv[PER], yv[PER], pv[PER], gv[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int e = t + u * kTail;
    const int ec = e < d ? e : d - 1;
    xv[u] = a.X[ec];
    zv[u] = zsrc[ec];
    yv[u] = ysrc[ec];
    pv[u] = a.pdir[ec];
    gv[u] = a.g[ec];
  }
  constexpr int kLp = 1024 / 64;  // partial sums per lane and candidate
  double lp[kLp];
  {
    const int k = wave < nslots ? wave : nslots - 1;
#pragma unroll
    for (int j = 0; j < kLp; ++j) {
      const int b = lane + 64 * j;
      lp[j] = a.lpart[(size_t)k * a.nblocks + (b < a.nblocks ? b : a.nblocks - 1)];
    }
  }
  // ---- candidate sums: wave w takes candidates w, w + 16, ... ----
  for (int k = wave; k < nslots; k += kTail / 64) {
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < kLp; ++j) {
      const int b = lane + 64 * j;
      double v = lp[j];
      if (k != wave) v = a.lpart[(size_t)k * a.nblocks + (b < a.nblocks ? b : a.nblocks - 1)];  // uniform: beyond 16 candidates
      acc += b < a.nblocks ? v : 0.0;
    }
    acc = wave_sum(acc);
    if (lane == 0) cand[k] = acc;
  }
  // ---- penalty along the line: q0 + alpha q1 + alpha^2 q2, and the slope <p, g> ----
  double q0 = 0.0, q1 = 0.0, q2 = 0.0, sl = 0.0;
  const double inv_rho = 1.0 / (double)rho_;
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    if (t + u * kTail < d) {
      const double x = xv[u];
      const double uu = x - (a.z ? (double)zv[u] : 0.0) + (a.y ? (double)yv[u] : 0.0) * inv_rho;
      const double pvd = pv[u];
      q0 += 0.5 * (double)a.lambda * x * x + 0.5 * (double)rho_ * uu * uu;
      q1 += (double)a.lambda * x * pvd + (double)rho_ * uu * pvd;
      q2 += 0.5 * ((double)a.lambda + (double)rho_) * pvd * pvd;
      sl += pvd * (double)gv[u];
    }
  }
  q0 = wave_sum(q0); q1 = wave_sum(q1); q2 = wave_sum(q2); sl = wave_sum(sl);
  if (lane == 0) { sm4[0][wave] = q0; sm4[1][wave] = q1; sm4[2][wave] = q2; sm4[3][wave] = sl; }
  __syncthreads();  // also publishes cand[]
  if (t == 0) {
    q0 = q1 = q2 = sl = 0.0;
    for (int w = 0; w < kTail / 64; ++w) { q0 += sm4[0][w]; q1 += sm4[1][w]; q2 += sm4[2][w]; sl += sm4[3][w]; }
    double f0;
    if (a.zero_slot >= 0) f0 = (double)a.scale * cand[a.zero_slot] + q0;
    else if (a.use_state_loss) f0 = st->loss;
    else f0 = a.loss_at_X;
    int k = 0, ok = 1;
    double fk = 0.0;
    for (;;) {
      const double al = (double)a.alphas[k];
      fk = (double)a.scale * cand[k] + q0 + al * q1 + al * al * q2;
      if (!(fk > f0 + al * (double)a.beta * sl)) break;       // Armijo holds (eq. armijo)
      if (k + 1 >= a.ncand) { ok = 0; break; }                 // the i > i_max break of Algorithm 2
      ++k;
    }
    const float alpha = a.alphas[k];
    s_alpha = alpha;
    st->alpha = alpha;
    st->loss_new = fk;
    st->armijo_ok = ok;
    st->ls_evals = k + 1;
    if (a.alpha_out) *a.alpha_out = alpha;
    if (a.loss_new_out) *a.loss_new_out = fk;
    if (a.ok_out) *a.ok_out = ok;
    if (a.iter >= 0) {
      nadmm_stats* s = &st->stats;
      s->newton_iters += 1;
      s->cg_iters_total += st->cg_iters;
      s->ls_evals_total += k + 1;
      s->armijo_failed += ok ? 0 : 1;
      s->loss_final = fk;
      if (a.iter < NADMM_TRACE_LEN) { s->alpha[a.iter] = alpha; s->cg_iters[a.iter] = st->cg_iters; }
    }
  }
  __syncthreads();
  if (a.X_apply != nullptr) {
    const float alpha = s_alpha;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = t + u * kTail;
      if (e < d) a.X_apply[e] = fmaf(alpha, pv[u], xv[u]);
    }
  }
}

template <typename F>
hipError_t dispatch_ncp(int NC, F&& f) {
  if (NC <= 1) return f(std::integral_constant<int, 1>());
  if (NC <= 2) return f(std::integral_constant<int, 2>());
  if (NC <= 4) return f(std::integral_constant<int, 4>());
  if (NC <= 9) return f(std::integral_constant<int, 9>());
  if (NC <= 16) return f(std::integral_constant<int, 16>());
  if (NC <= 19) return f(std::integral_constant<int, 19>());
  return f(std::integral_constant<int, 32>());
}

}  // namespace

int reduce_out_blocks(int64_t d) {
  return d > kWideFrom ? (int)((d + kWideChunk - 1) / kWideChunk) : (int)((d + 31) / 32);
}

hipError_t launch_reduce_out(const ReduceArgs& a, hipStream_t st) {
  const int blocks = reduce_out_blocks(a.d);
  if (a.lf_loss_out != nullptr && (a.kind != 1 || a.d > kReduceFinishMax || a.lf_loss_part == nullptr || a.lf_nblocks < 1))
    return hipErrorInvalidValue;
  if (a.has_head != 0 && (a.kind != 0 || a.d > kReduceFinishMax || a.lf_loss_out != nullptr || a.head.st == nullptr ||
                          a.head.gg_part == nullptr || a.head.pen_part == nullptr))
    return hipErrorInvalidValue;
  if (a.d > kWideFrom) hipLaunchKernelGGL(reduce_out_wide_kernel, dim3(blocks), dim3(256), 0, st, a);
  else if (a.lf_loss_out != nullptr || a.has_head != 0) hipLaunchKernelGGL(reduce_out_kernel<true>, dim3(blocks + 1), dim3(256), 0, st, a);
  else hipLaunchKernelGGL(reduce_out_kernel<false>, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_loss_finish(const LossFinishArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(kTail), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_state_init(DevState* s, const int32_t* outer_flag, hipStream_t st) {
  hipLaunchKernelGGL(state_init_kernel, dim3(1), dim3(64), 0, st, s, outer_flag);
  return hipGetLastError();
}

hipError_t launch_newton_head(const NewtonHeadArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(newton_head_kernel, dim3(1), dim3(kTail), 0, st, a);
  return hipGetLastError();
}

int cg_update_blocks(int64_t d) {
  int64_t b = (d + kCgChunk - 1) / kCgChunk;
  return (int)(b < 1024 ? b : 1024);
}

hipError_t launch_cg_update(const CgUpdateArgs& a, hipStream_t st) {
  if (a.d <= 8 * kTail) {
    hipLaunchKernelGGL(cg_update_kernel<8>, dim3(1), dim3(kTail), 0, st, a);
  } else if (a.d <= 24 * kTail) {
    hipLaunchKernelGGL(cg_update_kernel<24>, dim3(1), dim3(kTail), 0, st, a);
  } else {
    const int blocks = cg_update_blocks(a.d);
    hipLaunchKernelGGL(cg_residual_kernel, dim3(blocks), dim3(kCgThreads), 0, st, a);
    hipLaunchKernelGGL(cg_direction_kernel, dim3(blocks), dim3(kCgThreads), 0, st, a);
  }
  return hipGetLastError();
}

bool cg_fused_tail_supported(int64_t d, int nparts) {
  if (d < 1 || d > kTail) return false;
  const int groups = kTail / (int)d;
  return (nparts + groups - 1) / groups <= 64;
}

hipError_t launch_cg_reduce_update(const ReduceArgs& r, const CgUpdateArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(cg_reduce_update_kernel, dim3(1), dim3(kTail), 0, st, r, a);
  return hipGetLastError();
}

hipError_t launch_cg_pending_finish(const CgPend& c, hipStream_t st) {
  if (c.st == nullptr || c.final_p == 0 || c.dlen > (int64_t)4 * kPendThreads * kPendPer || c.ndot > kPendThreads || c.ndot < 1)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(cg_pending_finish_kernel, dim3(1), dim3(kPendThreads), 0, st, c);
  return hipGetLastError();
}

hipError_t launch_cg_finish(const CgFinishArgs& a, hipStream_t st) {
  int blocks = (int)((a.d + 255) / 256);
  if (blocks > 256) blocks = 256;
  hipLaunchKernelGGL(cg_finish_kernel, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

constexpr int64_t kLsRowsPerThreadFrom = (int64_t)1 << 17;

// Whether the line-search row kernel for n rows can apply a pending last CG update itself (LsEvalArgs.has_pend).
bool ls_eval_takes_pending(int64_t n) { return n <= kLsRowsPerThreadFrom; }

int ls_eval_blocks(int64_t n) {
  // up to 2^17 rows: 16 rows x 16 candidate slots per workgroup and pass; beyond: 256 rows per workgroup and pass
  int64_t b = n <= kLsRowsPerThreadFrom ? (n + 15) / 16 : (n + 255) / 256;
  if (b > 1024) b = 1024;
  if (b < 1) b = 1;
  return (int)b;
}

hipError_t launch_ls_eval(const LsEvalArgs& a, hipStream_t st) {
  const int blocks = ls_eval_blocks(a.n);
  return dispatch_ncp(a.NC, [&](auto ncp) {
    constexpr int NCP = decltype(ncp)::value;
    if (a.Zp == nullptr && (a.hist == nullptr || a.st == nullptr || a.nbuf < 1 || a.nbuf > kCgHist)) return hipErrorInvalidValue;
    if (a.has_pend != 0 && (!ls_eval_takes_pending(a.n) || a.Zp != nullptr || a.pend.st == nullptr || a.pend.final_p == 0 ||
                            a.pend.ndot < 1 || a.pend.dlen < 1))
      return hipErrorInvalidValue;
    if (a.n > kLsRowsPerThreadFrom) {
      hipLaunchKernelGGL(ls_eval_rows_kernel<NCP>, dim3(blocks), dim3(256), 0, st, a);
    } else if (a.Zp != nullptr) {
      hipLaunchKernelGGL((ls_eval_kernel<NCP, 0>), dim3(blocks), dim3(256), 0, st, a);
    } else if constexpr (NCP <= 16) {  // 4 rows of a wave are at most 64 elements
      const dim3 grid(blocks + (a.has_pend != 0 ? 1 : 0));
      if (a.nbuf <= 8) hipLaunchKernelGGL((ls_eval_kernel<NCP, 8>), grid, dim3(256), 0, st, a);
      else if (a.nbuf <= 12) hipLaunchKernelGGL((ls_eval_kernel<NCP, 12>), grid, dim3(256), 0, st, a);
      else if (a.nbuf <= 16) hipLaunchKernelGGL((ls_eval_kernel<NCP, 16>), grid, dim3(256), 0, st, a);
      else hipLaunchKernelGGL((ls_eval_kernel<NCP, kCgHist>), grid, dim3(256), 0, st, a);
    } else {
      return hipErrorInvalidValue;
    }
    return hipGetLastError();
  });
}

// Workgroups that form the sums over d of the line-search tail: none up to 8192 elements (one workgroup does everything,
// ls_tail_fast_kernel), else one per 2048 elements, at most 256.  4 sums per workgroup fit the 2 reduce_out_blocks(d)
// doubles of the dot-product partials in every case.
int ls_tail_parts(int64_t d) {
  if (d <= 8 * kTail) return 0;
  int64_t b = d > kWideFrom ? reduce_out_blocks(d) / 2 : (d + kWideChunk - 1) / kWideChunk;
  if (b > 256) b = 256;
  return (int)(b < 1 ? 1 : b);
}

hipError_t launch_ls_tail(const LsTailArgs& a, hipStream_t st) {
  const int nq = a.qpart != nullptr ? ls_tail_parts(a.d) : 0;
  if (nq == 0 && a.d <= 8 * kTail && a.nblocks >= 1 && a.nblocks <= 1024 && (a.X_apply == nullptr || a.X_apply == a.X)) {
    hipLaunchKernelGGL(ls_tail_fast_kernel<8>, dim3(1), dim3(kTail), 0, st, a);
    return hipGetLastError();
  }
  if (nq > 0) hipLaunchKernelGGL(ls_vec_part_kernel, dim3(nq), dim3(256), 0, st, a, nq);
  hipLaunchKernelGGL(ls_tail_kernel, dim3(1), dim3(kTail), 0, st, a, nq);
  if (nq > 0 && a.X_apply != nullptr)
    hipLaunchKernelGGL(ls_apply_kernel, dim3(nq), dim3(256), 0, st, (const DevState*)a.st, a.pdir, a.X_apply, a.d, a.flag);
  return hipGetLastError();
}

}  // namespace nadmm
