// One CG update (Section 2.4) applied cooperatively by a whole workgroup, for kernels that consume its result
// (see CgPend): a = rr / <d, q>; r' = r - a q; stop on ||r'|| <= tol ||g|| (eq. inexact); p' = p + a d;
// d' = r' + (rr'/rr) d.  float32 vectors, float64 inner products summed in a fixed order.
#pragma once

#include "nadmm_internal.h"
#include "nadmm_mfma.h"

namespace nadmm {

// Barrier that orders the LDS operations of the workgroup only.  __syncthreads() would also wait for every
// outstanding global memory operation once a global store is pending, i.e. for the caller's first tile.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int THREADS>
__device__ __forceinline__ double cg_block_sum(double v, double* sm /* THREADS / 64 + 1 doubles */) {
  v = mfma_detail::wave64_sum(v);  // rotations inside rows of 16 lanes, the four row totals in a fixed order
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  lds_barrier();  // previous users of sm are done
  if (lane == 0) sm[wave] = v;
  lds_barrier();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) t += sm[w];
  return t;
}

// Leaves the vector the caller wants (d', or p' if c.final_p) in vec[0 .. dlen) (LDS or global, 16-byte aligned;
// complete and visible to the whole workgroup on return).  Returns false if the caller wants d and CG is, or has
// just become, inactive: there is no product left to form.  dlen <= 4 THREADS * PERQ, ndot <= THREADS, the vectors
// of CgPend 16-byte aligned.  `sm`: THREADS / 64 + 1 doubles of LDS.
// `writer`: this workgroup stores the new vectors and the new state (workgroup 0 of the kernel).
// Every load the update needs is issued up front into registers, as few 16-byte loads per thread, then
// `after_issue()` runs (the caller starts its own first loads there, in flight right behind the vectors: loads
// return in order and a wave holds 63 of them at most), then the arithmetic follows: the update costs one memory
// round trip and hides behind the caller's first tile.
template <int THREADS, int PERQ, typename F>
__device__ __forceinline__ bool cg_pending_update(const CgPend& c, bool writer, float* vec, double* sm, F&& after_issue) {
  DevState* st = c.st;
  const CgSlot in = st->cgs[c.slot_in];
  const double gg = st->gg_cg;
  CgSlot out = in;
  const int cur = in.cur & 1;
  const int n = (int)c.dlen;
  const int n4 = n >> 2;                 // whole quads
  const int t = threadIdx.x;
  const float* __restrict__ r_in = cur ? c.r[1] : c.r[0];
  const float* __restrict__ d_in = cur ? c.d[1] : c.d[0];
  const float* __restrict__ p_in = cur ? c.p[1] : c.p[0];

  // one partial sum of <d, q> per thread, fetched without a branch like everything else
  const double dqv = c.dot_part[t < c.ndot ? t : c.ndot - 1];
  double dq = t < c.ndot ? dqv : 0.0;
  // quads t, t + THREADS, ... of every vector and one element of the tail of dlen % 4 elements.  No branches at
  // all (a branch that assigns these registers on both sides makes the compiler wait for the loads at the join,
  // before the caller's tile has been requested): indices past the end are clamped, the surplus loads hit the
  // cache line of the last quad.  The vectors are workspace buffers padded to 256 bytes, so quad 0 is readable
  // even if dlen < 4.
  float4 qv[PERQ], rv[PERQ], dv[PERQ], pv[PERQ];
#pragma unroll
  for (int u = 0; u < PERQ; ++u) {
    const int k = t + u * THREADS;
    const int kc = k < n4 ? k : (n4 > 0 ? n4 - 1 : 0);
    qv[u] = reinterpret_cast<const float4*>(c.q)[kc];
    rv[u] = reinterpret_cast<const float4*>(r_in)[kc];
    dv[u] = reinterpret_cast<const float4*>(d_in)[kc];
    pv[u] = reinterpret_cast<const float4*>(p_in)[kc];
  }
  const int te = 4 * n4 + (t & 3);       // tail element of threads 0 .. dlen % 4 - 1
  const bool tail = t < (n & 3);
  const int tec = te < n ? te : n - 1;
  float tq = c.q[tec], tr = r_in[tec], td = d_in[tec], tp = p_in[tec];
  // keep the order of issue
  __builtin_amdgcn_sched_barrier(0);
  after_issue();
  __builtin_amdgcn_sched_barrier(0);

  bool updated = false;
  float al = 0.f, be = 0.f;
  if (in.active != 0) {  // uniform
    dq = cg_block_sum<THREADS>(dq, sm);
    if (!(dq > 0.0) || !isfinite(dq)) {  // no positive curvature: keep the current iterate
      out.active = 0;
    } else {
      al = (float)(in.rr / dq);
      double acc = 0.0;
#pragma unroll
      for (int u = 0; u < PERQ; ++u) {
        rv[u].x = fmaf(-al, qv[u].x, rv[u].x);
        rv[u].y = fmaf(-al, qv[u].y, rv[u].y);
        rv[u].z = fmaf(-al, qv[u].z, rv[u].z);
        rv[u].w = fmaf(-al, qv[u].w, rv[u].w);
        if (t + u * THREADS < n4)
          acc += ((double)rv[u].x * (double)rv[u].x + (double)rv[u].y * (double)rv[u].y) +
                 ((double)rv[u].z * (double)rv[u].z + (double)rv[u].w * (double)rv[u].w);
      }
      tr = fmaf(-al, tq, tr);
      if (tail) acc += (double)tr * (double)tr;
      const double rr_new = cg_block_sum<THREADS>(acc, sm);
      const bool stop = sqrt(rr_new) <= (double)c.tol * sqrt(gg);
      be = (float)(rr_new / in.rr);
      out.rr = rr_new;
      out.iters = in.iters + 1;
      out.cur = cur ^ 1;
      if (stop) out.active = 0;
      updated = true;
    }
  }
  float* __restrict__ r_out = cur ? c.r[0] : c.r[1];
  float* __restrict__ d_out = cur ? c.d[0] : c.d[1];
  float* __restrict__ p_out = cur ? c.p[0] : c.p[1];
  const bool want_p = c.final_p != 0;
  auto finish = [&](float rn, float dv_, float pv_, float& want, float& dn, float& pn) {
    dn = updated ? fmaf(be, dv_, rn) : dv_;   // nothing applied: the wanted vector is the current one
    pn = updated ? fmaf(al, dv_, pv_) : pv_;  // (dead code in workgroups that neither write nor want p)
    want = want_p ? pn : dn;
  };
#pragma unroll
  for (int u = 0; u < PERQ; ++u) {
    const int k = t + u * THREADS;
    if (k < n4) {
      float4 w4, d4, p4;
      finish(rv[u].x, dv[u].x, pv[u].x, w4.x, d4.x, p4.x);
      finish(rv[u].y, dv[u].y, pv[u].y, w4.y, d4.y, p4.y);
      finish(rv[u].z, dv[u].z, pv[u].z, w4.z, d4.z, p4.z);
      finish(rv[u].w, dv[u].w, pv[u].w, w4.w, d4.w, p4.w);
      reinterpret_cast<float4*>(vec)[k] = w4;
      if (writer) {
        if (updated) {
          reinterpret_cast<float4*>(r_out)[k] = rv[u];
          reinterpret_cast<float4*>(d_out)[k] = d4;
          reinterpret_cast<float4*>(p_out)[k] = p4;
        }
        if (want_p) reinterpret_cast<float4*>(c.p_final)[k] = p4;
      }
    }
  }
  if (tail) {
    float w1, d1, p1;
    finish(tr, td, tp, w1, d1, p1);
    vec[te] = w1;
    if (writer) {
      if (updated) { r_out[te] = tr; d_out[te] = d1; p_out[te] = p1; }
      if (want_p) c.p_final[te] = p1;
    }
  }
  if (writer && t == 0) {
    st->cgs[c.slot_in ^ 1] = out;
    if (updated && in.iters < kCgHist) st->cg_alphas[in.iters] = al;
    if (want_p) {  // the scalars that the line search and the statistics read
      st->rr = out.rr;
      st->cg_iters = out.iters;
      st->cg_active = out.active;
    }
  }
  lds_barrier();  // vec is complete (workgroup 0's global stores may still be on their way)
  return want_p || out.active != 0;
}

// The scalars of a pending update alone, for a kernel whose workgroups all need the step length of the last CG
// iteration (identical arithmetic in every workgroup): <d, q> from its partial sums in a fixed order, a = rr / <d, q>.
struct CgPendScalars {
  CgSlot in;
  double dq;
  float al;
  bool updated;   // the update takes place (CG active, positive curvature)
};
template <int THREADS>
__device__ __forceinline__ CgPendScalars cg_pending_scalars(const CgPend& c, double* sm) {
  CgPendScalars s;
  s.in = c.st->cgs[c.slot_in];
  double v = 0.0;
  for (int k = threadIdx.x; k < c.ndot; k += THREADS) v += c.dot_part[k];
  s.dq = cg_block_sum<THREADS>(v, sm);
  s.updated = s.in.active != 0 && s.dq > 0.0 && isfinite(s.dq);
  s.al = s.updated ? (float)(s.in.rr / s.dq) : 0.f;
  return s;
}

// The last update of a CG solve (c.final_p) by one workgroup that walks over the vectors in pieces (few registers: it
// runs beside other work in the same kernel): leaves the iterate in c.p_final and the final scalars in the state.
// The vector sets themselves are not advanced: nothing reads them after the last update.
template <int THREADS>
__device__ __forceinline__ void cg_pending_final_walk(const CgPend& c, double* sm) {
  const CgPendScalars s = cg_pending_scalars<THREADS>(c, sm);
  DevState* st = c.st;
  const int cur = s.in.cur & 1;
  const float* __restrict__ r_in = cur ? c.r[1] : c.r[0];
  const float* __restrict__ d_in = cur ? c.d[1] : c.d[0];
  const float* __restrict__ p_in = cur ? c.p[1] : c.p[0];
  const int n = (int)c.dlen, n4 = n >> 2;
  const float al = s.al;
  double acc = 0.0;
  constexpr int U = 2;
  for (int k0 = threadIdx.x; k0 < n4; k0 += U * THREADS) {
    float4 qv[U], rv[U], dv[U], pv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = k0 + u * THREADS < n4 ? k0 + u * THREADS : n4 - 1;
      qv[u] = reinterpret_cast<const float4*>(c.q)[k];
      rv[u] = reinterpret_cast<const float4*>(r_in)[k];
      dv[u] = reinterpret_cast<const float4*>(d_in)[k];
      pv[u] = reinterpret_cast<const float4*>(p_in)[k];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (k0 + u * THREADS < n4) {
        float4 pn = pv[u];
        if (s.updated) {
          const float r0 = fmaf(-al, qv[u].x, rv[u].x), r1 = fmaf(-al, qv[u].y, rv[u].y);
          const float r2 = fmaf(-al, qv[u].z, rv[u].z), r3 = fmaf(-al, qv[u].w, rv[u].w);
          acc += ((double)r0 * (double)r0 + (double)r1 * (double)r1) + ((double)r2 * (double)r2 + (double)r3 * (double)r3);
          pn.x = fmaf(al, dv[u].x, pv[u].x); pn.y = fmaf(al, dv[u].y, pv[u].y);
          pn.z = fmaf(al, dv[u].z, pv[u].z); pn.w = fmaf(al, dv[u].w, pv[u].w);
        }
        reinterpret_cast<float4*>(c.p_final)[k0 + u * THREADS] = pn;
      }
    }
  }
  if ((int)threadIdx.x < (n & 3)) {
    const int e = 4 * n4 + threadIdx.x;
    float pn = p_in[e];
    if (s.updated) {
      const float rn = fmaf(-al, c.q[e], r_in[e]);
      acc += (double)rn * (double)rn;
      pn = fmaf(al, d_in[e], pn);
    }
    c.p_final[e] = pn;
  }
  const double rr_new = cg_block_sum<THREADS>(acc, sm);
  if (threadIdx.x == 0) {
    CgSlot out = s.in;
    if (s.updated) {
      out.rr = rr_new;
      out.iters = s.in.iters + 1;
      if (sqrt(rr_new) <= (double)c.tol * sqrt(st->gg_cg)) out.active = 0;
      if (s.in.iters < kCgHist) st->cg_alphas[s.in.iters] = al;
    } else if (s.in.active != 0) {
      out.active = 0;  // no positive curvature: the current iterate stays
    }
    st->cgs[c.slot_in ^ 1] = out;
    st->rr = out.rr;
    st->cg_iters = out.iters;
    st->cg_active = out.active;
  }
}

}  // namespace nadmm
