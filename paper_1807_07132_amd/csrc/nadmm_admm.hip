// ADMM outer solver, consensus step (gfx950): z-update in closed form, multiplier update, residuals
// and stopping tolerances of Section 2.3 / 2.3.1 for N workers whose iterates sit in device memory.
// O(N d) streaming work; the sums are taken per workgroup and finished in a fixed order by one
// workgroup, so the result does not depend on scheduling.
#include "nadmm_internal.h"
#include "nadmm_mfma.h"

namespace nadmm {
namespace {

constexpr int kThreads = 256;
constexpr int kSums = 5;  // sum_i ||z - x_i||^2, sum_i rho_i^2 ||z - z_prev||^2, sum_i ||x_i||^2, ||z||^2, sum_i ||u_i||^2

__device__ __forceinline__ double wave_sum(double v) { return mfma_detail::wave64_sum(v); }  // in every lane, fixed order

__global__ __launch_bounds__(kThreads) void admm_init_kernel(AdmmState* st, float* u, float* z, int32_t N, int64_t d) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < (int64_t)N * d; e += stride) u[e] = 0.f;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < d; e += stride) z[e] = 0.f;
  if (st != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
    st->active = 1;
    st->rho_scale = 1.f;
    nadmm_admm_stats* s = &st->stats;
    s->outer_iters = 0;
    s->converged = 0;
    s->r_norm = 0.0; s->d_norm = 0.0; s->eps_pri = 0.0; s->eps_dual = 0.0;
    s->rho_scale = 1.0;
    for (int i = 0; i < NADMM_TRACE_LEN; ++i) { s->r_trace[i] = 0.0; s->d_trace[i] = 0.0; s->rho_scale_trace[i] = 0.0; }
  }
}

// z <- sum_i (rho_i x_i + u_i) / (lambda + sum_i rho_i);  u_i <- u_i + rho_i (x_i - z)
__global__ __launch_bounds__(kThreads) void admm_consensus_kernel(const AdmmConsensusArgs a) {
  if (a.st != nullptr && a.st->active == 0) return;
  __shared__ double sm[kThreads / 64][kSums];
  __shared__ float rho[NADMM_MAX_WORKERS];  // penalties of this iteration: the given ones times the common factor
  const float scale = a.st != nullptr ? a.st->rho_scale : 1.f;
  if (threadIdx.x < a.N) rho[threadIdx.x] = a.rho[threadIdx.x] * scale;
  __syncthreads();
  double rho_sum = 0.0, rho_sq = 0.0;
  for (int i = 0; i < a.N; ++i) {
    rho_sum += (double)rho[i];
    rho_sq += (double)rho[i] * (double)rho[i];
  }
  const float inv = (float)(1.0 / ((double)a.lambda + rho_sum));
  double acc[kSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < a.d; e += stride) {
    float num = 0.f;
    for (int i = 0; i < a.N; ++i) num += fmaf(rho[i], a.x[(size_t)i * a.d + e], a.u[(size_t)i * a.d + e]);
    const float zn = num * inv;
    const float zo = a.z[e];
    a.z[e] = zn;
    for (int i = 0; i < a.N; ++i) {
      const float xi = a.x[(size_t)i * a.d + e];
      const float un = fmaf(rho[i], xi - zn, a.u[(size_t)i * a.d + e]);
      a.u[(size_t)i * a.d + e] = un;
      const double r = (double)zn - (double)xi;
      acc[0] += r * r;
      acc[2] += (double)xi * (double)xi;
      acc[4] += (double)un * (double)un;
    }
    const double dz = (double)zn - (double)zo;
    acc[1] += rho_sq * dz * dz;
    acc[3] += (double)zn * (double)zn;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < kSums; ++k) {
    const double v = wave_sum(acc[k]);
    if (lane == 0) sm[wave][k] = v;
  }
  __syncthreads();
  if (threadIdx.x < kSums) {
    double t = 0.0;
    for (int wv = 0; wv < kThreads / 64; ++wv) t += sm[wv][threadIdx.x];
    a.part[(size_t)blockIdx.x * kSums + threadIdx.x] = t;
  }
}

// Norms, tolerances (Section 2.3.1) and the stopping decision.  The activity flag is written here and
// read by the kernels of the following launches only.
__global__ __launch_bounds__(kThreads) void admm_finish_kernel(const AdmmConsensusArgs a, int nblocks) {
  if (a.st != nullptr && a.st->active == 0) return;
  __shared__ double sm[kThreads / 64][kSums];
  __shared__ double tot[kSums];
  double acc[kSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  for (int b = threadIdx.x; b < nblocks; b += kThreads) {
#pragma unroll
    for (int k = 0; k < kSums; ++k) acc[k] += a.part[(size_t)b * kSums + k];
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < kSums; ++k) {
    const double v = wave_sum(acc[k]);
    if (lane == 0) sm[wave][k] = v;
  }
  __syncthreads();
  if (threadIdx.x < kSums) {
    double t = 0.0;
    for (int wv = 0; wv < kThreads / 64; ++wv) t += sm[wv][threadIdx.x];
    tot[threadIdx.x] = t;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  const double r_norm = sqrt(tot[0]), d_norm = sqrt(tot[1]);
  const double sx = sqrt(tot[2]), nz = sqrt((double)a.N * tot[3]), su = sqrt(tot[4]);
  const double eps_pri = sqrt((double)a.N) * (double)a.eps_abs + (double)a.eps_rel * (sx > nz ? sx : nz);
  const double eps_dual = sqrt((double)a.d) * (double)a.eps_abs + (double)a.eps_rel * su;
  if (a.out != nullptr) { a.out[0] = r_norm; a.out[1] = d_norm; a.out[2] = eps_pri; a.out[3] = eps_dual; }
  if (a.st != nullptr) {
    nadmm_admm_stats* s = &a.st->stats;
    s->outer_iters = a.iter + 1;
    s->r_norm = r_norm; s->d_norm = d_norm; s->eps_pri = eps_pri; s->eps_dual = eps_dual;
    float scale = a.st->rho_scale;
    if (a.iter < NADMM_TRACE_LEN) { s->r_trace[a.iter] = r_norm; s->d_trace[a.iter] = d_norm; s->rho_scale_trace[a.iter] = (double)scale; }
    if (r_norm <= eps_pri && d_norm <= eps_dual) {
      s->converged = 1;
      a.st->active = 0;
    } else if (a.penalty_rule == 1) {
      // residual balancing: a larger penalty shrinks the primal residual, a smaller one the dual residual
      if (r_norm > (double)a.rb_mu * d_norm) scale *= a.rb_tau;
      else if (d_norm > (double)a.rb_mu * r_norm) scale /= a.rb_tau;
      a.st->rho_scale = scale;
    }
    s->rho_scale = (double)scale;
  }
}

}  // namespace

int admm_blocks(int64_t d) {
  int64_t b = (d + kThreads - 1) / kThreads;
  return (int)(b < 1 ? 1 : (b > 1024 ? 1024 : b));
}

hipError_t launch_admm_init(AdmmState* st, float* u, float* z, int32_t N, int64_t d, hipStream_t stream) {
  int64_t b = ((int64_t)N * d + kThreads - 1) / kThreads;
  const int blocks = (int)(b < 1 ? 1 : (b > 1024 ? 1024 : b));
  hipLaunchKernelGGL(admm_init_kernel, dim3(blocks), dim3(kThreads), 0, stream, st, u, z, N, d);
  return hipGetLastError();
}

hipError_t launch_admm_consensus(const AdmmConsensusArgs& a, hipStream_t stream) {
  const int blocks = admm_blocks(a.d);
  hipLaunchKernelGGL(admm_consensus_kernel, dim3(blocks), dim3(kThreads), 0, stream, a);
  hipLaunchKernelGGL(admm_finish_kernel, dim3(1), dim3(kThreads), 0, stream, a, blocks);
  return hipGetLastError();
}

}  // namespace nadmm
