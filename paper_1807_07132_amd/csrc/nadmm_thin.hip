// Single-pass kernel for thin data (p <= 32 features, few classes), gfx950.
//
// With rows of 16..128 bytes the pass is a pure HBM stream (about 1.5 flop per
// byte for C = 2), so there is no contraction worth a matrix core: one lane owns
// one sample.  A workgroup copies a chunk of 256 consecutive rows -- a contiguous
// block of memory -- with coalesced 16-byte loads into LDS (row stride padded off
// the bank period), each lane reads its own row back, forms its logits Z = a_i X
// and W = a_i V with X and V as wave-uniform operands, the probabilities with the
// log-sum-exp shift (Section 2.2), its row of D (Section 2.6) or of P - Y, and
// accumulates a_i^T D into its private p x (C-1) registers.  The next chunk is
// already in flight in registers while the current one is consumed.  Per-lane
// accumulators are summed over the workgroup once, at the end, in a fixed order.
// Inside a Newton iteration the sweep of CG iteration k also does what lies between
// two sweeps (Section 2.4): it adds up the partial sums of sweep k - 1, forms q = H d
// and applies the CG update before it reads its operand (instantiations with CG).
#include <cstring>

#include "nadmm_internal.h"
#include "nadmm_cgstep.h"
#include "nadmm_mfma.h"

namespace nadmm {
namespace {

constexpr int kThinThreads = 256;
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct ThinArgs {
  RowArgs r;
  float* partial;      // gridDim.x x (p*NC) or NULL
  int32_t rows_per_wg; // multiple of 256
  int32_t lds_stride;  // floats per row in LDS
  int32_t q1024;       // 1024 / p
  int32_t r1024;       // 1024 % p
  // Deferred CG update (kernels instantiated with CG): the sweep of the previous CG iteration left only its per-workgroup
  // partial sums of A^T D.  Every workgroup of this sweep adds them up (fixed order), forms q = H d, applies the update of
  // Section 2.4 and takes its operand, the new direction (or, for the line search's pass, the final iterate), from there;
  // workgroup 0 stores the new vectors and state.  No reduction kernel and no CG kernel run between two sweeps.
  CgPend cg;           // cg.q and cg.dot_part are not used: this kernel forms both itself
  const float* prev;   // the previous sweep's partial sums, nprev x (p*NC)
  int32_t nprev;
  float scale, lambda, rho;
  const float* rho_scale;
};

// NQ = p / 4: float4 per row, which is also the float4 per lane in a chunk of 256 rows
template <int NQ, int NC, bool CG>
__global__ __launch_bounds__(kThinThreads) void thin_kernel(const ThinArgs ta) {
  constexpr int PP = 4 * NQ;
  constexpr int kMaxQuads = NQ;
  constexpr int nquads = NQ;
  const RowArgs& a = ta.r;
  if (a.flag != nullptr && *a.flag == 0) return;
  extern __shared__ __attribute__((aligned(16))) float tile[];  // 256 x lds_stride floats
  __shared__ double red[4];
  const int t = threadIdx.x;
  constexpr int p = PP;
  constexpr int PS = (PP % 8 == 0) ? PP + 4 : PP;  // LDS row stride, off the bank period
  const bool has0 = !CG && a.B0 != nullptr;
  const bool has1 = CG || a.B1 != nullptr;
  const bool with_cols = ta.partial != nullptr;

  const int64_t r_begin = (int64_t)blockIdx.x * ta.rows_per_wg;
  int64_t r_end = r_begin + ta.rows_per_wg;
  if (r_end > a.n) r_end = a.n;
  const f32x4* A4 = reinterpret_cast<const f32x4*>(a.A);
  const int64_t last4 = a.n * nquads - 1;  // last float4 of the matrix (lda == p)

  // X and V are the same for every lane: keep them as wave-uniform (scalar) registers
  float xs[PP][NC], vs[PP][NC];
  if constexpr (CG) {
    constexpr int D = PP * NC;      // length of the vectors, a multiple of 4
    constexpr int NQV = D / 4;      // quads per partial
    constexpr int GROUPS = kThinThreads / NQV;
    constexpr int U = 24;           // partials per thread and memory round trip
    __shared__ __attribute__((aligned(16))) float cgv[D];
    __shared__ __attribute__((aligned(16))) float cgq[D];
    __shared__ double cgdot[1];
    __shared__ double cgsm[kThinThreads / 64 + 1];
    const CgPend& c = ta.cg;
    const int cur = c.st->cgs[c.slot_in].cur & 1;
    const float* __restrict__ d_in = cur ? c.d[1] : c.d[0];
    const float rho_ = ta.rho_scale != nullptr ? ta.rho * *ta.rho_scale : ta.rho;
    const float dv = d_in[t < D ? t : D - 1];
    // thread (group g, quad qd) adds the partials g, g + GROUPS, ... of its quad, in that order
    const int qd = t % NQV, g = t / NQV;
    const int gc = g < GROUPS ? g : GROUPS - 1;
    const f32x4* __restrict__ pq = reinterpret_cast<const f32x4*>(ta.prev) + qd;
    f32x4 s4 = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k = gc; k < ta.nprev; k += U * GROUPS) {
      f32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = k + u * GROUPS;
        v[u] = pq[(size_t)(idx < ta.nprev ? idx : ta.nprev - 1) * NQV];
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (k + u * GROUPS < ta.nprev) s4 += v[u];
    }
    f32x4* gs = reinterpret_cast<f32x4*>(tile);  // [group][quad]: at most 256 quads, the smallest tile holds them
    if (g < GROUPS) gs[g * NQV + qd] = s4;
    __syncthreads();
    if (t < 64) {  // the vectors fit one wave
      double prod = 0.0;
      if (t < D) {
        float s2 = 0.f;
        for (int g2 = 0; g2 < GROUPS; ++g2) s2 += tile[(g2 * NQV + (t >> 2)) * 4 + (t & 3)];
        const float qv = fmaf(ta.lambda + rho_, dv, ta.scale * s2);
        cgq[t] = qv;
        prod = (double)dv * (double)qv;
      }
      prod = mfma_detail::wave64_sum(prod);
      if (t == 0) cgdot[0] = prod;
    }
    __syncthreads();
    CgPend c2 = c;
    c2.q = cgq;
    c2.dot_part = cgdot;
    c2.ndot = 1;
    if (!cg_pending_update<kThinThreads, 1>(c2, blockIdx.x == 0, cgv, cgsm, [] {})) return;
#pragma unroll
    for (int j = 0; j < PP; ++j)
#pragma unroll
      for (int c1 = 0; c1 < NC; ++c1) {
        xs[j][c1] = 0.f;
        vs[j][c1] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(cgv[j * NC + c1])));
      }
    __syncthreads();  // the tile is about to be overwritten by the first chunk
  } else {
#pragma unroll
    for (int j = 0; j < PP; ++j)
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        xs[j][c] = has0 ? __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.B0[j * NC + c]))) : 0.f;
        vs[j][c] = has1 ? __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.B1[j * NC + c]))) : 0.f;
      }
  }

  float acc[PP][NC];
#pragma unroll
  for (int j = 0; j < PP; ++j)
#pragma unroll
    for (int c = 0; c < NC; ++c) acc[j][c] = 0.f;
  double loss_acc = 0.0;

  // position of this lane's k-th float4 inside a chunk: element 4 (t + 256 k) = row * p + col
  int prow[kMaxQuads], pcol[kMaxQuads];
  {
    int row = (4 * t) / p, col = (4 * t) % p;
#pragma unroll
    for (int k = 0; k < kMaxQuads; ++k) {
      prow[k] = row;
      pcol[k] = col;
      row += ta.q1024;
      col += ta.r1024;
      if (col >= p) { col -= p; row += 1; }
    }
  }

  // Two chunks are in flight per workgroup: registers pf[0] and pf[1] alternate.  Loads are
  // unconditional (addresses clamped to the workgroup's own last float4), so the compiler can
  // wait for exactly the chunk it needs.
  f32x4 pf[2][kMaxQuads];
  const int64_t own_last4 = (r_end > r_begin ? r_end : r_begin + 1) * nquads - 1;
  auto load_chunk = [&](int b, int64_t row0) {
    const int64_t base4 = row0 * nquads + t;
#pragma unroll
    for (int k = 0; k < kMaxQuads; ++k) {
      int64_t i4 = base4 + (int64_t)k * kThinThreads;
      i4 = i4 < own_last4 ? i4 : own_last4;
      i4 = i4 < last4 ? i4 : last4;
      pf[b][k] = A4[i4];
    }
  };
  auto process = [&](int b, int64_t row0) {
    __syncthreads();  // rows of the previous chunk have been read
#pragma unroll
    for (int k = 0; k < kMaxQuads; ++k)
      *reinterpret_cast<f32x4*>(__builtin_assume_aligned(&tile[prow[k] * PS + pcol[k]], 16)) = pf[b][k];
    load_chunk(b, row0 + 2 * kThinThreads);
    __syncthreads();

    const int64_t row = row0 + t;
    const bool valid = row < r_end;
    float av[PP];
#pragma unroll
    for (int q = 0; q < PP / 4; ++q) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(__builtin_assume_aligned(&tile[t * PS + 4 * q], 16));
      av[4 * q + 0] = v[0]; av[4 * q + 1] = v[1]; av[4 * q + 2] = v[2]; av[4 * q + 3] = v[3];
    }
    float z[NC], w[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) { z[c] = 0.f; w[c] = 0.f; }
    if (has0) {
#pragma unroll
      for (int j = 0; j < PP; ++j)
#pragma unroll
        for (int c = 0; c < NC; ++c) z[c] = fmaf(av[j], xs[j][c], z[c]);
    }
    if (has1) {
#pragma unroll
      for (int j = 0; j < PP; ++j)
#pragma unroll
        for (int c = 0; c < NC; ++c) w[c] = fmaf(av[j], vs[j][c], w[c]);
    }
    const size_t ro = (size_t)row * NC;
    if (a.kind == kRowsLogits) {
      if (valid) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          if (has0 && a.Z0out) a.Z0out[ro + c] = z[c];
          if (has1 && a.Z1out) a.Z1out[ro + c] = w[c];
        }
      }
      return;
    }
    float P[NC], d[NC];
    float M = 0.f, alpha = 1.f;
    if (has0) {
#pragma unroll
      for (int c = 0; c < NC; ++c) M = fmaxf(M, z[c]);
      alpha = expf(-M);
#pragma unroll
      for (int c = 0; c < NC; ++c) { P[c] = expf(z[c] - M); alpha += P[c]; }
      const float inv = 1.f / alpha;
#pragma unroll
      for (int c = 0; c < NC; ++c) P[c] *= inv;
    } else {
#pragma unroll
      for (int c = 0; c < NC; ++c) P[c] = valid ? a.Pin[ro + c] : 0.f;
    }
    if (a.kind == kRowsHv) {
      float tt = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) tt = fmaf(P[c], w[c], tt);
#pragma unroll
      for (int c = 0; c < NC; ++c) d[c] = valid ? P[c] * (w[c] - tt) : 0.f;
    } else {
      const int b = valid ? a.labels[row] : -1;
      float zb = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        if (c == b) zb = z[c];
        d[c] = valid ? P[c] - (c == b ? 1.f : 0.f) : 0.f;
      }
      if (valid) loss_acc += (double)M + (double)logf(alpha) - (double)zb;
    }
    if (valid) {
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        if (a.Pout) a.Pout[ro + c] = P[c];
        if (has0 && a.Z0out) a.Z0out[ro + c] = z[c];
      }
    }
    if (with_cols) {
#pragma unroll
      for (int j = 0; j < PP; ++j)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[j][c] = fmaf(av[j], d[c], acc[j][c]);
    }
  };

  if (r_begin < r_end) {
    load_chunk(0, r_begin);
    load_chunk(1, r_begin + kThinThreads);
  }
  for (int64_t row0 = r_begin; row0 < r_end; row0 += 2 * kThinThreads) {
    process(0, row0);
    if (row0 + kThinThreads < r_end) process(1, row0 + kThinThreads);
  }

  // ---- workgroup sums: every accumulator over each row of 16 lanes by rotations (no shuffles: 28 trees of six
  // shuffles each took 5 us here, where nothing overlaps them), then the 16 row sums in a fixed order ----
  __syncthreads();
  float* wsum = tile;  // [wave][row of 16 lanes][PP*NC]: 16 sums per accumulator (at most 4 KB, the smallest tile)
  const int lane = t & 63, wave = t >> 6;
  if (with_cols) {
#pragma unroll
    for (int j = 0; j < PP; ++j)
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const float v = mfma_detail::row16_sum(acc[j][c]);
        if ((lane & 15) == 0) wsum[(wave * 4 + (lane >> 4)) * (PP * NC) + j * NC + c] = v;
      }
  }
  if (a.loss_part != nullptr) {
    loss_acc = mfma_detail::wave64_sum(loss_acc);
    if (lane == 0) red[wave] = loss_acc;
  }
  __syncthreads();
  if (with_cols && t < p * NC) {
    float w4[4];
#pragma unroll
    for (int w = 0; w < 4; ++w)
      w4[w] = (wsum[(4 * w) * (PP * NC) + t] + wsum[(4 * w + 1) * (PP * NC) + t]) +
              (wsum[(4 * w + 2) * (PP * NC) + t] + wsum[(4 * w + 3) * (PP * NC) + t]);
    ta.partial[(size_t)blockIdx.x * (p * NC) + t] = ((w4[0] + w4[1]) + w4[2]) + w4[3];
  }
  if (a.loss_part != nullptr && t == 0) a.loss_part[blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
}

int lds_stride_of(int p) { return (p % 8 == 0) ? p + 4 : p; }

template <int NQ, int NC>
hipError_t launch_thin_t(const ThinArgs& ta, int grid, bool cg, hipStream_t st) {
  const size_t lds = (size_t)kThinThreads * ta.lds_stride * sizeof(float);
  if (cg) hipLaunchKernelGGL((thin_kernel<NQ, NC, true>), dim3(grid), dim3(kThinThreads), lds, st, ta);
  else hipLaunchKernelGGL((thin_kernel<NQ, NC, false>), dim3(grid), dim3(kThinThreads), lds, st, ta);
  return hipGetLastError();
}

template <int NQ>
hipError_t launch_thin_nq(const ThinArgs& ta, int grid, bool cg, hipStream_t st) {
  switch (ta.r.NC) {
    case 1: return launch_thin_t<NQ, 1>(ta, grid, cg, st);
    case 2: return launch_thin_t<NQ, 2>(ta, grid, cg, st);
    case 3: return launch_thin_t<NQ, 3>(ta, grid, cg, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool thin_supported(const Shape& s, int64_t lda, const void* A) {
  if (s.p > 32 || (s.p & 3) != 0 || s.NC > 3 || s.p * s.NC > 64) return false;
  if (lda != s.p || (reinterpret_cast<uintptr_t>(A) & 15) != 0) return false;
  return true;
}

int thin_num_partials(const Shape& s) {
  // 3 resident workgroups per compute unit for small accumulator sets, else 2 (register budget);
  // every workgroup gets the same whole number of 256-row chunks
  const int64_t cap = (s.p * s.NC <= 32) ? 768 : 512;
  const int64_t chunks = (s.n + kThinThreads - 1) / kThinThreads;
  const int64_t g = chunks < cap ? chunks : cap;
  const int64_t per = (chunks + g - 1) / g;
  return (int)((chunks + per - 1) / per);
}

hipError_t launch_thin(const RowArgs& a, float* partial, int nparts, hipStream_t st, const CgPend* cg, const ReduceArgs* prev) {
  ThinArgs ta;
  std::memset(&ta, 0, sizeof(ta));
  ta.r = a;
  ta.partial = partial;
  const int64_t chunks = (a.n + kThinThreads - 1) / kThinThreads;
  ta.rows_per_wg = (int32_t)((chunks + nparts - 1) / nparts) * kThinThreads;
  ta.lds_stride = lds_stride_of(a.p);  // must equal the kernel's compile-time stride
  ta.q1024 = 1024 / a.p;
  ta.r1024 = 1024 % a.p;
  const bool with_cg = cg != nullptr;
  if (with_cg) {
    // the pending update of a CG iteration on cached probabilities (or the line search's logits pass on the final iterate)
    if (prev == nullptr || prev->partial == nullptr || prev->nparts < 1 || prev->d != (int64_t)a.p * a.NC) return hipErrorInvalidValue;
    if (a.B0 != nullptr || (a.kind != kRowsHv && a.kind != kRowsLogits) || cg->dlen != prev->d || cg->st == nullptr) return hipErrorInvalidValue;
    if (prev->partial == partial) return hipErrorInvalidValue;  // the sweep reads the previous partials while it writes its own
    ta.cg = *cg;
    ta.prev = prev->partial;
    ta.nprev = prev->nparts;
    ta.scale = prev->scale;
    ta.lambda = prev->lambda;
    ta.rho = prev->rho;
    ta.rho_scale = prev->rho_scale;
  }
  switch (a.p >> 2) {
    case 1: return launch_thin_nq<1>(ta, nparts, with_cg, st);
    case 2: return launch_thin_nq<2>(ta, nparts, with_cg, st);
    case 3: return launch_thin_nq<3>(ta, nparts, with_cg, st);
    case 4: return launch_thin_nq<4>(ta, nparts, with_cg, st);
    case 5: return launch_thin_nq<5>(ta, nparts, with_cg, st);
    case 6: return launch_thin_nq<6>(ta, nparts, with_cg, st);
    case 7: return launch_thin_nq<7>(ta, nparts, with_cg, st);
    case 8: return launch_thin_nq<8>(ta, nparts, with_cg, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nadmm
