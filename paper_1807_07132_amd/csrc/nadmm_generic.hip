// Two-pass float32 vector kernels for any shape (gfx950).
//
// Pass 1 (rows): one lane per sample.  Column tiles of A are staged through LDS
// so that global reads are coalesced along rows while each lane walks its own
// row; the entries of X / V for the current column are wave-uniform.  Each lane
// ends with its row of logits Z = a_i X and directional logits W = a_i V, forms
// the probabilities with the log-sum-exp shift (Section 2.2) and writes the row
// of D (Section 2.6, eq. matrix-c) or of P - Y.
// Pass 2 (columns): one lane per feature column accumulates A^T rows over a
// chunk of samples; chunk partials are summed in a fixed order afterwards.
#include "nadmm_internal.h"
#include "nadmm_mfma.h"
#include "nadmm_rows16.h"

namespace nadmm {
namespace {

constexpr int kRowsPerBlock = 256;  // 4 waves x 64 rows
constexpr int kTileCols = 32;

__device__ __forceinline__ double block_sum_double(double v, double* sm /* >= 4 doubles */) {
  v = mfma_detail::wave64_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sm[wave] = v;
  __syncthreads();
  double t = 0.0;
  const int nw = (blockDim.x + 63) >> 6;
  for (int w = 0; w < nw; ++w) t += sm[w];
  return t;
}

// Rows stage shared by the kernels that end with one lane holding the logits of one sample:
// probabilities with the log-sum-exp shift (Sections 2.2, 2.6), the row of D or of P - Y, the row loss,
// optional stores of P and of the logits.  Returns the row loss (0 for kinds without one).
template <int NCP>
__device__ __forceinline__ double finish_row(const RowArgs& a, int64_t row, bool valid, bool has0, bool has1,
                                             const float (&z)[NCP], const float (&w)[NCP]) {
  const int NC = a.NC;
  const size_t ro = (size_t)row * NC;
  if (a.kind == kRowsLogits) {
    if (valid) {
#pragma unroll
      for (int c = 0; c < NCP; ++c)
        if (c < NC) {
          if (has0 && a.Z0out) a.Z0out[ro + c] = z[c];
          if (has1 && a.Z1out) a.Z1out[ro + c] = w[c];
        }
    }
    return 0.0;
  }
  float P[NCP];
  float M = 0.f, alpha = 1.f;
  if (has0) {
#pragma unroll
    for (int c = 0; c < NCP; ++c)
      if (c < NC) M = fmaxf(M, z[c]);
    alpha = expf(-M);
#pragma unroll
    for (int c = 0; c < NCP; ++c) {
      P[c] = (c < NC) ? expf(z[c] - M) : 0.f;
      alpha += P[c];
    }
    const float inv = 1.f / alpha;
#pragma unroll
    for (int c = 0; c < NCP; ++c) P[c] *= inv;
  } else {
#pragma unroll
    for (int c = 0; c < NCP; ++c) P[c] = (valid && c < NC) ? a.Pin[ro + c] : 0.f;
  }
  if (a.kind == kRowsHv) {
    float t = 0.f;
#pragma unroll
    for (int c = 0; c < NCP; ++c) t = fmaf(P[c], w[c], t);
    if (valid) {
#pragma unroll
      for (int c = 0; c < NCP; ++c)
        if (c < NC) {
          a.rows_out[ro + c] = P[c] * (w[c] - t);
          if (a.Pout) a.Pout[ro + c] = P[c];
        }
    }
    return 0.0;
  }
  double ell = 0.0;
  if (valid) {
    const int b = a.labels[row];
    float zb = 0.f;
#pragma unroll
    for (int c = 0; c < NCP; ++c)
      if (c < NC && c == b) zb = z[c];
    ell = (double)M + (double)logf(alpha) - (double)zb;
#pragma unroll
    for (int c = 0; c < NCP; ++c)
      if (c < NC) {
        if (a.kind == kRowsGrad && a.rows_out) a.rows_out[ro + c] = P[c] - (c == b ? 1.f : 0.f);
        if (a.Pout) a.Pout[ro + c] = P[c];
        if (a.Z0out) a.Z0out[ro + c] = z[c];
      }
  }
  return ell;
}

template <int NCP>
__global__ __launch_bounds__(kRowsPerBlock) void rows_kernel(const RowArgs a) {
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ float tile[4][64][kTileCols + 1];
  __shared__ double red[4];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row0 = ((int64_t)blockIdx.x * 4 + wave) * 64;
  const int64_t row = row0 + lane;
  const int NC = a.NC;
  const bool has0 = a.B0 != nullptr;
  const bool has1 = a.B1 != nullptr;

  // The logits Z are summed in float32 over one column tile (32 terms) and the tile sums in float64: exp()
  // turns the absolute error of a logit into a relative error of the probabilities (Section 2.2), and a
  // float32 sum over thousands of columns would carry 1e-4 at logits of a few hundred.
  float z[NCP], w[NCP];
  double zd[NCP];
#pragma unroll
  for (int c = 0; c < NCP; ++c) { z[c] = 0.f; w[c] = 0.f; zd[c] = 0.0; }

  const int lr = lane >> 5, lc = lane & 31;
  for (int j0 = 0; j0 < a.p; j0 += kTileCols) {
    __syncthreads();
#pragma unroll 8
    for (int it = 0; it < 32; ++it) {
      const int r = 2 * it + lr;
      const int64_t gi = row0 + r;
      const int gj = j0 + lc;
      float v = 0.f;
      if (gi < a.n && gj < a.p) v = a.A[gi * a.lda + gj];
      tile[wave][r][lc] = v;
    }
    __syncthreads();
    const int jmax = min(kTileCols, a.p - j0);
    for (int jj = 0; jj < jmax; ++jj) {
      const float av = tile[wave][lane][jj];
      const size_t boff = (size_t)(j0 + jj) * NC;
      if (has0) {
        const float* __restrict__ x = a.B0 + boff;
#pragma unroll
        for (int c = 0; c < NCP; ++c)
          if (c < NC) z[c] = fmaf(av, x[c], z[c]);
      }
      if (has1) {
        const float* __restrict__ v = a.B1 + boff;
#pragma unroll
        for (int c = 0; c < NCP; ++c)
          if (c < NC) w[c] = fmaf(av, v[c], w[c]);
      }
    }
    if (has0) {
#pragma unroll
      for (int c = 0; c < NCP; ++c) { zd[c] += (double)z[c]; z[c] = 0.f; }
    }
  }
  if (has0) {
#pragma unroll
    for (int c = 0; c < NCP; ++c) z[c] = (float)zd[c];
  }

  const bool valid = row < a.n;
  const double ell = finish_row<NCP>(a, row, valid, has0, has1, z, w);
  if (a.kind != kRowsGrad && a.kind != kRowsLoss) return;
  const double tot = block_sum_double(ell, red);
  if (threadIdx.x == 0) a.loss_part[blockIdx.x] = tot;
}

// Rows stage on logits that were computed elsewhere: the column-sliced matrix-core pass leaves one partial
// n x {1,2} x (C-1) array [Z | W] per column slice (only the matrices whose operand was given); this kernel
// adds the slices in order and finishes the rows.
constexpr int kLogitThreads = 1024;  // 16 waves x 16 rows = the kRowsPerBlock rows of one partial loss

// Lane (g, m) of a wave holds classes m, 16 + m, ... of row 4 it + g: the loads and stores of a wave
// cover whole rows of the n x (C-1) arrays back to back; the rows are finished by rows16::finish.
template <int NB>
__global__ __launch_bounds__(kLogitThreads) void logit_rows_kernel(const RowArgs a, const float* __restrict__ zw,
                                                                   int nslices) {
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ double red[kLogitThreads / 64];
  constexpr int kIters = 4;
  const int NC = a.NC;
  const bool has0 = a.B0 != nullptr;
  const bool has1 = a.B1 != nullptr;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, g = lane >> 4;
  const int64_t wrow0 = (int64_t)blockIdx.x * kRowsPerBlock + wave * (4 * kIters);
  const bool with_loss = a.kind == kRowsGrad || a.kind == kRowsLoss;
  const int nmat = (has0 ? 1 : 0) + (has1 ? 1 : 0);  // matrices held per slice and row: [Z][W], [Z] or [W]
  const int woff = has0 ? NC : 0;
  const rows16::LaneClasses<NB> lc(m, NC);

  float z[kIters][NB], w[kIters][NB], aux[kIters][NB];
  int label[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int64_t row = wrow0 + 4 * it + g;
    const int64_t rowc = row < a.n ? row : a.n - 1;
    label[it] = with_loss ? a.labels[rowc] : 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      z[it][nb] = 0.f;
      w[it][nb] = 0.f;
      aux[it][nb] = (!has0 && a.kind == kRowsHv) ? a.Pin[(size_t)rowc * NC + lc.cl[nb]] : 0.f;
    }
  }
  for (int s = 0; s < nslices; ++s) {  // slices are added in order
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      const int64_t row = wrow0 + 4 * it + g;
      const int64_t rowc = row < a.n ? row : a.n - 1;
      const float* src = zw + ((size_t)s * a.n + rowc) * nmat * NC;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        if (has0) z[it][nb] += src[lc.cl[nb]];
        if (has1) w[it][nb] += src[woff + lc.cl[nb]];
      }
    }
  }

  double ell = 0.0;
#pragma unroll
  for (int it = 0; it < kIters; ++it)
    ell += rows16::finish<NB>(a, wrow0 + 4 * it + g, m, lc, has0, has1, z[it], w[it], aux[it], label[it]);
  if (!with_loss) return;
  ell = mfma_detail::wave64_sum(ell);
  if (lane == 0) red[wave] = ell;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int wv = 0; wv < kLogitThreads / 64; ++wv) t += red[wv];
    a.loss_part[blockIdx.x] = t;
  }
}

template <int NCP>
__global__ __launch_bounds__(256) void cols_kernel(const ColArgs a) {
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ float sm[3][NCP][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = blockIdx.x * 64 + lane;
  const bool jv = j < a.p;
  const int NC = a.NC;
  const int64_t r0 = (int64_t)blockIdx.y * a.rows_per_chunk;
  int64_t r1 = r0 + a.rows_per_chunk;
  if (r1 > a.n) r1 = a.n;

  float acc[NCP];
#pragma unroll
  for (int c = 0; c < NCP; ++c) acc[c] = 0.f;

  const float* __restrict__ Ap = a.A + (jv ? j : 0);
#pragma unroll 4
  for (int64_t i = r0 + wave; i < r1; i += 4) {
    const float av = jv ? Ap[i * a.lda] : 0.f;
    const float* __restrict__ drow = a.rows_in + (size_t)i * NC;
#pragma unroll
    for (int c = 0; c < NCP; ++c)
      if (c < NC) acc[c] = fmaf(av, drow[c], acc[c]);
  }
  if (wave > 0) {
#pragma unroll
    for (int c = 0; c < NCP; ++c) sm[wave - 1][c][lane] = acc[c];
  }
  __syncthreads();
  if (wave == 0 && jv) {
    float* out = a.partial + (size_t)blockIdx.y * ((size_t)a.p * NC) + (size_t)j * NC;
#pragma unroll
    for (int c = 0; c < NCP; ++c)
      if (c < NC) out[c] = ((acc[c] + sm[0][c][lane]) + sm[1][c][lane]) + sm[2][c][lane];
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

int generic_row_blocks(int64_t n) { return (int)((n + kRowsPerBlock - 1) / kRowsPerBlock); }

void generic_col_grid(const Shape& s, int* nslabs, int* nchunks, int* rows_per_chunk) {
  const int slabs = (s.p + 63) / 64;
  int64_t chunks = (2048 + slabs - 1) / slabs;
  const int64_t max_chunks = (s.n + 63) / 64;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  int64_t rpc = (s.n + chunks - 1) / chunks;
  rpc = (rpc + 3) / 4 * 4;
  chunks = (s.n + rpc - 1) / rpc;
  *nslabs = slabs;
  *nchunks = (int)chunks;
  *rows_per_chunk = (int)rpc;
}

hipError_t launch_generic_rows(const RowArgs& a, hipStream_t st) {
  const int blocks = generic_row_blocks(a.n);
  return dispatch_ncp(a.NC, [&](auto ncp) {
    constexpr int NCP = decltype(ncp)::value;
    hipLaunchKernelGGL(rows_kernel<NCP>, dim3(blocks), dim3(kRowsPerBlock), 0, st, a);
    return hipGetLastError();
  });
}

hipError_t launch_logit_rows(const RowArgs& a, const float* zw, int nslices, hipStream_t st) {
  const int blocks = generic_row_blocks(a.n);
  if (a.NC <= 16) hipLaunchKernelGGL(logit_rows_kernel<1>, dim3(blocks), dim3(kLogitThreads), 0, st, a, zw, nslices);
  else if (a.NC <= 32) hipLaunchKernelGGL(logit_rows_kernel<2>, dim3(blocks), dim3(kLogitThreads), 0, st, a, zw, nslices);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_generic_cols(const ColArgs& a, int nslabs, int nchunks, hipStream_t st) {
  return dispatch_ncp(a.NC, [&](auto ncp) {
    constexpr int NCP = decltype(ncp)::value;
    hipLaunchKernelGGL(cols_kernel<NCP>, dim3(nslabs, nchunks), dim3(256), 0, st, a);
    return hipGetLastError();
  });
}

}  // namespace nadmm
