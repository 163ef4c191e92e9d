// Kernels for A in sparse storage (gfx950): both products with A are the same operation, a
// compressed-rows matrix S times a dense matrix B with few columns,
//   pass 1:  [Z | W] = A [X | V]      S = row view of A,    B = [X | V]   (Sections 2.1, 2.6)
//   pass 2:  A^T D                    S = column view of A, B = D         (Section 2.6)
// followed by the rows stage on logits and the fixed-order reduction that the dense paths use.
//
// One lane per stored entry: a wave reads 64 (index, value) pairs with two coalesced loads, each
// lane then gathers the whole row of B that its entry points to with 16-byte loads (the rows of B
// are first copied into a buffer whose rows are padded to a multiple of 4 floats, so that they are
// 16-byte aligned) and keeps its own partial sums; at the end of a row of S the lanes' sums are
// added across the wave.  Work is cut into windows of equal cost (stored entries plus a fixed cost
// per row) by a binary search over the row pointers; a workgroup owns the rows that start in its
// window: short rows go to single waves, long ones are shared by its four waves and combined in
// LDS in wave order.  Every output row is written by exactly one workgroup, in an order of additions
// that depends on the matrix only: results are reproducible bit for bit.
#include "nadmm_internal.h"
#include "nadmm_mfma.h"

namespace nadmm {
namespace {

constexpr int kSpThreads = 256;
constexpr int kSpWaves = kSpThreads / 64;
constexpr int kWindow = 4096;  // cost units per workgroup
constexpr int kRowCost = 8;    // cost of a row beyond its entries (bounds the rows per window by kWindow / kRowCost)
constexpr int kLong = 512;     // rows with at least this many entries are shared by the waves of the workgroup
constexpr int kMaxLong = kWindow / (kLong + kRowCost) + 2;

// first row r in [0, nrows] whose cost prefix ptr[r] + kRowCost r reaches `target`
__global__ __launch_bounds__(256) void plan_kernel(const SparseView S, int32_t* __restrict__ win, int nwin) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k > nwin) return;
  if (k == nwin) {
    win[k] = (int32_t)S.nrows;
    return;
  }
  const int64_t target = (int64_t)k * kWindow;
  int64_t lo = 0, hi = S.nrows;  // answer in [lo, hi]
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (S.ptr[mid] + (int64_t)kRowCost * mid >= target) hi = mid;
    else lo = mid + 1;
  }
  win[k] = (int32_t)lo;
}

// dst[r][op][NCpad] = src_op[r][NC], zero in the padding; one thread per group of 4 floats
__global__ __launch_bounds__(256) void pack_kernel(const float* __restrict__ src0, const float* __restrict__ src1,
                                                   int64_t rows, int NC, int NCpad, int nops,
                                                   float* __restrict__ dst, const int32_t* flag) {
  if (flag != nullptr && *flag == 0) return;
  const int quads = NCpad >> 2;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = rows * nops * quads;
  if (t >= total) return;
  const int q = (int)(t % quads);
  const int64_t ro = t / quads;
  const int op = (int)(ro % nops);
  const int64_t r = ro / nops;
  const float* __restrict__ src = (op == 0 ? src0 : src1) + (size_t)r * NC;
  mfma_detail::f32x4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = (4 * q + e < NC) ? src[4 * q + e] : 0.f;
  reinterpret_cast<mfma_detail::f32x4*>(dst)[t] = v;
}

__device__ __forceinline__ float wave_sum64(float v) {
  v = mfma_detail::row16_sum(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

struct RowSpan {
  int64_t k0, k1;
};
__device__ __forceinline__ RowSpan row_span(const SparseView& S, int64_t r) {
  int64_t k0 = S.ptr[r], k1 = S.ptr[r + 1];
  k0 = k0 < 0 ? 0 : (k0 > S.nnz ? S.nnz : k0);
  k1 = k1 < k0 ? k0 : (k1 > S.nnz ? S.nnz : k1);
  return RowSpan{k0, k1};
}

// One wave-step: lane l takes entry kb + l of [.., k1); adds value * (row of B) to its sums.
template <int NQ>
struct Step {
  int col;
  float v;
  __device__ __forceinline__ void fetch(const SparseView& S, int64_t kb, int64_t k1, int lane) {
    const int64_t k = kb + lane;
    const bool ok = k < k1;
    const int64_t kc = ok ? k : k1 - 1;
    const int c = S.idx[kc];
    v = ok ? S.val[kc] : 0.f;
    col = c < 0 ? 0 : (c >= S.ncols ? S.ncols - 1 : c);
  }
};

template <int NQ>
__device__ __forceinline__ void gather(const float* __restrict__ B, int col, mfma_detail::f32x4 (&b)[NQ]) {
  const mfma_detail::f32x4* __restrict__ row = reinterpret_cast<const mfma_detail::f32x4*>(B) + (size_t)col * NQ;
#pragma unroll
  for (int q = 0; q < NQ; ++q) b[q] = row[q];
}

template <int NQ>
__device__ __forceinline__ void fma_row(float v, const mfma_detail::f32x4 (&b)[NQ], float (&acc)[4 * NQ]) {
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[4 * q + e] = fmaf(v, b[q][e], acc[4 * q + e]);
  }
}

// Entries kb0, kb0 + stride, ... (64 per step) of [.., k1): the sum of value * B row over them, added across the
// wave; lane j returns element j of the packed row.  Two steps are in flight at a time.
template <int NQ>
__device__ __forceinline__ float row_sum(const SpmmArgs& a, int64_t kb0, int64_t k1, int stride, int lane) {
  float acc[4 * NQ];
#pragma unroll
  for (int j = 0; j < 4 * NQ; ++j) acc[j] = 0.f;
  int64_t kb = kb0;
  for (; kb + stride < k1; kb += 2 * (int64_t)stride) {
    Step<NQ> s0, s1;
    s0.fetch(a.S, kb, k1, lane);
    s1.fetch(a.S, kb + stride, k1, lane);
    mfma_detail::f32x4 b0[NQ], b1[NQ];
    gather<NQ>(a.B, s0.col, b0);
    gather<NQ>(a.B, s1.col, b1);
    fma_row<NQ>(s0.v, b0, acc);
    fma_row<NQ>(s1.v, b1, acc);
  }
  if (kb < k1) {
    Step<NQ> s0;
    s0.fetch(a.S, kb, k1, lane);
    mfma_detail::f32x4 b0[NQ];
    gather<NQ>(a.B, s0.col, b0);
    fma_row<NQ>(s0.v, b0, acc);
  }
  float res = 0.f;
#pragma unroll
  for (int j = 0; j < 4 * NQ; ++j) {
    const float s = wave_sum64(acc[j]);
    res = (lane == j) ? s : res;
  }
  return res;
}

// element j of a packed row -> position in the output row [op][NC], or -1 for padding
__device__ __forceinline__ int out_col(const SpmmArgs& a, int j) {
  const int op = (a.nops == 2 && j >= a.NCpad) ? 1 : 0;
  const int c = j - op * a.NCpad;
  return c < a.NC ? op * a.NC + c : -1;
}

template <int NQ>
__global__ __launch_bounds__(kSpThreads) void spmm_kernel(const SpmmArgs a) {
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ int long_rows[kMaxLong];
  __shared__ int nlong_sh;
  __shared__ float part[kMaxLong][kSpWaves][4 * NQ];
  const int r0 = a.win[blockIdx.x], r1 = a.win[blockIdx.x + 1];
  if (r1 <= r0) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ldo = a.nops * a.NC;
  const int oc = lane < 4 * NQ ? out_col(a, lane) : -1;

  if (threadIdx.x == 0) nlong_sh = 0;
  __syncthreads();
  for (int r = r0 + (int)threadIdx.x; r < r1; r += kSpThreads) {
    const RowSpan sp = row_span(a.S, r);
    if (sp.k1 - sp.k0 >= kLong) {
      const int slot = atomicAdd(&nlong_sh, 1);
      if (slot < kMaxLong) long_rows[slot] = r;
    }
  }
  __syncthreads();
  const int nlong = nlong_sh < kMaxLong ? nlong_sh : kMaxLong;

  // long rows: wave w takes steps w, w + 4, ...; partial sums to LDS
  for (int s = 0; s < nlong; ++s) {
    const RowSpan sp = row_span(a.S, long_rows[s]);
    const float res = row_sum<NQ>(a, sp.k0 + 64 * wave, sp.k1, 64 * kSpWaves, lane);
    if (lane < 4 * NQ) part[s][wave][lane] = res;
  }
  // short rows: one wave each
  for (int r = r0 + wave; r < r1; r += kSpWaves) {
    const RowSpan sp = row_span(a.S, r);
    const int64_t len = sp.k1 - sp.k0;
    if (len >= kLong) continue;
    float res = 0.f;
    if (len > 0) res = row_sum<NQ>(a, sp.k0, sp.k1, 64, lane);
    if (oc >= 0) a.out[(size_t)r * ldo + oc] = res;
  }
  if (nlong == 0) return;
  __syncthreads();
  for (int t = threadIdx.x; t < nlong * 4 * NQ; t += kSpThreads) {
    const int s = t / (4 * NQ), j = t - s * (4 * NQ);
    float sum = part[s][0][j];
#pragma unroll
    for (int w = 1; w < kSpWaves; ++w) sum += part[s][w][j];
    const int c = out_col(a, j);
    if (c >= 0) a.out[(size_t)long_rows[s] * ldo + c] = sum;
  }
}

template <int NQ>
hipError_t launch_nq(const SpmmArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(spmm_kernel<NQ>, dim3(a.nwin), dim3(kSpThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace

int sparse_pad(int NC) { return (NC + 3) & ~3; }

int sparse_windows(int64_t nrows, int64_t nnz) {
  const int64_t total = nnz + (int64_t)kRowCost * nrows;
  const int64_t w = (total + kWindow - 1) / kWindow;
  return (int)(w < 1 ? 1 : w);
}

hipError_t launch_sparse_plan(const SparseView& S, int32_t* win, int nwin, hipStream_t st) {
  hipLaunchKernelGGL(plan_kernel, dim3((nwin + 1 + 255) / 256), dim3(256), 0, st, S, win, nwin);
  return hipGetLastError();
}

hipError_t launch_sparse_pack(const float* src0, const float* src1, int64_t rows, int NC, float* dst,
                              const int32_t* flag, hipStream_t st) {
  const float* s0 = src0 ? src0 : src1;
  const int nops = (src0 && src1) ? 2 : 1;
  const int NCpad = sparse_pad(NC);
  const int64_t total = rows * nops * (NCpad >> 2);
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s0, src1, rows, NC, NCpad,
                     nops, dst, flag);
  return hipGetLastError();
}

hipError_t launch_spmm(const SpmmArgs& a, hipStream_t st) {
  const int nq = a.nops * (a.NCpad >> 2);
  switch (nq) {
    case 1: return launch_nq<1>(a, st);
    case 2: return launch_nq<2>(a, st);
    case 3: return launch_nq<3>(a, st);
    case 4: return launch_nq<4>(a, st);
    case 5: return launch_nq<5>(a, st);
    case 6: return launch_nq<6>(a, st);
    case 7: return launch_nq<7>(a, st);
    case 8: return launch_nq<8>(a, st);
    case 10: return launch_nq<10>(a, st);
    case 12: return launch_nq<12>(a, st);
    case 14: return launch_nq<14>(a, st);
    case 16: return launch_nq<16>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nadmm
