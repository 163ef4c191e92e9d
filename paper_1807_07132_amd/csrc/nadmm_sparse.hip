// Kernels for A in sparse storage (gfx950): both products with A are the same operation, a
// compressed-rows matrix S times a dense matrix B with few columns,
//   pass 1:  [Z | W] = A [X | V]      S = row view of A,    B = [X | V]   (Sections 2.1, 2.6)
//   pass 2:  A^T D                    S = column view of A, B = D         (Section 2.6)
// followed by the rows stage on logits and the fixed-order reduction that the dense paths use.
//
// The rows of B are first copied into a buffer in which every row takes a power-of-two number G of
// 16-byte quads (zero padded), so that a row lies in one 128-byte cache line.  A wave reads 64 (index,
// value) pairs with two coalesced loads and hands them out by lane shuffles; as many neighbouring lanes
// as a row of B has quads then share an entry, each loading one quad of the row that the entry points to,
// so that a load instruction touches each of its rows once, and each lane keeps the partial sums of its quad; at the
// end of a row of S the lanes holding the same quad are added across the wave.  Work is cut into
// windows of equal cost (stored entries plus a fixed cost per row) by a binary search over the row
// pointers; a workgroup owns the rows that start in its window: short rows go to single waves, long
// ones are shared by its four waves and combined in LDS in wave order.  Every output row is written by
// exactly one workgroup, in an order of additions that depends on the matrix only: results are
// reproducible bit for bit.
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

// dst[r][op][slot] = src_op[r][NC], zero in the padding (slot = 4 G floats); one thread per group of 4 floats
__global__ __launch_bounds__(256) void pack_kernel(const float* __restrict__ src0, const float* __restrict__ src1,
                                                   int64_t rows, int NC, int G, int nops,
                                                   float* __restrict__ dst, const int32_t* flag) {
  if (flag != nullptr && *flag == 0) return;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = rows * nops * G;
  if (t >= total) return;
  const int q = (int)(t % G);
  const int64_t ro = t / G;
  const int op = (int)(ro % nops);
  const int64_t r = ro / nops;
  const float* __restrict__ src = (op == 0 ? src0 : src1) + (size_t)r * NC;
  mfma_detail::f32x4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = (4 * q + e < NC) ? src[4 * q + e] : 0.f;
  reinterpret_cast<mfma_detail::f32x4*>(dst)[t] = v;
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

// the stored entries of a chunk from kb on, one per lane (value 0 and a valid index beyond the end)
struct Chunk {
  int col;
  float v;
};
__device__ __forceinline__ Chunk fetch_chunk(const SparseView& S, int64_t kb, int64_t k1, int64_t kend, int lane) {
  const int64_t k = kb + lane;
  const bool ok = k < kend;  // kend = k1, or 0 in lanes that never hold an entry
  const int64_t kc = k < k1 ? k : k1 - 1;
  const int c = S.idx[kc];
  Chunk ch;
  ch.v = ok ? S.val[kc] : 0.f;
  ch.col = c < 0 ? 0 : (c >= S.ncols ? S.ncols - 1 : c);
  return ch;
}

// Lanes per wave that hold entries, for rows of NQ quads: S = 64 / NQ entries share a load instruction
// (lane = s NQ + q reads quad q of the B row of entry s), a chunk is T = 64 / S such groups.
template <int NQ>
struct Shape64 {
  static constexpr int S = 64 / NQ;
  static constexpr int T = 64 / S;
  static constexpr int CE = S * T;  // entries per chunk: 64, or a little less where NQ does not divide 64
};

// The sum of value * (row of B) over the entries of the chunks kb0, kb0 + stride, ... of [.., k1).
// NQ neighbouring lanes share an entry, one quad of its B row each, so that one load instruction touches
// every row once (several loads of one lane to one cache line would wait on each other in the vector
// L1).  Returns, in lanes 0 .. NQ-1, the sums of quad q = lane over the whole wave.
template <int NQ, int NOPS>
__device__ __forceinline__ void row_sum(const SpmmArgs& a, int64_t kb0, int64_t k1, int stride, int lane,
                                        mfma_detail::f32x4 (&acc)[NOPS]) {
  using mfma_detail::f32x4;
  constexpr int S = Shape64<NQ>::S, T = Shape64<NQ>::T, CE = Shape64<NQ>::CE;
  constexpr int G = NQ <= 1 ? 1 : (NQ <= 2 ? 2 : (NQ <= 4 ? 4 : 8));  // quads per row slot of B
  const int s = lane / NQ, q = lane - s * NQ;
  const bool active = lane < S * NQ;
  const f32x4* __restrict__ Bq = reinterpret_cast<const f32x4*>(a.B) + q;
#pragma unroll
  for (int op = 0; op < NOPS; ++op) acc[op] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (kb0 >= k1) return;
  const int64_t kend = (lane < CE) ? k1 : 0;  // lanes beyond the chunk hold no entry
  Chunk cur = fetch_chunk(a.S, kb0, k1, kend, lane);
  for (int64_t kb = kb0; kb < k1; kb += stride) {
    const int64_t left = k1 - kb;
    const int nsub = left >= CE ? T : (int)((left + S - 1) / S);
    f32x4 b[T][NOPS];
    float vv[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const int c = __shfl(cur.col, t * S + s, 64);
      vv[t] = __shfl(cur.v, t * S + s, 64);
      const f32x4* __restrict__ row = Bq + (size_t)c * (NOPS * G);
#pragma unroll
      for (int op = 0; op < NOPS; ++op) b[t][op] = (t < nsub && active) ? row[op * G] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (kb + stride < k1) cur = fetch_chunk(a.S, kb + stride, k1, kend, lane);  // in flight during the products
#pragma unroll
    for (int t = 0; t < T; ++t) {
#pragma unroll
      for (int op = 0; op < NOPS; ++op) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[op][e] = fmaf(vv[t], b[t][op][e], acc[op][e]);
      }
    }
  }
  // add the S lanes of each quad: halving tree over s, fixed order
  int cnt = S;
#pragma unroll
  for (int h = 32; h >= 1; h >>= 1) {
    if (h < cnt) {
      const bool take = s + h < cnt;
#pragma unroll
      for (int op = 0; op < NOPS; ++op) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float o = __shfl_down(acc[op][e], h * NQ, 64);
          acc[op][e] += take ? o : 0.f;
        }
      }
      cnt = h;
    }
  }
}

template <int NQ, int NOPS>
__global__ __launch_bounds__(kSpThreads) void spmm_kernel(const SpmmArgs a) {
  constexpr int G = 8;  // bound of NQ, for the LDS staging of long rows
  constexpr int CE = Shape64<NQ>::CE;
  using mfma_detail::f32x4;
  if (a.flag != nullptr && *a.flag == 0) return;
  __shared__ int long_rows[kMaxLong];
  __shared__ int nlong_sh;
  __shared__ float part[kMaxLong][kSpWaves][NOPS][G][4];
  const int r0 = a.win[blockIdx.x], r1 = a.win[blockIdx.x + 1];
  if (r1 <= r0) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ldo = a.ldo;

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

  // long rows: wave w takes chunks w, w + 4, ...; partial sums to LDS
  for (int sl = 0; sl < nlong; ++sl) {
    const RowSpan sp = row_span(a.S, long_rows[sl]);
    f32x4 acc[NOPS];
    row_sum<NQ, NOPS>(a, sp.k0 + CE * wave, sp.k1, CE * kSpWaves, lane, acc);
    if (lane < NQ) {
#pragma unroll
      for (int op = 0; op < NOPS; ++op) {
#pragma unroll
        for (int e = 0; e < 4; ++e) part[sl][wave][op][lane][e] = acc[op][e];
      }
    }
  }
  // short rows: one wave each
  for (int r = r0 + wave; r < r1; r += kSpWaves) {
    const RowSpan sp = row_span(a.S, r);
    if (sp.k1 - sp.k0 >= kLong) continue;
    f32x4 acc[NOPS];
    row_sum<NQ, NOPS>(a, sp.k0, sp.k1, CE, lane, acc);
    if (lane < NQ) {
      float* __restrict__ orow = a.out + (size_t)r * ldo;
#pragma unroll
      for (int op = 0; op < NOPS; ++op) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int c = 4 * lane + e;
          if (c < a.NC) orow[a.ooff + op * a.NC + c] = acc[op][e];
        }
      }
    }
  }
  if (nlong == 0) return;
  __syncthreads();
  constexpr int kPer = NOPS * G * 4;
  for (int t = threadIdx.x; t < nlong * kPer; t += kSpThreads) {
    const int sl = t / kPer, j = t - sl * kPer;
    const int op = j / (4 * G), c = j - op * (4 * G);
    const float* pj = &part[sl][0][0][0][0] + j;
    float sum = pj[0];
#pragma unroll
    for (int w = 1; w < kSpWaves; ++w) sum += pj[w * kPer];
    if (c < a.NC) a.out[(size_t)long_rows[sl] * ldo + a.ooff + op * a.NC + c] = sum;
  }
}

template <int NQ, int NOPS>
hipError_t launch_q(const SpmmArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((spmm_kernel<NQ, NOPS>), dim3(a.nwin), dim3(kSpThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace

// lanes (16-byte quads) per operand row: the smallest power of two that holds C-1 floats
int sparse_group(int NC) {
  const int nq = (NC + 3) >> 2;
  return nq <= 1 ? 1 : (nq <= 2 ? 2 : (nq <= 4 ? 4 : 8));
}

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
  const int G = sparse_group(NC);
  const int64_t total = rows * nops * G;
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s0, src1, rows, NC, G,
                     nops, dst, flag);
  return hipGetLastError();
}

hipError_t launch_spmm(const SpmmArgs& a, hipStream_t st) {
  // two operands only where both rows share a 128-byte line (C-1 <= 16); wider ones are multiplied one by one
  if (a.nq != (a.NC + 3) / 4 || a.nq < 1 || a.nq > 8 || a.nops < 1 || a.nops > (a.nq <= 4 ? 2 : 1)) return hipErrorInvalidValue;
  switch (a.nq * 2 + (a.nops - 1)) {
    case 2: return launch_q<1, 1>(a, st);
    case 3: return launch_q<1, 2>(a, st);
    case 4: return launch_q<2, 1>(a, st);
    case 5: return launch_q<2, 2>(a, st);
    case 6: return launch_q<3, 1>(a, st);
    case 7: return launch_q<3, 2>(a, st);
    case 8: return launch_q<4, 1>(a, st);
    case 9: return launch_q<4, 2>(a, st);
    case 10: return launch_q<5, 1>(a, st);
    case 12: return launch_q<6, 1>(a, st);
    case 14: return launch_q<7, 1>(a, st);
    case 16: return launch_q<8, 1>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nadmm
