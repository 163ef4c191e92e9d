// Column-sliced matrix-core path for wide data and for up to 32 free classes (gfx950).
//
// When the p x (C-1) operands and accumulators of a whole row no longer fit one compute unit
// (p > 960 or C-1 > 16), the columns are cut into slices of at most 24 steps of 32 columns and the
// Hessian-vector product of Section 2.6 (or the gradient A^T (P - Y)) is taken in two sweeps over A:
//   sweep 1  every workgroup owns a range of rows and takes the slices in turn: the slice's share of the
//            logits Z|W = A[:, slice] [X|V][slice, :] with bf16-split MFMAs is added to the rows' logits,
//            which stay in LDS (the range is chosen so that they fit); after the last slice the
//            workgroup finishes its rows: P, D, the row losses (nadmm_rows16.h);
//   sweep 2  every workgroup forms out^T[:, slice] += D^T A[:, slice] for its row range; the tile is
//            transposed through a wave-private swizzled LDS copy; no workgroup barrier is needed.
// Operand layouts, the bf16 high/low split and the three-term product are those of the fused kernel.
#include "nadmm_internal.h"
#include "nadmm_mfma.h"
#include "nadmm_rows16.h"

namespace nadmm {
namespace {

using namespace mfma_detail;

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kTileRows = 32;
constexpr int kStepCols = 32;
constexpr int kSliceSteps = 24;   // at most 3 steps per wave
constexpr int kStepBytes = 4096;
constexpr size_t kLogitLdsBytes = 159 * 1024;  // sweep 1: K-split partials + the logits of the workgroup's rows

struct SlicedArgs {
  RowArgs r;
  int32_t nslices;            // column slices
  int32_t logit_rows_per_wg;  // sweep 1: rows per workgroup (their logits fit the LDS)
  int32_t logit_tile_rows;    // sweep 1: rows per tile, <= 32: the range is cut into equal tiles, so that no workgroup ends on
                              //   a tile of a few rows that costs as much as a full one
  const float* rows_in;  // sweep 2 in:  [n][NC]
  float* partial;        // sweep 2 out: [row group][p*NC]
  int32_t steps_total;   // ceil(p / 32)
  int32_t steps_q;       // slice s holds steps_q + (s < steps_r) steps, starting at s steps_q + min(s, steps_r)
  int32_t steps_r;
  int32_t steps_max;     // steps of the largest slice
  int32_t rows_per_wg;
  int32_t sync_tiles;    // sweep 2: keep the waves of a workgroup within one tile of each other
};

// Steps of one wave inside its slice: the slice's steps are dealt out in contiguous, balanced runs,
// wave w owning steps [w nsteps / 8, (w+1) nsteps / 8).  Every wave then holds at least
// ceil(steps_max / 8) - 1 steps, so only the last of a wave's SPW step slots is conditional, and a
// row's bytes are shared between neighbouring waves at one place only (rows need not start on a
// cache line).
struct WaveSteps {
  int step0;   // first step of this wave, counted over the whole matrix
  int local0;  // the same, counted inside the slice
  int count;
};
__device__ __forceinline__ WaveSteps wave_steps(const SlicedArgs& sa, int slice, int wave) {
  const int nsteps = sa.steps_q + (slice < sa.steps_r ? 1 : 0);
  const int first = slice * sa.steps_q + (slice < sa.steps_r ? slice : sa.steps_r);
  const int b0 = (wave * nsteps) >> 3, b1 = ((wave + 1) * nsteps) >> 3;
  return WaveSteps{first + b0, b0, b1 - b0};
}

// Loads of one step (2 row blocks x 8 columns per lane), addresses clamped into the matrix.
// ANY: rows need not start on 16-byte boundaries; col_max is then p - 4, the last piece that lies inside a row.
template <bool ANY>
__device__ __forceinline__ void load_step_regs(const RowArgs& a, float4 (&pf)[2][2], int64_t row0, int64_t r_end,
                                               int col, int col_max, int m) {
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    int64_t row = row0 + m + 16 * rb;
    row = row < r_end ? row : r_end - 1;
    const float* src = a.A + row * a.lda;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c0 = col + 4 * h;
      const float* at = src + (c0 < col_max ? c0 : col_max);
      if constexpr (ANY) {
        const Quad q = *reinterpret_cast<const Quad*>(at);
        pf[rb][h] = float4{q.x, q.y, q.z, q.w};
      } else {
        pf[rb][h] = *reinterpret_cast<const float4*>(at);
      }
    }
  }
}

// Registers of one step -> bf16 high/low operands of both row blocks (and, if THREE, the third parts
// that the full-accuracy logit product needs); columns past p are zeroed.
template <bool THREE, bool ANY>
__device__ __forceinline__ void convert_step(const float4 (&pf)[2][2], int col, int col_max, int p, bool ragged,
                                             u32x4 (&ahi)[2], u32x4 (&alo)[2], u32x4 (&alo2)[2]) {
  float av[2][8];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    av[rb][0] = pf[rb][0].x; av[rb][1] = pf[rb][0].y; av[rb][2] = pf[rb][0].z; av[rb][3] = pf[rb][0].w;
    av[rb][4] = pf[rb][1].x; av[rb][5] = pf[rb][1].y; av[rb][6] = pf[rb][1].z; av[rb][7] = pf[rb][1].w;
  }
  if (ragged) {  // uniform branch: only the step that contains column p
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c0 = col + 4 * h;
      if constexpr (ANY) {
        // a piece fetched from column p - 4 holds its columns `shift` places further up; what lies past p is zero
        const int shift = c0 - (c0 < col_max ? c0 : col_max);  // 0: the piece is its own; >= 4: all of it is past p
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const float q0 = av[rb][4 * h], q1 = av[rb][4 * h + 1], q2 = av[rb][4 * h + 2], q3 = av[rb][4 * h + 3];
          av[rb][4 * h + 0] = shift == 0 ? q0 : (shift == 1 ? q1 : (shift == 2 ? q2 : (shift == 3 ? q3 : 0.f)));
          av[rb][4 * h + 1] = shift == 0 ? q1 : (shift == 1 ? q2 : (shift == 2 ? q3 : 0.f));
          av[rb][4 * h + 2] = shift == 0 ? q2 : (shift == 1 ? q3 : 0.f);
          av[rb][4 * h + 3] = shift == 0 ? q3 : 0.f;
        }
      } else {
        const int nv = c0 <= col_max ? p - c0 : 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          av[0][4 * h + e] = e < nv ? av[0][4 * h + e] : 0.f;
          av[1][4 * h + e] = e < nv ? av[1][4 * h + e] : 0.f;
        }
      }
    }
  }
  if (THREE) {
    split8_3(av[0], ahi[0], alo[0], alo2[0]);
    split8_3(av[1], ahi[1], alo[1], alo2[1]);
  } else {
    split8(av[0], ahi[0], alo[0]);
    split8(av[1], ahi[1], alo[1]);
  }
}

// ------------------------------------------------------------------------------------------------
// sweep 1 and the rows stage: a workgroup owns a range of rows and keeps their logits in LDS
// ------------------------------------------------------------------------------------------------
// LDS: the K-split partials of one tile, [wave][quad (matrix, class block, row block)][component][lane], then the
// logits of the workgroup's rows, [local row][matrix][class].
template <int NB, int MATS>
constexpr size_t logits_part_floats() { return (size_t)kWaves * (MATS * NB * 2) * 4 * 64; }

template <int SPW, int NB, bool HAS0, bool HAS1, bool ANY>
__global__ __launch_bounds__(kThreads) void slice_logits_kernel(const SlicedArgs sa) {
  const RowArgs& a = sa.r;
  if (a.flag != nullptr && *a.flag == 0) return;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int kMats = (HAS0 ? 1 : 0) + (HAS1 ? 1 : 0);
  constexpr int kQuads = kMats * NB * 2;
  constexpr int kMatW = HAS0 ? 1 : 0;  // index of W among the matrices held
  float* part = reinterpret_cast<float*>(lds);
  float* zres = part + logits_part_floats<NB, kMats>();
  // kWaves doubles behind the logits (a multiple of 32 rows, so 8-byte aligned) for the sum of the row losses: the kernel
  // has no static LDS, its whole allowance is dynamic
  const size_t alloc_rows = ((size_t)sa.logit_rows_per_wg + kTileRows - 1) / kTileRows * kTileRows;
  double* red = reinterpret_cast<double*>(zres + alloc_rows * kMats * a.NC);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kg = lane >> 4;
  const int NC = a.NC, p = a.p;
  const int col_max = ANY ? p - 4 : ((p + 3) & ~3) - 4;  // no load goes past element 4 ceil(p/4) of a row (ANY: past column p - 1)

  const int64_t r_begin = (int64_t)blockIdx.x * sa.logit_rows_per_wg;
  int64_t r_end = r_begin + sa.logit_rows_per_wg;
  if (r_end > a.n) r_end = a.n;
  if (r_begin >= r_end) return;

  // Workgroup b takes the slices in the order b, b + 1, ... (mod their number): when the sweep ends, the part of the matrix
  // that the memory-side cache still holds is spread evenly over the slices, and so over the workgroups of sweep 2.
  auto slice_at = [&](int k) { return (int)((blockIdx.x + (unsigned)k) % (unsigned)sa.nslices); };
  // rows of a tile past its end are not fetched: the loads repeat the tile's last row, and what is computed from them is dropped
  const int th = sa.logit_tile_rows;
  auto tile_end = [&](int64_t row0) { return row0 + th < r_end ? row0 + th : r_end; };
  float4 pf[SPW][2][2];
  {  // first tile of the first slice
    const WaveSteps w0 = wave_steps(sa, slice_at(0), wave);
#pragma unroll
    for (int i = 0; i < SPW; ++i)
      if (i < SPW - 1 || i < w0.count)
        load_step_regs<ANY>(a, pf[i], r_begin, tile_end(r_begin), kStepCols * (w0.step0 + i) + 8 * kg, col_max, m);
  }

  // Entries of X and V of one slice's steps as they lie in memory (indices clamped into the arrays; what does not
  // exist is zeroed when the operands are formed).  Where the registers allow it, those of the next slice are
  // requested during the last tile of the current one.
  constexpr bool kOperandsAhead = kMats * NB * SPW * 8 <= 24;
  float raw_x[HAS0 ? SPW : 1][NB][8], raw_v[HAS1 ? SPW : 1][NB][8];
  auto fetch_operands = [&](const WaveSteps& w) {
#pragma unroll
    for (int i = 0; i < SPW; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int cls = 16 * nb + m;
        const int clc = cls < NC ? cls : NC - 1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int j = kStepCols * (w.step0 + i) + 8 * kg + e;
          const size_t idx = (size_t)(j < p ? j : p - 1) * NC + clc;
          if (HAS0) raw_x[i][nb][e] = a.B0[idx];
          if (HAS1) raw_v[i][nb][e] = a.B1[idx];
        }
      }
  };
  if (kOperandsAhead) fetch_operands(wave_steps(sa, slice_at(0), wave));

  for (int sk = 0; sk < sa.nslices; ++sk) {
    const WaveSteps ws = wave_steps(sa, slice_at(sk), wave);
    // the steps of this wave in the slice after this one (none after the last): their first tile is requested
    // while the last tile of this slice is being multiplied
    const bool more = sk + 1 < sa.nslices;
    const WaveSteps wn = more ? wave_steps(sa, slice_at(sk + 1), wave) : WaveSteps{0, 0, 0};
    auto step_exists = [&](int i) { return i < SPW - 1 || i < ws.count; };
    auto col_of = [&](int i) { return kStepCols * (ws.step0 + i) + 8 * kg; };

    // operands [X|V] of this wave's steps: hi / lo, per class block; X in three parts (full-accuracy logits)
    if (!kOperandsAhead) fetch_operands(ws);
    u32x4 bx_hi[SPW][NB], bx_lo[SPW][NB], bx_lo2[SPW][NB], bv_hi[SPW][NB], bv_lo[SPW][NB];
#pragma unroll
    for (int i = 0; i < SPW; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const bool cvn = 16 * nb + m < NC;
        float x[8], v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const bool ok = cvn && col_of(i) + e < p && i < ws.count;
          x[e] = (HAS0 && ok) ? raw_x[i][nb][e] : 0.f;
          v[e] = (HAS1 && ok) ? raw_v[i][nb][e] : 0.f;
        }
        split8_3(x, bx_hi[i][nb], bx_lo[i][nb], bx_lo2[i][nb]);
        split8(v, bv_hi[i][nb], bv_lo[i][nb]);
      }

    for (int64_t row0 = r_begin; row0 < r_end; row0 += th) {
      // the tile fetched ahead: the next one of this slice, or the first one of the next slice (one place of issue
      // for both, so that the addresses are formed where they are used and not kept for the whole slice)
      const bool last_tile = row0 + th >= r_end;
      const int64_t next_row0 = last_tile ? r_begin : row0 + th;
      const int next_step0 = last_tile ? wn.step0 : ws.step0;
      const int next_count = last_tile ? wn.count : ws.count;
      const bool next_any = !last_tile || more;
      f32x4 accZ[NB][2], accW[NB][2];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        accZ[nb][0] = accZ[nb][1] = accW[nb][0] = accW[nb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int i = 0; i < SPW; ++i) {
        const bool here = step_exists(i);
        u32x4 ahi[2], alo[2], alo2[2];
        if (here)
          convert_step<HAS0, ANY>(pf[i], col_of(i), col_max, p, kStepCols * (ws.step0 + i + 1) > p, ahi, alo, alo2);
        if (next_any && (i < SPW - 1 || i < next_count))
          load_step_regs<ANY>(a, pf[i], next_row0, tile_end(next_row0), kStepCols * (next_step0 + i) + 8 * kg, col_max, m);
        if (kOperandsAhead && i == SPW - 1 && last_tile && more) fetch_operands(wn);
        if (here) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
              if (HAS0)
                accZ[nb][rb] = mfma6(ahi[rb], alo[rb], alo2[rb], bx_hi[i][nb], bx_lo[i][nb], bx_lo2[i][nb], accZ[nb][rb]);
              if (HAS1) accW[nb][rb] = mfma3(ahi[rb], alo[rb], bv_hi[i][nb], bv_lo[i][nb], accW[nb][rb]);
            }
        }
      }
      // K-split partials: quad index = (mat * NB + nb) * 2 + rb
      {
        float* pw = part + (size_t)(wave * kQuads * 4) * 64 + lane;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (HAS0) pw[(((0 * NB + nb) * 2 + rb) * 4 + e) * 64] = accZ[nb][rb][e];
              if (HAS1) pw[(((kMatW * NB + nb) * 2 + rb) * 4 + e) * 64] = accW[nb][rb][e];
            }
      }
      __syncthreads();
      // wave e adds the 8 partials of rows row0 + 4 kg + (e & 3) + 16 (e >> 2) and adds the sum to the rows' logits
      // (the slices in the order this workgroup takes them)
      {
        const int rb = wave >> 2, comp = wave & 3;
        const int r_tile = 4 * kg + comp + 16 * rb;
        const int r_local = (int)(row0 - r_begin) + r_tile;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int cls = 16 * nb + m;
          float z = 0.f, w = 0.f;
#pragma unroll
          for (int sw = 0; sw < kWaves; ++sw) {
            const float* pr = part + (size_t)(sw * kQuads * 4) * 64 + lane;
            if (HAS0) z += pr[(((0 * NB + nb) * 2 + rb) * 4 + comp) * 64];
            if (HAS1) w += pr[(((kMatW * NB + nb) * 2 + rb) * 4 + comp) * 64];
          }
          if (cls < NC && r_tile < th) {
            float* zr = zres + (size_t)(r_local * kMats) * NC + cls;
            if (HAS0) zr[0] = sk == 0 ? z : zr[0] + z;
            if (HAS1) zr[kMatW * NC] = sk == 0 ? w : zr[kMatW * NC] + w;
          }
        }
      }
      __syncthreads();
    }
  }

  // rows stage: lane (g, m) of wave v finishes row 32 pass + 4 v + g of the range.  Nothing overlaps this stage, so the
  // memory round trips in it are kept few: the cached probabilities and labels of several passes are requested together.
  const rows16::LaneClasses<NB> lc(m, NC);
  const bool with_loss = a.kind == kRowsGrad || a.kind == kRowsLoss;
  const bool use_pin = !HAS0 && a.kind == kRowsHv;
  constexpr int RG = NB == 1 ? 8 : 4;  // passes per group
  double ell = 0.0;
  for (int64_t g0 = r_begin; g0 < r_end; g0 += 4 * kWaves * RG) {
    float pin[RG][NB];
    int label[RG];
#pragma unroll
    for (int u = 0; u < RG; ++u) {
      const int64_t row = g0 + 4 * kWaves * u + 4 * wave + kg;
      const int64_t rowc = row < r_end ? row : r_end - 1;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) pin[u][nb] = use_pin ? a.Pin[(size_t)rowc * NC + lc.cl[nb]] : 0.f;
      label[u] = with_loss ? a.labels[rowc] : 0;
    }
#pragma unroll
    for (int u = 0; u < RG; ++u) {
      if (g0 + 4 * kWaves * u < r_end) {  // uniform
        const int64_t row = g0 + 4 * kWaves * u + 4 * wave + kg;
        const int64_t rowc = row < r_end ? row : r_end - 1;
        const float* zr = zres + (size_t)((int)(rowc - r_begin) * kMats) * NC;
        float z[NB], w[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          z[nb] = HAS0 ? zr[lc.cl[nb]] : 0.f;
          w[nb] = HAS1 ? zr[kMatW * NC + lc.cl[nb]] : 0.f;
        }
        // rows past the range belong to another workgroup (or do not exist): a row index of n marks them invalid
        ell += rows16::finish<NB>(a, row < r_end ? row : a.n, m, lc, HAS0, HAS1, z, w, pin[u], label[u]);
      }
    }
  }
  if (!with_loss) return;
  ell = mfma_detail::wave64_sum(ell);
  if (lane == 0) red[wave] = ell;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int wv = 0; wv < kWaves; ++wv) t += red[wv];
    a.loss_part[blockIdx.x] = t;
  }
}

// ------------------------------------------------------------------------------------------------
// sweep 2: out^T[:, slice] += D^T A[:, slice]
// ------------------------------------------------------------------------------------------------
template <int SPW, int NB, bool ANY>
__global__ __launch_bounds__(kThreads) void slice_cols_kernel(const SlicedArgs sa) {
  const RowArgs& a = sa.r;
  if (a.flag != nullptr && *a.flag == 0) return;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  char* cm = lds;  // steps_max x 4 KB, every step slot used by the one wave that owns the step

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kg = lane >> 4;
  const int NC = a.NC, p = a.p;
  const int slice = blockIdx.x;
  const WaveSteps ws = wave_steps(sa, slice, wave);
  const int col_max = ANY ? p - 4 : ((p + 3) & ~3) - 4;  // no load goes past element 4 ceil(p/4) of a row (ANY: past column p - 1)

  const int64_t r_begin = (int64_t)blockIdx.y * sa.rows_per_wg;
  int64_t r_end = r_begin + sa.rows_per_wg;
  if (r_end > a.n) r_end = a.n;

  auto step_exists = [&](int i) { return i < SPW - 1 || i < ws.count; };
  auto col_of = [&](int i) { return kStepCols * (ws.step0 + i) + 8 * kg; };

  f32x4 acc2[SPW][2][NB];
#pragma unroll
  for (int i = 0; i < SPW; ++i)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc2[i][h][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // D entries of this lane: class 16 nb + m, rows row0 + 4 kg + (e & 3) + 16 (e >> 2), e = 0..7
  float dn[NB][8];
  auto load_d = [&](int64_t row0) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int cls = 16 * nb + m;
      const int clc = cls < NC ? cls : NC - 1;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int64_t row = row0 + 4 * kg + (e & 3) + ((e >> 2) << 4);
        row = row < r_end ? row : r_end - 1;
        dn[nb][e] = sa.rows_in[(size_t)row * NC + clc];
      }
    }
  };

  // The row range is walked from its last tile to its first: sweep 1 went forward over the same range, so the part of
  // the matrix it read last is what the memory-side cache still holds (the matrix is larger than that cache), and the
  // next forward sweep finds the first part there in turn.
  const int64_t ntiles = r_begin < r_end ? (r_end - r_begin + kTileRows - 1) / kTileRows : 0;
  const int64_t r_last = r_begin + (ntiles - 1) * kTileRows;  // first row of the last tile
  float4 pf[SPW][2][2];
  if (ntiles > 0) {
#pragma unroll
    for (int i = 0; i < SPW; ++i)
      if (step_exists(i)) load_step_regs<ANY>(a, pf[i], r_last, r_end, col_of(i), col_max, m);
    load_d(r_last);
  }

  for (int64_t row0 = r_last; row0 >= r_begin; row0 -= kTileRows) {
    const int64_t row_next = row0 > r_begin ? row0 - kTileRows : r_begin;  // the tile fetched ahead (the first one again at the end)
    // this tile's D operand (rows past the range and padded classes contribute nothing)
    u32x4 dhi[NB], dlo[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const bool cvn = 16 * nb + m < NC;
      unsigned h[4], l[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool v0 = cvn && row0 + 4 * kg + e < r_end;
        const bool v1 = cvn && row0 + 16 + 4 * kg + e < r_end;
        const float d0 = v0 ? dn[nb][e] : 0.f, d1 = v1 ? dn[nb][4 + e] : 0.f;
        h[e] = pack2(d0, d1);
        l[e] = pack2(d0 - low_as_float(h[e]), d1 - high_as_float(h[e]));
      }
      dhi[nb] = u32x4{h[0], h[1], h[2], h[3]};
      dlo[nb] = u32x4{l[0], l[1], l[2], l[3]};
    }
    load_d(row_next);  // next tile's D

#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      if (step_exists(i)) {
        const int col = col_of(i);
        const int sl = ws.local0 + i;  // step inside the slice
        u32x4 ahi[2], alo[2], unused[2];
        convert_step<false, ANY>(pf[i], col, col_max, p, kStepCols * (ws.step0 + i + 1) > p, ahi, alo, unused);
        load_step_regs<ANY>(a, pf[i], row_next, r_end, col, col_max, m);
        char* base = cm + (size_t)sl * kStepBytes;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
          const unsigned hp = __builtin_amdgcn_perm(ahi[1][c >> 1], ahi[0][c >> 1], sel);
          const unsigned lp = __builtin_amdgcn_perm(alo[1][c >> 1], alo[0][c >> 1], sel);
          const int off = cm_offset(8 * kg + c, m >> 2) + ((m & 3) << 2);
          *reinterpret_cast<unsigned*>(base + off) = hp;
          *reinterpret_cast<unsigned*>(base + 2048 + off) = lp;
        }
        // LDS operations of one wave execute in order: the copy just written is read back transposed
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int off = cm_offset(16 * h + m, kg);
          const u32x4 thi = *reinterpret_cast<const u32x4*>(base + off);
          const u32x4 tlo = *reinterpret_cast<const u32x4*>(base + 2048 + off);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc2[i][h][nb] = mfma3(dhi[nb], dlo[nb], thi, tlo, acc2[i][h][nb]);
        }
      }
    }
    // Rows that do not start on a cache line share lines between neighbouring waves: waves that
    // drift apart would fetch such lines from memory twice.
    if (sa.sync_tiles) __builtin_amdgcn_s_barrier();
  }

  float* out = sa.partial + (size_t)blockIdx.y * ((size_t)p * NC);
#pragma unroll
  for (int i = 0; i < SPW; ++i) {
    if (i < ws.count) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int j = kStepCols * (ws.step0 + i) + 16 * h + m;
        if (j < p) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int c = 16 * nb + 4 * kg + e;
              if (c < NC) out[(size_t)j * NC + c] = acc2[i][h][nb][e];
            }
        }
      }
    }
  }
}

bool rows_16_byte_aligned(const RowArgs& a) { return (a.lda & 3) == 0 && (reinterpret_cast<uintptr_t>(a.A) & 15) == 0; }

template <int SPW, int NB, bool HAS0, bool HAS1, bool ANY>
hipError_t launch_logits_a(const SlicedArgs& sa, dim3 grid, hipStream_t st) {
  constexpr int kMats = (HAS0 ? 1 : 0) + (HAS1 ? 1 : 0);
  const size_t alloc_rows = ((size_t)sa.logit_rows_per_wg + kTileRows - 1) / kTileRows * kTileRows;
  const size_t lds = (logits_part_floats<NB, kMats>() + alloc_rows * kMats * sa.r.NC) * sizeof(float) + kWaves * sizeof(double);
  if (lds > kLogitLdsBytes) return hipErrorInvalidValue;
  static uint64_t lds_set = 0;  // per device
  hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(&slice_logits_kernel<SPW, NB, HAS0, HAS1, ANY>), &lds_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((slice_logits_kernel<SPW, NB, HAS0, HAS1, ANY>), grid, dim3(kThreads), lds, st, sa);
  return hipGetLastError();
}

template <int SPW, int NB, bool HAS0, bool HAS1>
hipError_t launch_logits_t(const SlicedArgs& sa, dim3 grid, hipStream_t st) {
  if (rows_16_byte_aligned(sa.r)) return launch_logits_a<SPW, NB, HAS0, HAS1, false>(sa, grid, st);
  return launch_logits_a<SPW, NB, HAS0, HAS1, true>(sa, grid, st);
}

template <int SPW, int NB>
hipError_t launch_logits_nb(const SlicedArgs& sa, dim3 grid, hipStream_t st) {
  const bool h0 = sa.r.B0 != nullptr, h1 = sa.r.B1 != nullptr;
  if (h0 && h1) return launch_logits_t<SPW, NB, true, true>(sa, grid, st);
  if (h1) return launch_logits_t<SPW, NB, false, true>(sa, grid, st);
  if (h0) return launch_logits_t<SPW, NB, true, false>(sa, grid, st);
  return hipErrorInvalidValue;
}

template <int SPW, int NB, bool ANY>
hipError_t launch_cols_a(const SlicedArgs& sa, dim3 grid, hipStream_t st) {
  const size_t lds = (size_t)sa.steps_max * kStepBytes;
  static uint64_t lds_set = 0;  // per device
  hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(&slice_cols_kernel<SPW, NB, ANY>), &lds_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((slice_cols_kernel<SPW, NB, ANY>), grid, dim3(kThreads), lds, st, sa);
  return hipGetLastError();
}

template <int SPW, int NB>
hipError_t launch_cols_t(const SlicedArgs& sa, dim3 grid, hipStream_t st) {
  if (rows_16_byte_aligned(sa.r)) return launch_cols_a<SPW, NB, false>(sa, grid, st);
  return launch_cols_a<SPW, NB, true>(sa, grid, st);
}

}  // namespace

bool sliced_supported(const Shape& s, int64_t lda, const void* A) {
  if (s.NC > 32) return false;
  if ((reinterpret_cast<uintptr_t>(A) & 3) != 0 || lda < s.p) return false;
  if (((lda & 3) != 0 || (reinterpret_cast<uintptr_t>(A) & 15) != 0) && s.p < 4) return false;  // whole 16-byte pieces inside a row
  return true;
}

// One workgroup per compute unit: (column slices) x (row groups) = at most 256 workgroups; both sweeps use
// the same plan.  (Finer slices or two workgroups per compute unit in sweep 1 measured no faster.)
void sliced_grid(const Shape& s, int* nslices, int* steps_per_slice, int* row_groups) {
  const int steps = (s.p + kStepCols - 1) / kStepCols;
  const int S = (steps + kSliceSteps - 1) / kSliceSteps;
  const int64_t tiles = (s.n + kTileRows - 1) / kTileRows;
  int64_t rg = 256 / S;
  if (rg < 1) rg = 1;
  if (rg > tiles) rg = tiles;
  *nslices = S;
  *steps_per_slice = (steps + S - 1) / S;  // the largest slice; slices differ by at most one step
  *row_groups = (int)rg;
}

// Sweep 1: the fewest row ranges, in multiples of 256 workgroups, whose logits (mats matrices of C-1 columns) fit the
// LDS beside the K-split partials of a tile.
void sliced_logit_plan(const Shape& s, int mats, int* groups, int* rows_per_wg) {
  const int nb = s.NC > 16 ? 2 : 1;
  const size_t part = (size_t)kWaves * (mats * nb * 2) * 4 * 64 * sizeof(float);
  const size_t room = kLogitLdsBytes - part - kWaves * sizeof(double);
  const int64_t tiles = (s.n + kTileRows - 1) / kTileRows;
  int64_t rows = kTileRows;
  for (int64_t k = 1;; ++k) {
    int64_t g = 256 * k;
    if (g > tiles) g = tiles;
    if (g < 1) g = 1;
    rows = (s.n + g - 1) / g;
    if (rows < 1) rows = 1;
    const size_t alloc = (size_t)((rows + kTileRows - 1) / kTileRows * kTileRows);
    if (alloc * mats * s.NC * sizeof(float) <= room || g == tiles || tiles == 0) break;  // one tile always fits
  }
  *rows_per_wg = (int)rows;
  *groups = (int)((s.n + rows - 1) / rows > 0 ? (s.n + rows - 1) / rows : 1);
}

int sliced_loss_blocks(const Shape& s) {
  int g, r;
  sliced_logit_plan(s, 1, &g, &r);  // the calls with a loss have the operand X alone
  return g;
}

static SlicedArgs make_args(const RowArgs& a, int S, int sps, int rg) {
  SlicedArgs sa;
  sa.r = a;
  sa.nslices = S;
  sa.logit_rows_per_wg = 0;
  sa.logit_tile_rows = kTileRows;
  sa.rows_in = nullptr;
  sa.partial = nullptr;
  sa.steps_total = (a.p + kStepCols - 1) / kStepCols;
  sa.steps_q = sa.steps_total / S;
  sa.steps_r = sa.steps_total % S;
  sa.steps_max = sps;
  sa.rows_per_wg = (int32_t)((a.n + rg - 1) / rg);
  sa.sync_tiles = ((a.lda * sizeof(float)) % 128 != 0 || (reinterpret_cast<uintptr_t>(a.A) & 127) != 0) ? 1 : 0;
  return sa;
}

hipError_t launch_sliced_logits(const RowArgs& a, hipStream_t st) {
  Shape s{a.n, a.p, a.NC, (int64_t)a.p * a.NC};
  int S, sps, rg;
  sliced_grid(s, &S, &sps, &rg);
  SlicedArgs sa = make_args(a, S, sps, rg);
  const int mats = (a.B0 != nullptr ? 1 : 0) + (a.B1 != nullptr ? 1 : 0);
  if (mats == 0) return hipErrorInvalidValue;
  if ((a.kind == kRowsGrad || a.kind == kRowsLoss) && mats != 1) return hipErrorInvalidValue;  // see sliced_loss_blocks
  int groups = 0, rows = 0;
  sliced_logit_plan(s, mats, &groups, &rows);
  sa.logit_rows_per_wg = rows;
  const int tiles_per_wg = (rows + kTileRows - 1) / kTileRows;
  sa.logit_tile_rows = (rows + tiles_per_wg - 1) / tiles_per_wg;
  const dim3 grid(groups);
  const int spw = (sps + kWaves - 1) / kWaves;
  const int nb = a.NC > 16 ? 2 : 1;
  if (nb == 1) {
    switch (spw) {
      case 1: return launch_logits_nb<1, 1>(sa, grid, st);
      case 2: return launch_logits_nb<2, 1>(sa, grid, st);
      case 3: return launch_logits_nb<3, 1>(sa, grid, st);
    }
  } else {
    switch (spw) {
      case 1: return launch_logits_nb<1, 2>(sa, grid, st);
      case 2: return launch_logits_nb<2, 2>(sa, grid, st);
      case 3: return launch_logits_nb<3, 2>(sa, grid, st);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t launch_sliced_cols(const RowArgs& a, const float* rows_in, float* partial, hipStream_t st) {
  Shape s{a.n, a.p, a.NC, (int64_t)a.p * a.NC};
  int S, sps, rg;
  sliced_grid(s, &S, &sps, &rg);
  SlicedArgs sa = make_args(a, S, sps, rg);
  sa.rows_in = rows_in;
  sa.partial = partial;
  const dim3 grid(S, rg);
  const int spw = (sps + kWaves - 1) / kWaves;
  const int nb = a.NC > 16 ? 2 : 1;
  if (nb == 1) {
    switch (spw) {
      case 1: return launch_cols_t<1, 1>(sa, grid, st);
      case 2: return launch_cols_t<2, 1>(sa, grid, st);
      case 3: return launch_cols_t<3, 1>(sa, grid, st);
    }
  } else {
    switch (spw) {
      case 1: return launch_cols_t<1, 2>(sa, grid, st);
      case 2: return launch_cols_t<2, 2>(sa, grid, st);
      case 3: return launch_cols_t<3, 2>(sa, grid, st);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace nadmm
