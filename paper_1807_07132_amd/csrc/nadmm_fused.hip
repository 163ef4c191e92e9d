// Fused single-pass kernel for gfx950: rows pass and transpose product in one
// sweep over A (Section 2.6: H v = A^T D with D formed row by row from W = A V
// and the probabilities P; same structure for the gradient A^T (P - Y)).
//
// One persistent workgroup of 8 waves per compute unit owns a contiguous range
// of rows and walks it in tiles of 32 rows.  Columns are cut into steps of 32;
// wave w owns steps w, w+8, ... in BOTH contractions:
//   phase 1  Z|W tile (32 x 2*16) = A_tile [X|V]   -- A straight from global
//            loads in MFMA A-operand layout, [X|V] resident in registers;
//   rows     cross-wave sum of the K-split partials through LDS; wave e forms the
//            log-sum-exp / probabilities / D of 4 of the 32 rows with 16-lane DPP
//            reductions and hands its D entries to the others through LDS;
//   phase 2  out^T (16 x cols) += D^T A_tile        -- A re-read from a
//            wave-private, bank-swizzled LDS copy written in phase 1.
// A is read from HBM exactly once; the p x (C-1) accumulators stay in registers
// for the whole row range and are written once as a per-workgroup partial.
//
// Arithmetic: every fp32 operand is split into bf16 high and low parts
// (x = hi + lo + O(2^-18 |x|)), and each product uses the three MFMA terms
// hi*hi + hi*lo + lo*hi with fp32 accumulation (v_mfma_f32_16x16x32_bf16).
#include "nadmm_internal.h"
#include "nadmm_cgstep.h"
#include "nadmm_mfma.h"

namespace nadmm {
namespace {

using namespace mfma_detail;

__device__ __forceinline__ void tile_barrier() { __syncthreads(); }

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kTileRows = 32;
constexpr int kStepCols = 32;
constexpr int kMaxSteps = 30;                 // LDS: steps * 4 KB + 36 KB <= 160 KB
constexpr int kStepBytes = 4096;              // hi plane 2 KB + lo plane 2 KB
constexpr int kPartBytes = kWaves * 4 * 64 * 16;
constexpr int kSumBytes = 8 * 64 * 4;    // exchange buffer of the rows stage

struct FusedArgs {
  RowArgs r;
  float* partial;     // gridDim.x x (p*NC) or NULL (no transpose product)
  int32_t steps;      // ceil(p / 32)
  int32_t rows_per_wg;
  CgPend cg;          // cg.st != NULL: the operand B1 is the result of a pending CG update (kernels without B0 only)
};

// HALFQ: the vectors of a pending CG update fit SPW quads per thread (half the capacity): the update then carries
// no surplus work (a wave issues one instruction per four cycles or so, and every workgroup repeats the update).
// ANYSTRIDE: rows of A need not start on 16-byte boundaries (any row stride, A 4-byte aligned): the 16-byte pieces are
// loaded as such, and the last piece of a row is fetched from column p - 4 and shifted into place, so that no load goes
// past a row's column p - 1.  (A variant of its own: the shifting costs the aligned kernel registers it does not have.)
template <int SPW, int KIND, bool HAS0, bool HAS1, bool STORES, bool HALFQ = false, bool ANYSTRIDE = false>
__global__ __launch_bounds__(kThreads) void fused_kernel(const FusedArgs fa) {
  const RowArgs& a = fa.r;
  if (a.flag != nullptr && *a.flag == 0) return;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int steps = fa.steps;
  char* cm = lds;                                                  // steps x 4 KB, every step slot private to the wave that owns the step
  float* part = reinterpret_cast<float*>(lds + (size_t)steps * kStepBytes);  // [wave][quad][comp][lane]
  float* dbuf = part + kPartBytes / 4;                             // [e][lane]

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // The slots of one wave's steps (s = wave, wave + 8, ...) lie back to back, so that the slot of step slot i is a
  // compile-time offset from one per-wave base and needs no address arithmetic per tile.
  char* cmw = cm + (size_t)(wave * (steps >> 3) + (wave < (steps & 7) ? wave : (steps & 7))) * kStepBytes;
  const int m = lane & 15;   // phase 1: row within the row block; rows stage / phase 2: class or column
  const int kg = lane >> 4;  // k-group of the MFMA operands
  const int NC = a.NC;
  const int p = a.p;
  constexpr bool has0 = HAS0;
  constexpr bool has1 = HAS1;
  constexpr bool with_cols = KIND == kRowsHv || KIND == kRowsGrad;
  const bool cv = m < NC;  // this lane's class is a real one
  const int mc = cv ? m : NC - 1;

  f32x4 acc2[SPW][2];
#pragma unroll
  for (int i = 0; i < SPW; ++i) {
    acc2[i][0] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc2[i][1] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  double loss_acc = 0.0;

  const int64_t r_begin = (int64_t)blockIdx.x * fa.rows_per_wg;
  int64_t r_end = r_begin + fa.rows_per_wg;
  if (r_end > a.n) r_end = a.n;
  // last column offset a 16-byte piece is fetched from.  Aligned rows: the last aligned piece that holds a column of A (no
  // load goes past element 4 ceil(p/4) of a row, <= lda); ANYSTRIDE: the last piece that lies inside the row
  const int col_max = ANYSTRIDE ? p - 4 : ((p + 3) & ~3) - 4;

  // ---- prefetch registers: [step][row block][half of the 8 columns] ----
  // Addresses are clamped into the matrix, so the loads need no branches; rows
  // past the range and columns past p are zeroed when the registers are used.
  float4 pf[SPW][2][2];
  // Steps i < SPW-1 exist for every wave (steps > 8 (SPW-1)); only the last one is conditional.
  auto step_exists = [&](int i) { return i < SPW - 1 || wave + kWaves * i < steps; };
  auto load_step = [&](int i, int64_t row0) {
    const int col = kStepCols * (wave + kWaves * i) + 8 * kg;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      int64_t row = row0 + m + 16 * rb;
      row = row < r_end ? row : r_end - 1;
      const float* src = a.A + row * a.lda;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int c0 = col + 4 * h;
        const float* at = src + (c0 < col_max ? c0 : col_max);
        if constexpr (ANYSTRIDE) {
          const Quad q = *reinterpret_cast<const Quad*>(at);
          pf[i][rb][h] = float4{q.x, q.y, q.z, q.w};
        } else {
          pf[i][rb][h] = *reinterpret_cast<const float4*>(at);
        }
      }
    }
  };

  auto load_first_tile = [&]() {
    if (r_begin < r_end) {
#pragma unroll
      for (int i = 0; i < SPW; ++i)
        if (step_exists(i)) load_step(i, r_begin);
    }
  };
  bool deferred = false;
  if constexpr (!HAS0 && HAS1) deferred = fa.cg.st != nullptr;
  if (!deferred) load_first_tile();

  // ---- [X|V] operands of this wave's steps, split and packed once (branch-free loads,
  //      issued while the first tile is already on its way) ----
  //      X in three bf16 parts: the logit product is taken to full fp32 accuracy (mfma6)
  // Deferred CG update: the operand is the new direction (or the final iterate), which every workgroup forms
  // for itself in LDS (the step slots are idle until the first tile is converted); its loads go out first, the
  // first tile right behind them.  If CG has stopped there is no product to form.
  // This lane's entries of X and V: rows 32 s + 8 kg + e (e < 8), class m.  The index is a uniform part (step and e)
  // plus a lane part, so that a load needs no address arithmetic of its own.  Nothing is masked here: padded class
  // lanes read class C-2 again and columns past p (last step only, index clamped into the operand) read some other
  // entry; both only ever meet zeros of the other operand (the rows stage ignores padded classes and gives them D = 0,
  // the tile's columns past p are zeroed when it is converted).
  float xop[SPW][8], vop[SPW][8];
  const unsigned lane_part = 8 * kg * NC + mc;
  const int last_index = p * NC - 1;
  // uniform element offset of (step slot i, e) and the lane's offset from it; only the last step slot can leave the
  // operand, there both parts are clamped so that their sum stays inside it
  auto operand_base = [&](int i, int e) {
    const int u = (kStepCols * (wave + kWaves * i) + e) * NC;
    return i < SPW - 1 ? u : (u < last_index ? u : last_index);
  };
  auto operand_lane = [&](int i, int e) {
    if (i < SPW - 1) return lane_part;
    const unsigned room = (unsigned)(last_index - operand_base(i, e));
    return lane_part < room ? lane_part : room;
  };
  bool from_lds = false;
  if constexpr (!HAS0 && HAS1) {
    if (deferred) {
      float* vec = reinterpret_cast<float*>(cm);  // p (C-1) floats; 4 p (C-1) <= 128 p bytes of step slots
      if (!cg_pending_update<kThreads, HALFQ ? SPW : 2 * SPW>(fa.cg, blockIdx.x == 0, vec, reinterpret_cast<double*>(part), load_first_tile))
        return;
      // LDS reads proper (a generic pointer would make these flat loads, whose results the compiler can only wait for
      // together with every outstanding global load, i.e. with the whole first tile)
#pragma unroll
      for (int i = 0; i < SPW; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) vop[i][e] = vec[operand_base(i, e) + operand_lane(i, e)];
      from_lds = true;
    }
  }
  if (!from_lds) {
#pragma unroll
    for (int i = 0; i < SPW; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) vop[i][e] = has1 ? (a.B1 + operand_base(i, e))[operand_lane(i, e)] : 0.f;
  }
#pragma unroll
  for (int i = 0; i < SPW; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) xop[i][e] = has0 ? (a.B0 + operand_base(i, e))[operand_lane(i, e)] : 0.f;
  u32x4 bx_hi[SPW], bx_lo[SPW], bx_lo2[SPW], bv_hi[SPW], bv_lo[SPW];
#pragma unroll
  for (int i = 0; i < SPW; ++i) {
    split8_3(xop[i], bx_hi[i], bx_lo[i], bx_lo2[i]);
    split8(vop[i], bv_hi[i], bv_lo[i]);
  }
  if (deferred) lds_barrier();  // every wave has picked its operands from LDS: the step slots may be overwritten

  u32x4 dhi, dlo;  // D of the current tile as MFMA operand
  for (int64_t row0 = r_begin; row0 < r_end; row0 += kTileRows) {
    // the row this wave handles in the rows stage: e = wave, row = row0 + 4 kg + (e & 3) + 16 (e >> 2)
    const int64_t my_row = row0 + 4 * kg + (wave & 3) + ((wave >> 2) << 4);
    const bool my_valid = my_row < r_end;
    const int64_t my_rowc = my_valid ? my_row : r_end - 1;
    float aux = 0.f;  // cached probability (Hessian-vector rows without X) or label (gradient / loss rows)
    if (KIND == kRowsHv && !has0) aux = a.Pin[(size_t)my_rowc * NC + mc];
    if (KIND == kRowsGrad || KIND == kRowsLoss) aux = __int_as_float(a.labels[my_rowc]);

    // ---------------- phase 1 ----------------
    f32x4 accZ[2], accW[2];
    accZ[0] = accZ[1] = accW[0] = accW[1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      const int s = wave + kWaves * i;
      if (step_exists(i)) {
        float av[2][8];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          av[rb][0] = pf[i][rb][0].x; av[rb][1] = pf[i][rb][0].y; av[rb][2] = pf[i][rb][0].z; av[rb][3] = pf[i][rb][0].w;
          av[rb][4] = pf[i][rb][1].x; av[rb][5] = pf[i][rb][1].y; av[rb][6] = pf[i][rb][1].z; av[rb][7] = pf[i][rb][1].w;
        }
        // Rows past the range were loaded as copies of the last row; they get D = 0 below.
        // Columns past p (last step only, uniform branch) must be zeroed: the row padding may hold anything.
        if (kStepCols * (s + 1) > p) {
          const int col = kStepCols * s + 8 * kg;
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int c0 = col + 4 * h;
            if constexpr (ANYSTRIDE) {
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
              const int nv = c0 <= col_max ? p - c0 : 0;  // valid elements of this float4 (clamped loads hold other columns)
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                av[0][4 * h + e] = e < nv ? av[0][4 * h + e] : 0.f;
                av[1][4 * h + e] = e < nv ? av[1][4 * h + e] : 0.f;
              }
            }
          }
        }
        // Both row blocks are converted first and the products are issued term by term across the (up to four)
        // accumulators, so that consecutive MFMAs never depend on each other.
        u32x4 ahi[2], alo[2], alo2[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          if (has0) split8_3(av[rb], ahi[rb], alo[rb], alo2[rb]);
          else split8(av[rb], ahi[rb], alo[rb]);
        }
        if (has0) {  // the three smallest of the six terms of Z (see mfma6)
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) accZ[rb] = mfma(alo2[rb], bx_hi[i], accZ[rb]);
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) accZ[rb] = mfma(ahi[rb], bx_lo2[i], accZ[rb]);
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) accZ[rb] = mfma(alo[rb], bx_lo[i], accZ[rb]);
        }
#pragma unroll
        for (int t = 0; t < 3; ++t) {  // lo * hi, hi * lo, hi * hi of Z and W
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) {
            const u32x4 aa = t == 0 ? alo[rb] : ahi[rb];
            if (has0) accZ[rb] = mfma(aa, t == 1 ? bx_lo[i] : bx_hi[i], accZ[rb]);
            if (has1) accW[rb] = mfma(aa, t == 1 ? bv_lo[i] : bv_hi[i], accW[rb]);
          }
        }
        // the registers are free again: prefetch the next tile (past the range the rows clamp to the last row)
        load_step(i, row0 + kTileRows);
        if (with_cols) {
          // transposed copy for phase 2: pair (row m, row m+16) of one column per 32-bit word
          char* base = cmw + i * kStepBytes;
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
            const unsigned hp = __builtin_amdgcn_perm(ahi[1][c >> 1], ahi[0][c >> 1], sel);
            const unsigned lp = __builtin_amdgcn_perm(alo[1][c >> 1], alo[0][c >> 1], sel);
            const int off = cm_offset(8 * kg + c, m >> 2) + ((m & 3) << 2);
            *reinterpret_cast<unsigned*>(base + off) = hp;
            *reinterpret_cast<unsigned*>(base + 2048 + off) = lp;
          }
        }
      }
    }
    // K-split partials of this wave, one 256-byte row per (quad, component)
    {
      float* pw = part + (size_t)(wave * 16) * 64 + lane;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (has0) { pw[(0 + e) * 64] = accZ[0][e]; pw[(4 + e) * 64] = accZ[1][e]; }
        if (has1) { pw[(8 + e) * 64] = accW[0][e]; pw[(12 + e) * 64] = accW[1][e]; }
      }
    }
    tile_barrier();

    // ---------------- rows stage: wave e handles rows row0 + 4 kg + (e & 3) + 16 (e >> 2) ----------------
    float z = 0.f, w = 0.f;
    {
      const float* pr = part + (size_t)(((wave >> 2) * 4 + (wave & 3))) * 64 + lane;
      float zp[kWaves], wp[kWaves];  // all partials requested before the first is added
#pragma unroll
      for (int sw = 0; sw < kWaves; ++sw) {
        zp[sw] = has0 ? pr[(sw * 16) * 64] : 0.f;
        wp[sw] = has1 ? pr[(sw * 16 + 8) * 64] : 0.f;
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int sw = 0; sw < kWaves; ++sw) {
        if (has0) z += zp[sw];
        if (has1) w += wp[sw];
      }
    }
    const size_t my_off = (size_t)my_row * NC + m;
    if (KIND == kRowsLogits) {
      if (cv && my_valid) {
        if (has0 && a.Z0out) a.Z0out[my_off] = z;
        if (has1 && a.Z1out) a.Z1out[my_off] = w;
      }
      tile_barrier();  // the partials are rewritten by the next tile
      continue;
    }
    float P, M = 0.f, alpha = 1.f, d;
    if (has0) {
      const float zc = cv ? z : 0.f;
      M = fmaxf(row16_max(zc), 0.f);       // max{0, Z_1..Z_{C-1}} (eq. max_x); with 16 free classes no padded lane supplies the 0
      const float E = cv ? expf(zc - M) : 0.f;
      alpha = row16_sum(E) + expf(-M);
      P = E / alpha;
    } else {
      P = cv ? aux : 0.f;
    }
    if (KIND == kRowsHv) {
      const float t = row16_sum(P * w);
      d = my_valid ? P * (w - t) : 0.f;
    } else {
      const bool mine = cv && m == __float_as_int(aux);
      d = my_valid ? P - (mine ? 1.f : 0.f) : 0.f;
      const float zb = row16_sum(mine ? z : 0.f);
      if (m == 0 && my_valid) loss_acc += (double)M + (double)logf(alpha) - (double)zb;
    }
    if (STORES && cv && my_valid) {
      if (a.Pout) a.Pout[my_off] = P;
      if (has0 && a.Z0out) a.Z0out[my_off] = z;
      if (KIND == kRowsHv && a.Z1out) a.Z1out[my_off] = w;  // directional logits A V, kept for the line search
    }
    if (!with_cols) {
      tile_barrier();  // the partials are rewritten by the next tile
      continue;
    }
    dbuf[wave * 64 + lane] = d;
    tile_barrier();

    // ---------------- phase 2 ----------------
    // out^T[:, step] += D^T (tile held in the step's LDS slot).  All LDS reads of the stage are requested ahead of their
    // use: the entries of D together, and the transposed tile of step i + 1 while the products of step i run, the two
    // column halves of a step taking turns so that no matrix instruction waits for the one before it.
    u32x4 th[2][2], tl[2][2];
    auto fetch_step = [&](int i, int b) {
      const char* base = cmw + i * kStepBytes;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int off = cm_offset(16 * h + m, kg);
        th[b][h] = *reinterpret_cast<const u32x4*>(base + off);
        tl[b][h] = *reinterpret_cast<const u32x4*>(base + 2048 + off);
      }
    };
    {
      float d0[4], d1[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {  // k-slot pair (2e, 2e+1) = (row 4kg+e, row 16+4kg+e)
        d0[e] = dbuf[e * 64 + lane];
        d1[e] = dbuf[(4 + e) * 64 + lane];
      }
      if (step_exists(0)) fetch_step(0, 0);
      __builtin_amdgcn_sched_barrier(0);  // keep the requests ahead of the packing below
      unsigned h[4], l[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        h[e] = pack2(d0[e], d1[e]);
        l[e] = pack2(d0[e] - low_as_float(h[e]), d1[e] - high_as_float(h[e]));
      }
      dhi = u32x4{h[0], h[1], h[2], h[3]};
      dlo = u32x4{l[0], l[1], l[2], l[3]};
    }
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      const int b = i & 1;
      if (i + 1 < SPW && step_exists(i + 1)) fetch_step(i + 1, b ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      if (step_exists(i)) {  // the three terms of mfma3 for both halves
        acc2[i][0] = mfma(dlo, th[b][0], acc2[i][0]);
        acc2[i][1] = mfma(dlo, th[b][1], acc2[i][1]);
        acc2[i][0] = mfma(dhi, tl[b][0], acc2[i][0]);
        acc2[i][1] = mfma(dhi, tl[b][1], acc2[i][1]);
        acc2[i][0] = mfma(dhi, th[b][0], acc2[i][0]);
        acc2[i][1] = mfma(dhi, th[b][1], acc2[i][1]);
      }
    }
  }

  // ---- epilogue: per-workgroup partial of A^T rows, and the partial loss ----
  // The 32 columns of a step are one contiguous run of 32 (C-1) floats of the partial: each wave lays its steps
  // out in that order in its own (now idle) LDS step slots and writes them with 16-byte stores, a whole run per
  // instruction, instead of 4-byte stores scattered at a stride of C-1 floats.
  if (with_cols) {
    float* out = fa.partial + (size_t)blockIdx.x * ((size_t)p * NC);
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      const int s = wave + kWaves * i;
      if (s < steps) {
        float* stage = reinterpret_cast<float*>(cmw + i * kStepBytes);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int c = 4 * kg + e;
            if (c < NC) stage[(16 * h + m) * NC + c] = acc2[i][h][e];
          }
      }
    }
    // LDS operations of one wave execute in order; the slots are private to the wave
    if (((p * NC) & 3) == 0) {  // every partial starts on a 16-byte boundary
      // a step's run is at most 32 * 16 floats = 128 pieces of 16 bytes, two per lane: all of them are read back before
      // the first is stored, so that the stage costs one LDS round trip instead of one per piece
      f32x4 va[SPW], vb[SPW];
#pragma unroll
      for (int i = 0; i < SPW; ++i) {
        const int s = wave + kWaves * i;
        const int cols = p - kStepCols * s < kStepCols ? p - kStepCols * s : kStepCols;
        const int quads = s < steps ? (cols * NC) >> 2 : 0;
        const f32x4* stage = reinterpret_cast<const f32x4*>(cmw + i * kStepBytes);
        const int last = quads > 0 ? quads - 1 : 0;
        va[i] = stage[lane < last ? lane : last];
        vb[i] = stage[lane + 64 < last ? lane + 64 : last];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < SPW; ++i) {
        const int s = wave + kWaves * i;
        if (s < steps) {
          const float* stage = reinterpret_cast<const float*>(cmw + i * kStepBytes);
          const int cols = p - kStepCols * s < kStepCols ? p - kStepCols * s : kStepCols;
          const int total = cols * NC;                       // floats of this step's run
          float* dst = out + (size_t)kStepCols * s * NC;     // 128 (C-1) s bytes into the partial
          const int quads = total >> 2;
          if (lane < quads) *reinterpret_cast<f32x4*>(dst + 4 * lane) = va[i];
          if (lane + 64 < quads) *reinterpret_cast<f32x4*>(dst + 4 * (lane + 64)) = vb[i];
          const int tail = total & 3;
          if (lane < tail) dst[4 * quads + lane] = stage[4 * quads + lane];
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < SPW; ++i) {
        const int s = wave + kWaves * i;
        if (s < steps) {
          const float* stage = reinterpret_cast<const float*>(cmw + i * kStepBytes);
          const int cols = p - kStepCols * s < kStepCols ? p - kStepCols * s : kStepCols;
          const int total = cols * NC;
          float* dst = out + (size_t)kStepCols * s * NC;
          for (int q = lane; q < total; q += 64) dst[q] = stage[q];
        }
      }
    }
  }
  if (KIND == kRowsGrad || KIND == kRowsLoss) {
    loss_acc = mfma_detail::wave64_sum(loss_acc);
    double* red = reinterpret_cast<double*>(dbuf);
    __syncthreads();
    if (lane == 0) red[wave] = loss_acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int wv = 0; wv < kWaves; ++wv) t += red[wv];
      a.loss_part[blockIdx.x] = t;
    }
  }
}

int num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
    else
      cus = 256;
  }
  return cus;
}

int steps_of(int p) { return (p + kStepCols - 1) / kStepCols; }

template <int SPW, int KIND, bool HAS0, bool HAS1, bool STORES, bool HALFQ, bool ANYSTRIDE>
hipError_t launch_ks(const FusedArgs& fa, int grid, size_t lds_bytes, hipStream_t st) {
  static uint64_t lds_set = 0;  // per device
  hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(&fused_kernel<SPW, KIND, HAS0, HAS1, STORES, HALFQ, ANYSTRIDE>), &lds_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((fused_kernel<SPW, KIND, HAS0, HAS1, STORES, HALFQ, ANYSTRIDE>), dim3(grid), dim3(kThreads), lds_bytes, st, fa);
  return hipGetLastError();
}

bool rows_16_byte_aligned(const RowArgs& a) { return (a.lda & 3) == 0 && (reinterpret_cast<uintptr_t>(a.A) & 15) == 0; }

template <int SPW, int KIND, bool HAS0, bool HAS1, bool STORES, bool HALFQ = false>
hipError_t launch_k(const FusedArgs& fa, int grid, size_t lds_bytes, hipStream_t st) {
  if (rows_16_byte_aligned(fa.r)) return launch_ks<SPW, KIND, HAS0, HAS1, STORES, HALFQ, false>(fa, grid, lds_bytes, st);
  return launch_ks<SPW, KIND, HAS0, HAS1, STORES, HALFQ, true>(fa, grid, lds_bytes, st);
}

// Kernels that may store rows of P / Z are separate instantiations: a store between the prefetch
// and its use makes the compiler wait for all outstanding loads.
template <int SPW, int KIND, bool HAS0, bool HAS1>
hipError_t launch_one(const FusedArgs& fa, int grid, size_t lds_bytes, hipStream_t st) {
  const RowArgs& a = fa.r;
  const bool stores = KIND == kRowsLogits || a.Pout != nullptr || a.Z0out != nullptr || a.Z1out != nullptr;
  if constexpr (!HAS0 && HAS1 && (KIND == kRowsHv || KIND == kRowsLogits)) {
    // the instantiation with the larger update capacity needs more registers in its prologue: it is taken only for a
    // pending CG update on vectors that do not fit the smaller one
    if (fa.cg.st == nullptr || (fa.cg.dlen >> 2) <= (int64_t)kThreads * SPW) {
      if (stores) return launch_k<SPW, KIND, HAS0, HAS1, true, true>(fa, grid, lds_bytes, st);
      return launch_k<SPW, KIND, HAS0, HAS1, false, true>(fa, grid, lds_bytes, st);
    }
  }
  if (stores) return launch_k<SPW, KIND, HAS0, HAS1, true>(fa, grid, lds_bytes, st);
  return launch_k<SPW, KIND, HAS0, HAS1, false>(fa, grid, lds_bytes, st);
}

template <int SPW>
hipError_t launch_spw(const FusedArgs& fa, int grid, size_t lds_bytes, hipStream_t st) {
  const RowArgs& a = fa.r;
  const bool h0 = a.B0 != nullptr, h1 = a.B1 != nullptr;
  switch (a.kind) {
    case kRowsHv:
      if (fa.partial == nullptr || !h1) return hipErrorInvalidValue;
      if (h0) return launch_one<SPW, kRowsHv, true, true>(fa, grid, lds_bytes, st);
      if (a.Pin == nullptr) return hipErrorInvalidValue;
      return launch_one<SPW, kRowsHv, false, true>(fa, grid, lds_bytes, st);
    case kRowsGrad:
      if (fa.partial == nullptr || !h0 || a.labels == nullptr || a.loss_part == nullptr) return hipErrorInvalidValue;
      return launch_one<SPW, kRowsGrad, true, false>(fa, grid, lds_bytes, st);
    case kRowsLoss:
      if (!h0 || a.labels == nullptr || a.loss_part == nullptr) return hipErrorInvalidValue;
      return launch_one<SPW, kRowsLoss, true, false>(fa, grid, lds_bytes, st);
    case kRowsLogits:
      if (h0 && h1) return launch_one<SPW, kRowsLogits, true, true>(fa, grid, lds_bytes, st);
      if (h1) return launch_one<SPW, kRowsLogits, false, true>(fa, grid, lds_bytes, st);
      if (h0) return launch_one<SPW, kRowsLogits, true, false>(fa, grid, lds_bytes, st);
      return hipErrorInvalidValue;
    default:
      return hipErrorInvalidValue;
  }
}

}  // namespace

bool fused_supported(const Shape& s, int64_t lda, const void* A) {
  if (s.NC > 16) return false;
  if (steps_of(s.p) > kMaxSteps) return false;
  if ((reinterpret_cast<uintptr_t>(A) & 3) != 0 || lda < s.p) return false;
  if (((lda & 3) != 0 || (reinterpret_cast<uintptr_t>(A) & 15) != 0) && s.p < 4) return false;  // whole 16-byte pieces inside a row
  return true;
}

int fused_num_partials(const Shape& s) {
  // host-only upper bound used for the workspace layout: one partial per workgroup
  const int64_t tiles = (s.n + kTileRows - 1) / kTileRows;
  const int64_t g = tiles < 256 ? tiles : 256;
  return (int)(g < 1 ? 1 : g);
}

hipError_t launch_fused(const RowArgs& a, float* partial, int nparts, hipStream_t st, const CgPend* cg) {
  FusedArgs fa;
  fa.r = a;
  if (cg != nullptr) {
    if (a.B0 != nullptr || a.B1 == nullptr || (a.kind != kRowsHv && a.kind != kRowsLogits)) return hipErrorInvalidValue;
    if (cg->ndot < 1 || cg->ndot > kThreads || cg->dlen != (int64_t)a.p * a.NC) return hipErrorInvalidValue;
    fa.cg = *cg;
  } else {
    fa.cg = CgPend{};
  }
  fa.partial = partial;
  fa.steps = steps_of(a.p);
  const int grid = nparts;
  fa.rows_per_wg = (int)((a.n + grid - 1) / grid);
  const size_t lds_bytes = (size_t)fa.steps * kStepBytes + kPartBytes + kSumBytes;
  const int spw = (fa.steps + kWaves - 1) / kWaves;
  switch (spw) {
    case 1: return launch_spw<1>(fa, grid, lds_bytes, st);
    case 2: return launch_spw<2>(fa, grid, lds_bytes, st);
    case 3: return launch_spw<3>(fa, grid, lds_bytes, st);
    case 4: return launch_spw<4>(fa, grid, lds_bytes, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nadmm
