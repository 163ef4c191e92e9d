// Device helpers shared by the matrix-core kernels (gfx950): bf16 high/low splitting of fp32 operands,
// the three-term MFMA product, 16-lane DPP reductions and the swizzled LDS layout of the transposed tile.
#pragma once

#include <hip/hip_runtime.h>

namespace nadmm {
namespace mfma_detail {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned pack2(float a, float b) {  // round-to-nearest-even, a in the low half
  bf16x2 v = {(__bf16)a, (__bf16)b};
  unsigned r = __builtin_bit_cast(unsigned, v);
  asm volatile("" : "+v"(r));  // keep the packed conversion as one instruction (no per-half re-conversion)
  return r;
}
__device__ __forceinline__ float low_as_float(unsigned h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float high_as_float(unsigned h) { return __uint_as_float(h & 0xffff0000u); }

// 8 floats -> packed bf16 high parts and packed bf16 residuals
__device__ __forceinline__ void split8(const float (&a)[8], u32x4& hi, u32x4& lo) {
  unsigned h[4], l[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    h[k] = pack2(a[2 * k], a[2 * k + 1]);
    l[k] = pack2(a[2 * k] - low_as_float(h[k]), a[2 * k + 1] - high_as_float(h[k]));
  }
  hi = u32x4{h[0], h[1], h[2], h[3]};
  lo = u32x4{l[0], l[1], l[2], l[3]};
}

// 8 floats -> three packed bf16 parts, x = hi + mid + lo + O(2^-24 |x|): the residual after each rounding is
// exact in fp32, so the three parts carry the whole fp32 significand
__device__ __forceinline__ void split8_3(const float (&a)[8], u32x4& hi, u32x4& mid, u32x4& lo) {
  unsigned h[4], m[4], l[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    h[k] = pack2(a[2 * k], a[2 * k + 1]);
    const float r0 = a[2 * k] - low_as_float(h[k]), r1 = a[2 * k + 1] - high_as_float(h[k]);
    m[k] = pack2(r0, r1);
    l[k] = pack2(r0 - low_as_float(m[k]), r1 - high_as_float(m[k]));
  }
  hi = u32x4{h[0], h[1], h[2], h[3]};
  mid = u32x4{m[0], m[1], m[2], m[3]};
  lo = u32x4{l[0], l[1], l[2], l[3]};
}

__device__ __forceinline__ f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
// c += (ahi + alo) (bhi + blo) without the lo*lo term
__device__ __forceinline__ f32x4 mfma3(u32x4 ahi, u32x4 alo, u32x4 bhi, u32x4 blo, f32x4 c) {
  c = mfma(alo, bhi, c);
  c = mfma(ahi, blo, c);
  return mfma(ahi, bhi, c);
}

// c += (ahi + amid + alo) (bhi + bmid + blo) keeping the six terms of relative weight >= 2^-16 (the
// dropped ones are below 2^-23): the product is then as accurate as an fp32 one.  Used for the logits
// Z = A X only, whose absolute error exp() turns into a relative error of the probabilities (Section 2.2).
__device__ __forceinline__ f32x4 mfma6(u32x4 ahi, u32x4 amid, u32x4 alo, u32x4 bhi, u32x4 bmid, u32x4 blo, f32x4 c) {
  c = mfma(alo, bhi, c);
  c = mfma(ahi, blo, c);
  c = mfma(amid, bmid, c);
  c = mfma(amid, bhi, c);
  c = mfma(ahi, bmid, c);
  return mfma(ahi, bhi, c);
}

template <int N>
__device__ __forceinline__ float row_ror(float v) {  // rotate within each group of 16 lanes
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += row_ror<8>(v);
  v += row_ror<4>(v);
  v += row_ror<2>(v);
  v += row_ror<1>(v);
  return v;
}
// Sum over the 64 lanes of a wave, the same value in every lane: rotations inside the four rows of 16 lanes, then the
// four row totals in a fixed order.  Vector instructions only; a tree of cross-lane shuffles goes through the LDS pipe
// with its latency at every stage.
__device__ __forceinline__ float wave64_sum(float v) {
  v = row16_sum(v);
  const int b = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}
// The same for float64 (two 32-bit rotations per step).
template <int N>
__device__ __forceinline__ double row_ror(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), 0x120 + N, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), 0x120 + N, 0xf, 0xf, false);
  return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned)lo);
}
__device__ __forceinline__ double row16_sum(double v) {
  v += row_ror<8>(v);
  v += row_ror<4>(v);
  v += row_ror<2>(v);
  v += row_ror<1>(v);
  return v;
}
__device__ __forceinline__ double lane_value(double v, int lane) {  // lane: a constant
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), lane);
  const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
  return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned)lo);
}
__device__ __forceinline__ double wave64_sum(double v) {
  v = row16_sum(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
// sums over lanes 0..31 and over lanes 32..63, each returned in its own lanes
__device__ __forceinline__ double half32_sum(double v) {
  v = row16_sum(v);
  const double lo = lane_value(v, 0) + lane_value(v, 16), hi = lane_value(v, 32) + lane_value(v, 48);
  return (threadIdx.x & 32) ? hi : lo;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, row_ror<8>(v));
  v = fmaxf(v, row_ror<4>(v));
  v = fmaxf(v, row_ror<2>(v));
  v = fmaxf(v, row_ror<1>(v));
  return v;
}

// LDS offset (bytes, within one 2 KB plane of a step) of column q (0..31), 16-byte chunk ck (0..3)
__device__ __forceinline__ int cm_offset(int q, int ck) {
  const int qs = q ^ ((q >> 3) & 1);
  const int g = (qs >> 1) & 3;
  return qs * 64 + ((ck ^ g) << 4);
}

}  // namespace mfma_detail
}  // namespace nadmm
