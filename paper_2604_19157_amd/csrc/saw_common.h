// Device-side helpers shared by the SAW-INT4 kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "saw.h"

#define SAW_WAVE 64

namespace saw {

// ---- 16-bit element conversions (exact widening; round-to-nearest-even narrowing) ----
__device__ __forceinline__ float bf16_to_f32(uint32_t u16) { return __uint_as_float(u16 << 16); }
__device__ __forceinline__ float f16_to_f32(uint32_t u16) {
  union { uint16_t u; _Float16 h; } c;
  c.u = (uint16_t)u16;
  return (float)c.h;
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t f32_to_f16(float f) {
  union { uint16_t u; _Float16 h; } c;
  c.h = (_Float16)f;
  return c.u;
}

// Widen the two 16-bit halves of a dword.
template <int DT>
__device__ __forceinline__ void widen2(uint32_t w, float& lo, float& hi) {
  if (DT == SAW_BF16) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
  } else {
    lo = f16_to_f32(w & 0xffffu);
    hi = f16_to_f32(w >> 16);
  }
}

__device__ __forceinline__ float load_elem(const void* p, int dtype, int64_t i) {
  if (dtype == SAW_F32) return ((const float*)p)[i];
  uint32_t u = ((const uint16_t*)p)[i];
  return dtype == SAW_BF16 ? bf16_to_f32(u) : f16_to_f32(u);
}
__device__ __forceinline__ void store_elem(void* p, int dtype, int64_t i, float v) {
  if (dtype == SAW_F32) ((float*)p)[i] = v;
  else if (dtype == SAW_BF16) ((uint16_t*)p)[i] = f32_to_bf16(v);
  else ((uint16_t*)p)[i] = f32_to_f16(v);
}

// Randomised Hadamard (Sec. 3): R = diag(sigma) H_blk, sigma given as one bit per channel (set =
// negated).  sign_pairs<T>(bits, c0) turns the 8 bits of channels c0 .. c0+7 into four dwords whose
// bits 15 and 31 flip the signs of eight packed 16-bit floats (bf16 or fp16 alike); sign_of(bits, c)
// is +1 or -1 for one channel.
struct SignBits { uint32_t w[4]; };
__device__ __forceinline__ void sign_pairs(const SignBits& sb, int c0, uint32_t (&x)[4]) {
  const uint32_t word = (c0 >> 5) == 0 ? sb.w[0] : (c0 >> 5) == 1 ? sb.w[1] : (c0 >> 5) == 2 ? sb.w[2] : sb.w[3];
  const uint32_t m8 = (word >> (c0 & 31)) & 0xffu;
#pragma unroll
  for (int i = 0; i < 4; ++i) x[i] = (((m8 >> (2 * i)) & 1u) << 15) | (((m8 >> (2 * i + 1)) & 1u) << 31);
}
__device__ __forceinline__ uint32_t sign_flip32(const SignBits& sb, int c) {      // 0x80000000 if channel c is negated
  const uint32_t word = (c >> 5) == 0 ? sb.w[0] : (c >> 5) == 1 ? sb.w[1] : (c >> 5) == 2 ? sb.w[2] : sb.w[3];
  return ((word >> (c & 31)) & 1u) << 31;
}
__device__ __forceinline__ float apply_sign(const SignBits& sb, int c, float v) {
  return __uint_as_float(__float_as_uint(v) ^ sign_flip32(sb, c));
}

// The prepared form of a learned per-layer rotation R_l (App. A.3) for head_dim 128, as
// saw_prepare_dense_rotation lays it out:
//   [0, 64 KiB)        R_l, fp32 row-major [i][j]                (y = x R_l: query, appended token)
//   [64 KiB, 128 KiB)  R_l^T, fp32 row-major                     (outputs, read-backs)
//   [128 KiB, 224 KiB) three bf16 limbs (hi, mid, lo; hi + mid + lo = R_l to 24 bits) as A operands of
//                      v_mfma_f32_16x16x32_bf16 for the store kernel: 16 bytes per (limb L, output tile
//                      J < 8, k-step a < 4, lane) at index ((L * 8 + J) * 4 + a) * 64 + lane, holding
//                      R_l[32 a + 8 (lane / 16) + e][dense_out_channel(J, lane % 16)], e = 0..7.
constexpr int kDenseD = 128;
constexpr size_t kDenseRtOffset = (size_t)kDenseD * kDenseD * 4;
constexpr size_t kDenseLimbOffset = 2 * kDenseRtOffset;
constexpr size_t kDenseBytes = kDenseLimbOffset + (size_t)3 * 8 * 4 * 64 * 16;
// output channel of row m (0..15) of output tile J (0..7): tiles 2 a' and 2 a' + 1 together give lane
// (token, rg) the eight contiguous channels 32 a' + 8 rg .. + 7, the layout the store kernel quantises from
__host__ __device__ inline int dense_out_channel(int J, int m) { return 32 * (J >> 1) + 8 * (m >> 2) + 4 * (J & 1) + (m & 3); }

// 1/sqrt(h) for the supported Hadamard orders (correctly rounded constants).
__device__ __forceinline__ float had_norm(int h) {
  return h == 16 ? 0.25f : h == 32 ? 0.17677669529663687f : h == 64 ? 0.125f
       : h == 128 ? 0.08838834764831845f : 1.0f;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Split-KV geometry shared by host and device code.
struct SplitPlan {
  int32_t num_splits;     // partitions per sequence
  int32_t chunk_tokens;   // tokens per partition (multiple of 64)
  int32_t bound;          // clamp for seq_lens
  int32_t waves_per_item; // wavefronts that share one partition in the MFMA decode kernel
};

}  // namespace saw
