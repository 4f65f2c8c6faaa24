// Wavefront-level helpers shared by the MFMA decode kernels (gfx950): operand types, the nibble ->
// bf16 expansion, bf16 hi/lo splitting, lane-row exchanges, DPP row reductions, barrier-free LDS
// hand-over inside one wavefront, and an LDS Walsh-Hadamard transform.
#pragma once

#include "saw_common.h"

namespace saw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define LDS_AS __attribute__((address_space(3)))
#define GLOBAL_AS __attribute__((address_space(1)))

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Eight packed nibbles -> eight bf16 values 128 + c, in k-order (n0, n4, n1, n5, n2, n6, n3, n7).
// `k` holds 0x43004300 in a VGPR (see bf16_bias()), which lets each mask-and-bias be one
// v_and_or_b32 with a single scalar operand.
__device__ __forceinline__ bf16x8 unpack8(uint32_t w, uint32_t k) {
  u32x4 r;
  r.x = (w & 0x000F000Fu) | k;
  r.y = ((w >> 4) & 0x000F000Fu) | k;
  r.z = ((w >> 8) & 0x000F000Fu) | k;
  r.w = ((w >> 12) & 0x000F000Fu) | k;
  return as_bf16x8(r);
}
__device__ __forceinline__ uint32_t bf16_bias() {
  uint32_t k;
  asm volatile("v_mov_b32 %0, 0x43004300" : "=v"(k));
  return k;
}

__device__ __forceinline__ f32x4 mfma_bf16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// x = hi + lo with hi a truncated bf16 and lo a rounded bf16 of the remainder.
__device__ __forceinline__ void split_bf16(float x, uint32_t& hi16, uint32_t& lo16, float& sum) {
  const uint32_t u = __float_as_uint(x);
  const float hf = __uint_as_float(u & 0xffff0000u);
  hi16 = u >> 16;
  uint32_t r = __float_as_uint(x - hf);
  r += 0x7fffu + ((r >> 16) & 1u);
  lo16 = r >> 16;
  sum = hf + __uint_as_float(r & 0xffff0000u);
}

// v_permlane16_swap: x <- rows (a0, b0, a2, b2), y <- rows (a1, b1, a3, b3)   (row = 16 lanes)
__device__ __forceinline__ void swap16(float a, float b, float& x, float& y) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  x = __uint_as_float(r[0]);
  y = __uint_as_float(r[1]);
}
// v_permlane32_swap: x <- rows (a0, a1, b0, b1), y <- rows (a2, a3, b2, b3)
__device__ __forceinline__ void swap32(float a, float b, float& x, float& y) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  x = __uint_as_float(r[0]);
  y = __uint_as_float(r[1]);
}

// v + (v of the lane 16 / 32 away, index xor), as two register permutes instead of a trip through
// the LDS crossbar (ds_bpermute)
__device__ __forceinline__ float add_xor16(float v) {
  float x, y;
  swap16(v, v, x, y);              // x rows (v0, v0, v2, v2), y rows (v1, v1, v3, v3)
  return x + y;
}
__device__ __forceinline__ float add_xor32(float v) {
  float x, y;
  swap32(v, v, x, y);              // x rows (v0, v1, v0, v1), y rows (v2, v3, v2, v3)
  return x + y;
}
__device__ __forceinline__ float max_xor16(float v) {
  float x, y;
  swap16(v, v, x, y);
  return fmaxf(x, y);
}
__device__ __forceinline__ float max_xor32(float v) {
  float x, y;
  swap32(v, v, x, y);
  return fmaxf(x, y);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xf, 0xf, false));
}
// max over the 16 lanes of each row (rotations by 1, 2, 4, 8)
__device__ __forceinline__ float row_allmax(float v) {
  v = fmaxf(v, dpp_f<0x121>(v));
  v = fmaxf(v, dpp_f<0x122>(v));
  v = fmaxf(v, dpp_f<0x124>(v));
  v = fmaxf(v, dpp_f<0x128>(v));
  return v;
}
__device__ __forceinline__ float row_allsum(float v) {
  v += dpp_f<0x121>(v);
  v += dpp_f<0x122>(v);
  v += dpp_f<0x124>(v);
  v += dpp_f<0x128>(v);
  return v;
}

// The block is one wavefront: LDS operations of a wave execute in order, so exchanging data
// between lanes through LDS needs no barrier and no wait, only a point the compiler will not
// move memory accesses across.  (A workgroup barrier would also wait for every LDS-DMA transfer
// in flight, which is exactly what the prefetch must not do.)
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// In-place un-normalised block Walsh-Hadamard transform (block size h = 16, 32, 64 or 128) of NVEC
// vectors of 128 floats in LDS (16-byte aligned), run by one wavefront.  Three passes with eight
// values per lane in registers: strides 1-2-4 inside chunks of eight contiguous values, strides
// 8-16-32 over values eight apart (as far as h reaches), and stride 64 when h = 128.
template <int NVEC>
__device__ __forceinline__ void wave_lds_fwht128(float* x, int h, int lane) {
  // (compile-time trip counts: every loop below is unrolled, there is no loop-carried address)
#pragma unroll
  for (int it = 0; it < (NVEC * 16 + 63) / 64; ++it) {
    const int ch = lane + 64 * it;
    if (NVEC * 16 % 64 == 0 || ch < NVEC * 16) {
      f32x4* const p = (f32x4*)(x + 8 * ch);
      const f32x4 a = p[0], b = p[1];
      float e[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
      for (int st = 1; st < 8; st <<= 1)
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (!(k & st)) { const float u = e[k], v = e[k + st]; e[k] = u + v; e[k + st] = u - v; }
      p[0] = f32x4{e[0], e[1], e[2], e[3]};
      p[1] = f32x4{e[4], e[5], e[6], e[7]};
    }
  }
  wave_sync();
#pragma unroll
  for (int it = 0; it < (NVEC * 16 + 63) / 64; ++it) {
    const int g = lane + 64 * it;
    if (NVEC * 16 % 64 == 0 || g < NVEC * 16) {
      float* const p = x + (g >> 4) * 128 + ((g >> 3) & 1) * 64 + (g & 7);
      float e[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) e[k] = p[8 * k];
#pragma unroll
      for (int st = 1; st < 8; st <<= 1) {
        if (8 * st < h) {                                    // wavefront-uniform
#pragma unroll
          for (int k = 0; k < 8; ++k)
            if (!(k & st)) { const float u = e[k], v = e[k + st]; e[k] = u + v; e[k + st] = u - v; }
        }
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) p[8 * k] = e[k];
    }
  }
  wave_sync();
  if (h > 64) {
#pragma unroll
    for (int v = 0; v < NVEC; ++v) {
      float* const b = x + lane;
      const float a = b[v * 128], c = b[v * 128 + 64];
      b[v * 128] = a + c;
      b[v * 128 + 64] = a - c;
    }
    wave_sync();
  }
}

// In-place x <- x M for NV vectors of 128 floats in LDS, run by one wavefront: out[v][j] =
// sum_i x[v][i] M[i][j] with M a global fp32 [128][128] row-major matrix (the learned rotation of
// App. A.3 or its transpose).  Lane l takes four consecutive columns 4 (l % 32) .. + 3 and the rows of
// half l / 32 (rows 64 h .. 64 h + 63): every load is 16 bytes, a load instruction covers two whole rows
// of M, and the 64 loads of a lane go out in four rounds of 16 (what bounds this routine is the latency
// of M coming from L2 while every wavefront of the chip asks for it, so few, wide rounds matter).  Two
// partial sums per output and half (rows of even and odd index), added pairwise at the end, keep the
// rounding error near that of a pairwise sum.
template <int NV>
__device__ __forceinline__ void wave_lds_matvec128(float* x, const float* __restrict__ M, int lane) {
  const int half = lane >> 5, cq = lane & 31;
  float acc[NV][2][4];
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[v][e][c] = 0.f;
  const float* const mbase = M + (64 * half) * 128 + 4 * cq;
#pragma unroll 1
  for (int t = 0; t < 4; ++t) {
    f32x4 m[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) m[u] = *(const f32x4*)(mbase + (16 * t + u) * 128);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const float* xr = x + v * 128 + 64 * half + 16 * t;
#pragma unroll
      for (int u4 = 0; u4 < 4; ++u4) {
        const f32x4 xv = *(const f32x4*)(xr + 4 * u4);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int u = 4 * u4 + k;
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[v][u & 1][c] = fmaf(xv[k], m[u][c], acc[v][u & 1][c]);
        }
      }
    }
  }
  wave_sync();                                               // every read of x is done
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    f32x4 r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r[c] = add_xor32(acc[v][0][c] + acc[v][1][c]);   // the two halves of the rows
    if (half == 0) *(f32x4*)(x + v * 128 + 4 * cq) = r;
  }
  wave_sync();
}

}  // namespace saw
