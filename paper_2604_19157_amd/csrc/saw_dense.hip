// Preparation of a learned per-layer rotation R_l (Sec. 3 "Hessian-Aware Quantization"; App. A.3,
// runtime application: q^ = (q H_b) R_l, k^ = (k H_b) R_l, the same for V) into the layouts the
// kernels read; see the layout comment in saw_common.h.  Run once per layer, not on the hot path.
#include "saw_common.h"

namespace saw {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bf16_rne_bits(float x) {       // round to nearest even (v_cvt_pk_bf16_f32)
  const uint32_t r = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{x, 0.f}, bf16x2_t));
  return r & 0xffffu;
}

// 64 blocks of 256 threads: thread t copies element t of R_l into the fp32 plane and into its
// transposed position, and each of the first 2048 threads also builds one (J, a, lane) group of
// the three limb planes.
__global__ __launch_bounds__(256) void prepare_dense_kernel(const float* __restrict__ R, uint8_t* __restrict__ out) {
  constexpr int D = kDenseD;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < D * D) {
    const int i = t / D, j = t % D;
    const float v = R[t];
    ((float*)out)[t] = v;                                              // R_l
    ((float*)(out + kDenseRtOffset))[j * D + i] = v;                   // R_l^T
  }
  // limb planes: one thread per (J, a, lane) builds the three 16-byte groups
  if (t < 8 * 4 * 64) {
    const int lane = t & 63, a = (t >> 6) & 3, J = t >> 8;
    const int j = dense_out_channel(J, lane & 15);
    uint32_t w[3][4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      uint32_t pk[3] = {0u, 0u, 0u};
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int i = 32 * a + 8 * (lane >> 4) + 2 * e2 + half;
        const float x = R[i * D + j];
        const uint32_t hb = bf16_rne_bits(x);
        const float r1 = x - __uint_as_float(hb << 16);
        const uint32_t mb = bf16_rne_bits(r1);
        const float r2 = r1 - __uint_as_float(mb << 16);
        const uint32_t lb = bf16_rne_bits(r2);
        pk[0] |= hb << (16 * half);
        pk[1] |= mb << (16 * half);
        pk[2] |= lb << (16 * half);
      }
#pragma unroll
      for (int L = 0; L < 3; ++L) w[L][e2] = pk[L];
    }
#pragma unroll
    for (int L = 0; L < 3; ++L) {
      uint4* dst = (uint4*)(out + kDenseLimbOffset) + ((L * 8 + J) * 4 + a) * 64 + lane;
      *dst = make_uint4(w[L][0], w[L][1], w[L][2], w[L][3]);
    }
  }
}

int launch_prepare_dense(const float* R, void* prepared, hipStream_t st) {
  prepare_dense_kernel<<<dim3(kDenseD * kDenseD / 256), dim3(256), 0, st>>>(R, (uint8_t*)prepared);
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

}  // namespace saw
