// Read-back (dequantise / un-rotate) of the INT4 pages, and the 16-bit comparison cache's store.
// Paper: App. A.1 (x^ = s (c - z)), App. A.4 (H is its own inverse).
//
// Lane layout: a head vector of D values is spread over D/8 adjacent lanes, eight contiguous
// channels per lane.  The Walsh-Hadamard butterfly runs its first three stages inside the lane
// and the remaining log2(h) - 3 stages across lanes; it is un-normalised (+/-1 sums only).
#include "saw_common.h"

namespace saw {


// One in-lane radix-2 stage over e[0..7] with span S.
template <int S>
__device__ __forceinline__ void stage8(float (&e)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if ((i & S) == 0) {
      float a = e[i], b = e[i + S];
      e[i] = a + b;
      e[i + S] = a - b;
    }
  }
}

// Un-normalised block Walsh-Hadamard transform of a vector held 8 channels per lane by
// LPV adjacent lanes; `sub` is this lane's index within the vector.
template <int LPV>
__device__ __forceinline__ void fwht(float (&e)[8], int sub, int h) {
  stage8<1>(e);
  stage8<2>(e);
  stage8<4>(e);
#pragma unroll
  for (int m = 1; m < LPV; m <<= 1) {
    if (8 * m < h) {  // wave-uniform: h is a kernel argument
      const bool upper = (sub & m) != 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float o = __shfl_xor(e[i], m, SAW_WAVE);
        e[i] = upper ? (o - e[i]) : (e[i] + o);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
struct DequantParams {
  const uint8_t* codes[2];
  const float* meta[2];
  float* out[2];
  const int32_t* page_table;
  int32_t max_pages, n_kv_heads, num_pages;
  int32_t seq, pos_begin, n_tokens;
  int32_t had_block;
  int32_t unrot[2];
  SignBits signs;
  const float* dense_t;   // transpose of a learned rotation R_l (App. A.3), fp32 [128][128] row-major; null: none
  int32_t undense[2];     // multiply K / V by R_l^T before the Hadamard's inverse
};

template <int D>
__global__ __launch_bounds__(256) void dequant_pages_kernel(DequantParams p) {
  constexpr int LPV = D / 8;
  constexpr int VPB = 256 / LPV;
  const int tid = threadIdx.x;
  const int sub = tid % LPV;
  const int which = blockIdx.y;
  if (p.out[which] == nullptr) return;
  const int64_t vid = (int64_t)blockIdx.x * VPB + tid / LPV;
  const int64_t n_vec = (int64_t)p.n_tokens * p.n_kv_heads;
  const bool live = vid < n_vec;
  const int64_t vv = live ? vid : 0;
  const int head = (int)(vv % p.n_kv_heads);
  const int t = (int)(vv / p.n_kv_heads);
  const int pos = p.pos_begin + t;
  int32_t page = p.page_table[(int64_t)p.seq * p.max_pages + (pos >> 4)];
  const bool ok = live && page >= 0 && page < p.num_pages;
  if (!ok) page = 0;
  const int64_t vec = ((int64_t)page * p.n_kv_heads + head) * 16 + (pos & 15);
  const uint32_t w = ((const uint32_t*)(p.codes[which] + vec * (D / 2)))[sub];
  const float2 sz = *(const float2*)(p.meta[which] + vec * 2);
  float e[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) e[i] = sz.x * ((float)((w >> (4 * i)) & 15u) - sz.y);
  if (D == 128 && p.undense[which]) {          // block-uniform: x^ R_l^T first (the inverse of a rotation is its transpose)
    __shared__ __attribute__((aligned(16))) float xs[VPB][D];
    float* const row = xs[tid / LPV];
#pragma unroll
    for (int i = 0; i < 8; ++i) row[8 * sub + i] = e[i];
    __syncthreads();
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll 4
    for (int k = 0; k < D; ++k) {
      const float xk = row[k];
      const float4 r0 = *(const float4*)(p.dense_t + k * D + 8 * sub);
      const float4 r1 = *(const float4*)(p.dense_t + k * D + 8 * sub + 4);
      acc[0] = fmaf(xk, r0.x, acc[0]); acc[1] = fmaf(xk, r0.y, acc[1]);
      acc[2] = fmaf(xk, r0.z, acc[2]); acc[3] = fmaf(xk, r0.w, acc[3]);
      acc[4] = fmaf(xk, r1.x, acc[4]); acc[5] = fmaf(xk, r1.y, acc[5]);
      acc[6] = fmaf(xk, r1.z, acc[6]); acc[7] = fmaf(xk, r1.w, acc[7]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = acc[i];
  }
  if (p.unrot[which]) {
    fwht<LPV>(e, sub, p.had_block);
    const float norm = had_norm(p.had_block);
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = apply_sign(p.signs, 8 * sub + i, e[i] * norm);   // y H_blk diag(sigma) = y R^T
  }
  if (!ok) return;
  float* dst = p.out[which] + ((int64_t)t * p.n_kv_heads + head) * D + sub * 8;
  *(float4*)dst = make_float4(e[0], e[1], e[2], e[3]);
  *(float4*)(dst + 4) = make_float4(e[4], e[5], e[6], e[7]);
}

// ---------------------------------------------------------------------------------------
// 16-bit comparison cache: plain paged copy of K/V rows.
struct Kv16StoreParams {
  uint16_t* pages[2];
  const void* in[2];
  const int32_t* page_table;
  const int32_t* slots;
  int64_t T, token_stride;
  int32_t n_seqs, max_pages, num_pages, n_kv_heads;
};

template <int D>
__global__ __launch_bounds__(256) void kv16_store_kernel(Kv16StoreParams p) {
  constexpr int LPV = D / 8;
  constexpr int VPB = 256 / LPV;
  const int tid = threadIdx.x;
  const int sub = tid % LPV;
  const int64_t vid = (int64_t)blockIdx.x * VPB + tid / LPV;
  if (vid >= p.T * 2 * p.n_kv_heads) return;
  const int head = (int)(vid % p.n_kv_heads);
  const int which = (int)((vid / p.n_kv_heads) & 1);
  const int64_t t = vid / (2 * p.n_kv_heads);
  const int32_t seq = p.slots[2 * t];
  const int32_t pos = p.slots[2 * t + 1];
  if (seq < 0 || seq >= p.n_seqs || pos < 0 || (pos >> 4) >= p.max_pages) return;
  const int32_t page = p.page_table[(int64_t)seq * p.max_pages + (pos >> 4)];
  if (page < 0 || page >= p.num_pages) return;
  const uint16_t* src = (const uint16_t*)p.in[which] + t * p.token_stride + head * D + sub * 8;
  const int64_t vec = ((int64_t)page * p.n_kv_heads + head) * 16 + (pos & 15);
  *(uint4*)(p.pages[which] + vec * D + sub * 8) = *(const uint4*)src;
}

// ---------------------------------------------------------------------------------------
// host launchers (called from saw_api.hip)
// the store kernel itself lives in saw_store_mfma.hip
int launch_store_mfma(const saw_cache_t* c, const void* const* K, const void* const* V, int n_layers, int dt,
                      int64_t T, int64_t stride, const int32_t* pt, int32_t n_seqs, int32_t max_pages,
                      const int32_t* slots, const int32_t* append_lens, int32_t append_bound, hipStream_t st);

// `slots` null: token t is appended to sequence t at position append_lens[t] (skipped when that
// exceeds append_bound).
int launch_store(const saw_cache_t* c, const void* K, const void* V, int dt, int64_t T, int64_t stride,
                 const int32_t* pt, int32_t n_seqs, int32_t max_pages, const int32_t* slots,
                 const int32_t* append_lens, int32_t append_bound, hipStream_t st) {
  return launch_store_mfma(c, &K, &V, 1, dt, T, stride, pt, n_seqs, max_pages, slots, append_lens, append_bound, st);
}

// Several layers' stores in one launch: `c`, `K`, `V` are host arrays of n_layers entries.
int launch_store_layers(const saw_cache_t* c, const void* const* K, const void* const* V, int n_layers, int dt,
                        int64_t T, int64_t stride, const int32_t* pt, int32_t n_seqs, int32_t max_pages,
                        const int32_t* slots, hipStream_t st) {
  return launch_store_mfma(c, K, V, n_layers, dt, T, stride, pt, n_seqs, max_pages, slots, nullptr, 0, st);
}

int launch_dequant(const saw_cache_t* c, const int32_t* pt, int32_t max_pages, int32_t seq,
                   int32_t pos_begin, int32_t pos_end, int32_t unrotate, float* k_out, float* v_out,
                   hipStream_t st) {
  DequantParams p;
  p.codes[0] = c->k_codes; p.codes[1] = c->v_codes;
  p.meta[0] = c->k_meta;   p.meta[1] = c->v_meta;
  p.out[0] = k_out; p.out[1] = v_out;
  p.page_table = pt; p.max_pages = max_pages; p.n_kv_heads = c->n_kv_heads; p.num_pages = c->num_pages;
  p.seq = seq; p.pos_begin = pos_begin; p.n_tokens = pos_end - pos_begin;
  p.had_block = c->had_block;
  p.unrot[0] = unrotate && (c->had_block > 1) && (c->rotate_mask & SAW_ROT_K);
  p.unrot[1] = unrotate && (c->had_block > 1) && (c->rotate_mask & SAW_ROT_V);
  for (int i = 0; i < 4; ++i) p.signs.w[i] = c->sign_bits[i];
  p.dense_t = c->dense_rot ? (const float*)((const uint8_t*)c->dense_rot + kDenseRtOffset) : nullptr;
  p.undense[0] = unrotate && c->dense_rot && (c->rotate_mask & SAW_ROT_K);
  p.undense[1] = unrotate && c->dense_rot && (c->rotate_mask & SAW_ROT_V);
  const int D = c->head_dim;
  const int vpb = 256 / (D / 8);
  const int64_t n_vec = (int64_t)p.n_tokens * c->n_kv_heads;
  dim3 grid((unsigned)((n_vec + vpb - 1) / vpb), 2), block(256);
  if (D == 128) dequant_pages_kernel<128><<<grid, block, 0, st>>>(p);
  else dequant_pages_kernel<64><<<grid, block, 0, st>>>(p);
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

int launch_kv16_store(const saw_cache_t* c, void* kp, void* vp, const void* K, const void* V, int64_t T,
                      int64_t stride, const int32_t* pt, int32_t n_seqs, int32_t max_pages,
                      const int32_t* slots, hipStream_t st) {
  Kv16StoreParams p;
  p.pages[0] = (uint16_t*)kp; p.pages[1] = (uint16_t*)vp;
  p.in[0] = K; p.in[1] = V; p.page_table = pt; p.slots = slots; p.T = T; p.token_stride = stride;
  p.n_seqs = n_seqs; p.max_pages = max_pages; p.num_pages = c->num_pages; p.n_kv_heads = c->n_kv_heads;
  const int D = c->head_dim;
  const int vpb = 256 / (D / 8);
  const int64_t n_vec = T * 2 * c->n_kv_heads;
  const int64_t blocks = (n_vec + vpb - 1) / vpb;
  if (blocks > 0x7fffffffLL) return SAW_EINVAL;
  dim3 grid((unsigned)blocks), block(256);
  if (D == 128) kv16_store_kernel<128><<<grid, block, 0, st>>>(p);
  else kv16_store_kernel<64><<<grid, block, 0, st>>>(p);
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

}  // namespace saw
