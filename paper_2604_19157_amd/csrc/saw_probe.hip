// Measurement aids (not part of the method): what the memory system delivers to a kernel that only
// READS an INT4 cache in the decode kernel's access pattern, and a plain vector-ALU INT4 store
// (no rotation, no matrix cores, no LDS staging) as the leanest "plain INT4" comparator for the fused
// rotate-quantise-store kernel (the quantiser is App. A.1's, the same formulas).
#include "saw_common.h"

namespace saw {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ReadProbeParams {
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const float* k_meta;
  const float* v_meta;
  const int32_t* page_ids;     // [n_pages]: the order in which pages are visited
  int64_t n_pages;
  int32_t n_kv_heads, num_pages;
  uint32_t* sink;              // one word per wavefront
};

// 2048 single-wavefront blocks, like the decode launch at the headline batch: wavefront w walks an
// equal share of the page list for kv head w % n_kv_heads in batches of four pages, 8 KiB of code tiles
// (1 KiB pieces: each lane 16 bytes) plus 1 KiB of (scale, zero) pairs per batch, one batch ahead, with
// the decode kernel's streaming cache policy.  Everything read is folded into one word per wavefront.
__global__ __launch_bounds__(64) void read_probe_kernel(ReadProbeParams p) {
  const int lane = threadIdx.x;
  const int head = blockIdx.x % p.n_kv_heads;
  const int64_t nw = gridDim.x / p.n_kv_heads;                 // wavefronts per head
  const int64_t w = blockIdx.x / p.n_kv_heads;
  const int64_t nb = (p.n_pages + 3) / 4;                      // batches of four pages
  const int64_t b0 = nb * w / nw, b1 = nb * (w + 1) / nw;
  const int64_t page_stride = (int64_t)p.n_kv_heads * 1024, page_meta = (int64_t)p.n_kv_heads * 32;
  u32x4 cur[9], nxt[9];
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  auto fetch = [&](int64_t b, u32x4 (&dst)[9]) {
    int ids[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int id = p.page_ids[min(4 * b + q, p.n_pages - 1)];
      ids[q] = (id < 0 || id >= p.num_pages) ? 0 : id;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      dst[q] = __builtin_nontemporal_load((const u32x4*)(p.k_codes + ids[q] * page_stride + head * 1024) + lane);
      dst[4 + q] = __builtin_nontemporal_load((const u32x4*)(p.v_codes + ids[q] * page_stride + head * 1024) + lane);
    }
    const int mq = (lane >> 3) & 3;
    const int id = mq == 0 ? ids[0] : mq == 1 ? ids[1] : mq == 2 ? ids[2] : ids[3];
    const float* mp = (lane < 32 ? p.k_meta : p.v_meta) + id * page_meta + head * 32 + 4 * (lane & 7);
    dst[8] = __builtin_nontemporal_load((const u32x4*)mp);
  };
  if (b0 < b1) fetch(b0, cur);
  for (int64_t b = b0; b < b1; ++b) {
    if (b + 1 < b1) fetch(b + 1, nxt);
#pragma unroll
    for (int i = 0; i < 9; ++i) acc ^= cur[i];
#pragma unroll
    for (int i = 0; i < 9; ++i) cur[i] = nxt[i];
  }
  const uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
  uint32_t r = v;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) r ^= __shfl_xor(r, m, 64);
  if (lane == 0) p.sink[blockIdx.x] = r;
}

// ---------------------------------------------------------------------------------------
// The longest-first order of a batch, computed on the device (no host read of the lengths): thread i
// counts the sequences that come before sequence i - longer (after clamping to the bound), or equally
// long with a lower index - and writes i at that rank.  One block; B <= 1024.  Run once per decode step,
// the order then serves every layer's hinted decode call.
__global__ __launch_bounds__(1024) void decode_order_kernel(const int32_t* __restrict__ seq_lens, int B, int bound,
                                                            int32_t* __restrict__ order) {
  __shared__ int lens[1024];
  const int i = threadIdx.x;
  if (i < B) lens[i] = max(min(seq_lens[i], bound), 0);
  __syncthreads();
  if (i >= B) return;
  const int mine = lens[i];
  int rank = 0;
  for (int j = 0; j < B; ++j) {
    const int l = lens[j];
    rank += (l > mine || (l == mine && j < i)) ? 1 : 0;
  }
  order[rank] = i;
}

int launch_decode_order(const int32_t* seq_lens, int B, int bound, int32_t* order, hipStream_t st) {
  decode_order_kernel<<<dim3(1), dim3(1024), 0, st>>>(seq_lens, B, bound, order);
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

int launch_read_probe(const saw_cache_t* c, const int32_t* page_ids, int64_t n_pages, void* sink, int32_t n_waves,
                      hipStream_t st) {
  ReadProbeParams p;
  p.k_codes = c->k_codes; p.v_codes = c->v_codes; p.k_meta = c->k_meta; p.v_meta = c->v_meta;
  p.page_ids = page_ids; p.n_pages = n_pages; p.n_kv_heads = c->n_kv_heads; p.num_pages = c->num_pages;
  p.sink = (uint32_t*)sink;
  read_probe_kernel<<<dim3(n_waves), dim3(64), 0, st>>>(p);
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

// ---------------------------------------------------------------------------------------
// Plain INT4 store on the vector ALU (head_dim 128, no rotation): 16 lanes hold one (token, head) vector,
// eight contiguous channels each; a block of 256 threads takes 16 consecutive tokens of the call for one
// (K|V, head), so a page-aligned run of tokens leaves as one 1 KiB code tile.
struct PlainStoreParams {
  uint8_t* codes[2];
  float* meta[2];
  const void* in[2];
  const int32_t* page_table;
  const int32_t* slots;
  int64_t T, token_stride;
  int32_t n_seqs, max_pages, num_pages, n_kv_heads;
};

template <int DT>
__global__ __launch_bounds__(256) void plain_store_valu_kernel(PlainStoreParams p) {
  constexpr int D = 128;
  const int tid = threadIdx.x, sub = tid & 15;
  const int64_t t = (int64_t)blockIdx.x * 16 + (tid >> 4);
  const int kind = blockIdx.y;
  const int which = kind >= p.n_kv_heads ? 1 : 0;
  const int head = kind - which * p.n_kv_heads;
  const bool live = t < p.T;
  const int64_t tt = live ? t : p.T - 1;
  const u32x4 raw = __builtin_nontemporal_load((const u32x4*)((const uint16_t*)p.in[which] + tt * p.token_stride + head * D) + sub);
  int2 slot = make_int2(-1, -1);
  if (live) slot = *(const int2*)(p.slots + 2 * t);
  float e[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) widen2<DT>(raw[i], e[2 * i], e[2 * i + 1]);
  float mn = e[0], mx = e[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) { mn = fminf(mn, e[i]); mx = fmaxf(mx, e[i]); }
#pragma unroll
  for (int m = 1; m < 16; m <<= 1) {
    mn = fminf(mn, __shfl_xor(mn, m, 64));
    mx = fmaxf(mx, __shfl_xor(mx, m, 64));
  }
  const float range = mx - mn;
  float inv, zq, s_store, z_store;
  if (range > 0.0f) {
    inv = 15.0f / range;
    s_store = range * (1.0f / 15.0f);
    zq = rintf(-mn * inv);
    z_store = zq;
  } else {  // constant vector
    inv = 0.0f;
    zq = 0.0f;
    s_store = (mn != 0.0f) ? fabsf(mn) : 1.0f;
    z_store = (mn > 0.0f) ? -1.0f : ((mn < 0.0f) ? 1.0f : 0.0f);
  }
  uint32_t w = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float c = __builtin_amdgcn_fmed3f(rintf(e[i] * inv) + zq, 0.0f, 15.0f);
    w |= ((uint32_t)c) << (4 * i);
  }
  const bool slot_ok = slot.x >= 0 && slot.x < p.n_seqs && slot.y >= 0 && (slot.y >> 4) < p.max_pages;
  if (!slot_ok) return;
  const int32_t page = p.page_table[(int64_t)slot.x * p.max_pages + (slot.y >> 4)];
  if (page < 0 || page >= p.num_pages) return;
  const int64_t vec = ((int64_t)page * p.n_kv_heads + head) * 16 + (slot.y & 15);
  __builtin_nontemporal_store(w, (uint32_t*)(p.codes[which] + vec * (D / 2)) + sub);
  if (sub == 0) *(float2*)(p.meta[which] + vec * 2) = make_float2(s_store, z_store);
}

int launch_plain_store_valu(const saw_cache_t* c, const void* K, const void* V, int dt, int64_t T, int64_t stride,
                            const int32_t* pt, int32_t n_seqs, int32_t max_pages, const int32_t* slots, hipStream_t st) {
  PlainStoreParams p;
  p.codes[0] = c->k_codes; p.codes[1] = c->v_codes;
  p.meta[0] = c->k_meta;   p.meta[1] = c->v_meta;
  p.in[0] = K; p.in[1] = V;
  p.page_table = pt; p.slots = slots; p.T = T; p.token_stride = stride;
  p.n_seqs = n_seqs; p.max_pages = max_pages; p.num_pages = c->num_pages; p.n_kv_heads = c->n_kv_heads;
  const int64_t tblocks = (T + 15) / 16;
  if (tblocks > 0x7fffffffLL || 2 * c->n_kv_heads > 65535) return SAW_EINVAL;
  dim3 grid((unsigned)tblocks, 2 * c->n_kv_heads), block(256);
  if (dt == SAW_BF16) plain_store_valu_kernel<SAW_BF16><<<grid, block, 0, st>>>(p);
  else plain_store_valu_kernel<SAW_F16><<<grid, block, 0, st>>>(p);
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

}  // namespace saw
