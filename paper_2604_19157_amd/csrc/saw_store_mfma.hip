// Fused rotate -> token-wise INT4 quantise -> pack -> paged store on the gfx950 matrix cores.
// Paper: Sec. 3 eqs. (1)-(3) (K~ = quant(K H_blk)), App. A.1 (s, z, codes, nibble packing),
// App. A.4 (block-diagonal Hadamard of order h | d).
//
// One wavefront takes 16 consecutive tokens of one (K|V, kv head): a 16 x D tile of 16-bit values.
//   * the tile is read with coalesced 128-bit loads (each 16-lane row reads 256 contiguous
//     bytes) and passed through LDS once, with an XOR chunk swizzle that keeps both sides free
//     of bank conflicts, to reach the MFMA operand layout (column = token);
//   * the Walsh-Hadamard transform over the low five channel bits (32 contiguous channels) is one
//     pair of v_mfma_f32_16x16x32 with a +/-1 matrix: the 16-bit inputs are the B operand as they
//     are (no widening), products with +/-1 are exact and the sums accumulate in fp32.  The
//     matrix also encodes smaller orders (block-diagonal for h = 16, identity for h = 1), so
//     every Hadamard order runs the same instruction stream; its rows are ordered so that a
//     lane ends up with eight *contiguous* output channels;
//   * a lane ends up with 8 values of each 32-channel group of ONE token, so the one or two
//     remaining butterfly stages of orders 64 and 128 are register-to-register;
//   * min/max: in-lane, then across the four 16-lane rows that hold the same token;
//   * quantise with a reciprocal multiply, pack eight nibbles per dword; when the 16 tokens are
//     the 16 slots of one page (prefill) the code dwords are transposed through LDS and leave as
//     one contiguous 1 KiB tile write, otherwise as per-token dword stores.
// The transform is un-normalised; 1/sqrt(h) is folded into the stored scale (codes unchanged).
#include "saw_common.h"

namespace saw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One launch can serve several layers (grid.z): the layers share the slots, the page table and the
// cache shape, and differ in their pools, their inputs and their learned rotation.
constexpr int kMaxStoreLayers = 32;
struct StoreLayerPtrs {
  uint8_t* codes[2];
  float* meta[2];
  const void* in[2];
  const void* dense_limbs;      // learned rotation R_l (App. A.3) as bf16 limb operands, see saw_common.h; or null
};
struct StoreMfmaParams {
  StoreLayerPtrs layer[kMaxStoreLayers];
  const int32_t* page_table;
  const int32_t* slots;         // [T][2] (sequence, position), or null:
  const int32_t* append_lens;   // then token t goes to sequence t at position append_lens[t],
  int32_t append_bound;         // unless that exceeds append_bound (the caller's bound on the lengths): skipped
  int64_t T;
  int64_t token_stride;
  int32_t n_seqs, max_pages, num_pages, n_kv_heads;
  int32_t had_block;
  int32_t rot[2];
  int32_t has_signs;            // any bit of `signs` set
  SignBits signs;               // diagonal in front of the Hadamard matrix (rotated tensors only)
  int32_t dense_on[2];          // R_l follows the Hadamard for K / for V
  int32_t kblocks;              // blocks that cover the (K|V, head) combinations of one token group
  int32_t kinds_fastest;        // block order: see launch_store_mfma
};

template <int DT>
__device__ __forceinline__ f32x4 mfma_pm1(u32x4 a, u32x4 b, f32x4 c) {
  if (DT == SAW_BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <int CTRL>
__device__ __forceinline__ float dppf(float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xf, 0xf, false));
}

// XS = number of register-to-register butterfly stages after the MFMA (0: h <= 32 or no rotation,
// 1: h = 64, 2: h = 128) when K and V agree; XS = -1 decides per wavefront at run time (K-only
// or V-only rotation).
// HP = 2 ("head pair", for head_dim 64 with an even number of kv heads): the wavefront takes two
// neighbouring heads of 64 channels as one row of D = 128 values (they are contiguous in the input
// and their code tiles and metadata are contiguous in the cache), so that loads, staging and the
// matrix products run exactly as for head_dim 128; only the min/max, the scales and the addresses
// are per head.
// DENSE (D = 128, one head per wavefront): a learned per-layer rotation follows the Hadamard, y = (x H_blk) R_l
// (App. A.3).  The Hadamard output of a lane - eight channels of each 32-channel group of one token - is
// already the B operand of a v_mfma_f32_16x16x32_bf16 over that group, so it is split into three bf16 limbs
// in registers (hi + mid + lo = the fp32 value to 24 bits) and multiplied by the three limbs of R_l, which
// arrive as ready-made A operands from the prepared buffer (224 KiB, cache-resident): the six limb products
// that matter (everything down to 2^-24 of the result), smallest first, accumulated in fp32.  The rows of the
// A operands are ordered so that the result lands in the very lane layout the quantiser below expects.
template <int D, int DT, int XS, int HP = 1, bool DENSE = false>
__global__ __launch_bounds__(256) void rotate_quant_store_mfma_kernel(StoreMfmaParams p) {
  static_assert(!DENSE || (D == 128 && HP == 1), "the learned rotation is built for head_dim 128");
  constexpr int DH = D / HP;             // channels of one head (D itself unless HP = 2: then 64)
  constexpr int ROWB = D * 2;            // bytes of one token's head vector (or head pair)
  constexpr int XC = ROWB / 16;          // 16-byte chunks per vector (16 | 8)
  constexpr int NA = D / 32;             // 32-channel groups per vector (4 | 2)
  constexpr int RP = 256 / ROWB;         // token rows per 256 bytes of LDS (1 | 2)
  constexpr int NLD = (16 * ROWB) / 1024;  // 128-bit loads per lane (4 | 2)
  constexpr int NV = 8 * NA;             // output values per lane
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, rg = lane >> 4;
  const int n_heads_w = p.n_kv_heads / HP;                    // heads (or head pairs) a tensor has
  const int n_kinds = 2 * n_heads_w;                          // (K|V, head or head pair) combinations
  const int kb_id = p.kinds_fastest ? (int)(blockIdx.x % p.kblocks) : (int)blockIdx.y;
  const int64_t tb_id = p.kinds_fastest ? (int64_t)(blockIdx.x / p.kblocks) : (int64_t)blockIdx.x;
  const int kind_raw = kb_id * 4 + __builtin_amdgcn_readfirstlane(wave);
  const bool wave_live = kind_raw < n_kinds;                  // wave-uniform
  const int kind = wave_live ? kind_raw : 0;                  // an idle wavefront shadows kind 0 and stores nothing
  const int which = kind >= n_heads_w ? 1 : 0;
  const int head = (kind - which * n_heads_w) * HP;           // (first) head of this wavefront
  // DENSE: a wavefront takes NT = 2 consecutive 16-token tiles, so that one set of limb operands of R_l
  // (96 KB per wavefront through L1) serves twice the tokens.
  constexpr int NT = DENSE ? 2 : 1;
  const int64_t t0 = tb_id * (16 * NT);
  const bool rot = p.rot[which] != 0;
  const StoreLayerPtrs& lp = p.layer[blockIdx.z];

  __shared__ __attribute__((aligned(16))) uint8_t stage_all[4][16 * ROWB];
  uint8_t* const stage = stage_all[wave];

  // ---- issue the tile loads (coalesced: each 16-lane row reads 256 contiguous bytes) ----
  u32x4 ld[NT][NLD];
  int2 slot[NT];
#pragma unroll
  for (int tile = 0; tile < NT; ++tile) {
#pragma unroll
    for (int r = 0; r < NLD; ++r) {
      const int off = r * 1024 + 16 * lane;                    // byte offset in the dense 16 x D tile
      const int tok = off / ROWB, x = (off % ROWB) / 16;
      const int64_t t = min(t0 + 16 * tile + tok, p.T - 1);    // tokens past the end shadow the last one; never stored
      // (the input is read once and the cache written once: both are marked streaming, "nt")
      ld[tile][r] = __builtin_nontemporal_load((const u32x4*)((const uint16_t*)lp.in[which] + t * p.token_stride + head * DH + 8 * x));
    }
    // this lane's token (column n16 of the tile) and where it goes
    const int64_t t_mine = t0 + 16 * tile + n16;
    slot[tile] = make_int2(-1, -1);
    if (wave_live && t_mine < p.T)
      slot[tile] = p.slots ? *(const int2*)(p.slots + 2 * t_mine) : make_int2((int)t_mine, p.append_lens[t_mine]);
    if (!p.slots && slot[tile].y > p.append_bound) slot[tile] = make_int2(-1, -1);
  }

  // ---- the +/-1 matrix: A[m][k], m = output row, k = input channel (low five bits) ----
  // MFMA #1 row m -> output channel (low five bits) 8*(m/4) + m%4, MFMA #2 row m -> that + 4,
  // so lane (n16, rg) receives channels 8*rg .. 8*rg+7 of every 32-channel group.
  // Entry = (-1)^popcount(lo & k & (hm-1)) where the bits above the order hm agree, else 0.
  const int hm = rot ? min(p.had_block, 32) : 1;              // order handled inside the MFMA
  u32x4 ha1, ha2;
  {
    const uint32_t one = (DT == SAW_BF16) ? 0x3F80u : 0x3C00u;
    const int lo1 = 8 * (n16 >> 2) + (n16 & 3);                // A operand: lane (m = n16, k-group = rg)
    uint32_t e1[8], e2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int cl = 8 * rg + j;
      const int lo2 = lo1 + 4;
      const bool on1 = (((lo1 ^ cl) & ~(hm - 1)) & 31) == 0;
      const bool on2 = (((lo2 ^ cl) & ~(hm - 1)) & 31) == 0;
      const uint32_t s1 = (__builtin_popcount(lo1 & cl & (hm - 1)) & 1) ? 0x8000u : 0u;
      const uint32_t s2 = (__builtin_popcount(lo2 & cl & (hm - 1)) & 1) ? 0x8000u : 0u;
      e1[j] = on1 ? (one | s1) : 0u;
      e2[j] = on2 ? (one | s2) : 0u;
    }
    ha1 = u32x4{e1[0] | (e1[1] << 16), e1[2] | (e1[3] << 16), e1[4] | (e1[5] << 16), e1[6] | (e1[7] << 16)};
    ha2 = u32x4{e2[0] | (e2[1] << 16), e2[2] | (e2[3] << 16), e2[4] | (e2[5] << 16), e2[6] | (e2[7] << 16)};
  }

  // Randomised Hadamard: x . diag(sigma) is a sign flip of the 16-bit inputs (exact), applied at the
  // staging step because a lane's chunk index (lane % (ROWB / 16)) is the same for all of its loads: one mask.
  u32x4 sflip = u32x4{0u, 0u, 0u, 0u};
  if (p.has_signs && rot) {                                     // wavefront-uniform
    uint32_t sx[4];
    sign_pairs(p.signs, (8 * (lane % (ROWB / 16))) % DH, sx);
    sflip = u32x4{sx[0], sx[1], sx[2], sx[3]};
  }

  float y[NT][NV];                                              // y[.][8a + i]: channel 32a + 8rg + i of token n16
#pragma unroll
  for (int tile = 0; tile < NT; ++tile) {
    // ---- through LDS into the B-operand layout: column = token, k-group rg = chunk 4a + rg ----
    // chunk x of token tok sits at chunk position x ^ ((tok / RP) & (XC-1)): both the row-wise
    // writes and the column-wise reads below touch every bank once.
#pragma unroll
    for (int r = 0; r < NLD; ++r) {
      const int off = r * 1024 + 16 * lane;
      const int tok = off / ROWB, x = (off % ROWB) / 16;
      *(u32x4*)(stage + tok * ROWB + 16 * (x ^ ((tok / RP) & (XC - 1)))) = ld[tile][r] ^ sflip;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      const int x = 4 * a + rg;
      const u32x4 bv = *(const u32x4*)(stage + n16 * ROWB + 16 * (x ^ ((n16 / RP) & (XC - 1))));
      const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
      const f32x4 d1 = mfma_pm1<DT>(ha1, bv, zero);
      const f32x4 d2 = mfma_pm1<DT>(ha2, bv, zero);
#pragma unroll
      for (int i = 0; i < 4; ++i) { y[tile][8 * a + i] = d1[i]; y[tile][8 * a + 4 + i] = d2[i]; }
    }
    if (NT > 1) {                                               // the next tile's staging overwrites what was just read
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    // ---- orders 64 / 128: butterflies across the 32-channel groups, now register to register ----
    if (XS >= 1 || (XS < 0 && rot && p.had_block >= 64)) {
#pragma unroll
      for (int a = 0; a < NA; a += 2)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float u = y[tile][8 * a + i], v = y[tile][8 * a + 8 + i];
          y[tile][8 * a + i] = u + v;
          y[tile][8 * a + 8 + i] = u - v;
        }
    }
    if (D == 128 && (XS >= 2 || (XS < 0 && rot && p.had_block >= 128))) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float u = y[tile][8 * a + i], v = y[tile][8 * a + 16 + i];
          y[tile][8 * a + i] = u + v;
          y[tile][8 * a + 16 + i] = u - v;
        }
    }
  }
  if constexpr (DENSE) {
    if (p.dense_on[which]) {                                    // wavefront-uniform
      typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
      typedef float f32x2_t __attribute__((ext_vector_type(2)));
      u32x4 bh[NT][NA], bm[NT][NA], bl[NT][NA];                 // limbs of y as B operands, one per k-step (32 channels)
#pragma unroll
      for (int tile = 0; tile < NT; ++tile) {
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          uint32_t wh[4], wm[4], wl[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float y0 = y[tile][8 * a + 2 * e], y1 = y[tile][8 * a + 2 * e + 1];
            wh[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{y0, y1}, bf16x2_t));
            const float r0 = y0 - __uint_as_float(wh[e] << 16), r1 = y1 - __uint_as_float(wh[e] & 0xffff0000u);
            wm[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{r0, r1}, bf16x2_t));
            const float q0 = r0 - __uint_as_float(wm[e] << 16), q1 = r1 - __uint_as_float(wm[e] & 0xffff0000u);
            wl[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{q0, q1}, bf16x2_t));
          }
          bh[tile][a] = u32x4{wh[0], wh[1], wh[2], wh[3]};
          bm[tile][a] = u32x4{wm[0], wm[1], wm[2], wm[3]};
          bl[tile][a] = u32x4{wl[0], wl[1], wl[2], wl[3]};
        }
      }
      const u32x4* const A = (const u32x4*)lp.dense_limbs + lane;
#pragma unroll
      for (int J = 0; J < 8; ++J) {
        u32x4 ah[NA], am[NA], al[NA];
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          ah[a] = A[((0 * 8 + J) * 4 + a) * 64];
          am[a] = A[((1 * 8 + J) * 4 + a) * 64];
          al[a] = A[((2 * 8 + J) * 4 + a) * 64];
        }
#pragma unroll
        for (int tile = 0; tile < NT; ++tile) {
          f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#define SAW_LIMB_PRODUCT(RA, YB)                                                                     \
  _Pragma("unroll") for (int a = 0; a < NA; ++a)                                                     \
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, RA[a]), __builtin_bit_cast(bf16x8, YB[tile][a]), acc, 0, 0, 0);
          SAW_LIMB_PRODUCT(al, bh)
          SAW_LIMB_PRODUCT(ah, bl)
          SAW_LIMB_PRODUCT(am, bm)
          SAW_LIMB_PRODUCT(am, bh)
          SAW_LIMB_PRODUCT(ah, bm)
          SAW_LIMB_PRODUCT(ah, bh)
#undef SAW_LIMB_PRODUCT
          // tile J holds channels 32 (J / 2) + 8 rg + 4 (J % 2) + 0..3 of token n16
#pragma unroll
          for (int i = 0; i < 4; ++i) y[tile][8 * (J >> 1) + 4 * (J & 1) + i] = acc[i];
        }
      }
    }
  }
  const float norm = rot ? had_norm(p.had_block) : 1.0f;
  if (!wave_live) return;

#pragma unroll
  for (int tile = 0; tile < NT; ++tile) {
    // ---- token-wise min / max per head: in-lane, then the four rows holding the same token ----
    constexpr int NVH = NV / HP;                                // this lane's values of one head
    float s_store[HP], z_store[HP];
    uint32_t packed[NA];
#pragma unroll
    for (int hh = 0; hh < HP; ++hh) {
      float mn = y[tile][NVH * hh], mx = y[tile][NVH * hh];
#pragma unroll
      for (int i = 1; i < NVH; ++i) { mn = fminf(mn, y[tile][NVH * hh + i]); mx = fmaxf(mx, y[tile][NVH * hh + i]); }
      mn = fminf(mn, __shfl_xor(mn, 16, 64)); mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mn = fminf(mn, __shfl_xor(mn, 32, 64)); mx = fmaxf(mx, __shfl_xor(mx, 32, 64));

      // ---- scale / zero (App. A.1), quantise, pack ----
      const float range = mx - mn;
      float inv, zq;
      if (range > 0.0f) {
        inv = 15.0f / range;
        s_store[hh] = range * (norm * (1.0f / 15.0f));
        zq = rintf(-mn * inv);
        z_store[hh] = zq;
      } else {  // constant vector
        inv = 0.0f;
        zq = 0.0f;
        s_store[hh] = (mn != 0.0f) ? fabsf(mn) * norm : 1.0f;
        z_store[hh] = (mn > 0.0f) ? -1.0f : ((mn < 0.0f) ? 1.0f : 0.0f);
      }
#pragma unroll
      for (int a = (NA / HP) * hh; a < (NA / HP) * (hh + 1); ++a) {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float c = rintf(y[tile][8 * a + i] * inv) + zq;
          c = __builtin_amdgcn_fmed3f(c, 0.0f, 15.0f);
          w |= ((uint32_t)c) << (4 * i);
        }
        packed[a] = w;                                          // dword 4 (a % (NA / HP)) + rg of the token's code row of head hh
      }
    }

    // ---- paged placement ----
    const int2 sl = slot[tile];
    int32_t page = -1;
    const bool slot_ok = sl.x >= 0 && sl.x < p.n_seqs && sl.y >= 0 && (sl.y >> 4) < p.max_pages;
    if (slot_ok) page = p.page_table[(int64_t)sl.x * p.max_pages + (sl.y >> 4)];
    const bool ok = slot_ok && page >= 0 && page < p.num_pages;
    // fast path: the 16 tokens are the 16 slots of one page, in order
    const int seq0 = __builtin_amdgcn_readfirstlane(sl.x);
    const int pos0 = __builtin_amdgcn_readfirstlane(sl.y);
    const bool aligned = __all(ok && sl.x == seq0 && sl.y == pos0 + n16) && ((pos0 & 15) == 0);
    constexpr int NAH = NA / HP;                                // 32-channel groups of one head
    if (aligned) {                                              // wavefront-uniform
      const int page0 = __builtin_amdgcn_readfirstlane(page);
      const int64_t vec0 = ((int64_t)page0 * p.n_kv_heads + head) * 16;
      // transpose the code dwords through LDS so that every lane writes 16 contiguous bytes
      // (a head pair's two tiles follow each other in the cache, so they leave as one run)
      uint32_t* const ob = (uint32_t*)stage;                   // [head of the pair][token][DH/8 dwords]
#pragma unroll
      for (int a = 0; a < NA; ++a) ob[(a / NAH) * (16 * DH / 8) + n16 * (DH / 8) + 4 * (a % NAH) + rg] = packed[a];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if (lane < 16 * (D / 2) / 16)
        __builtin_nontemporal_store(*(const u32x4*)(stage + 16 * lane), (u32x4*)(lp.codes[which] + vec0 * (DH / 2) + 16 * lane));
#pragma unroll
      for (int hh = 0; hh < HP; ++hh)
        if (rg == hh) *(float2*)(lp.meta[which] + (vec0 + 16 * hh + n16) * 2) = make_float2(s_store[hh], z_store[hh]);
      if (NT > 1) {                                             // the next tile's transposition reuses the buffer
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    } else if (ok) {
#pragma unroll
      for (int hh = 0; hh < HP; ++hh) {
        const int64_t vec = ((int64_t)page * p.n_kv_heads + head + hh) * 16 + (sl.y & 15);
#pragma unroll
        for (int a = NAH * hh; a < NAH * (hh + 1); ++a) ((uint32_t*)(lp.codes[which] + vec * (DH / 2)))[4 * (a % NAH) + rg] = packed[a];
        if (rg == hh) *(float2*)(lp.meta[which] + vec * 2) = make_float2(s_store[hh], z_store[hh]);
      }
    }
  }
}

// `c`, `K`, `V`: n_layers cache descriptors and input pointers (host arrays); the layers agree in shape,
// Hadamard block, mask and signs (checked by the caller).
int launch_store_mfma(const saw_cache_t* c, const void* const* K, const void* const* V, int n_layers, int dt,
                      int64_t T, int64_t stride,
                      const int32_t* pt, int32_t n_seqs, int32_t max_pages, const int32_t* slots,
                      const int32_t* append_lens, int32_t append_bound,
                      hipStream_t st) {
  StoreMfmaParams p;
  for (int l = 0; l < n_layers; ++l) {
    StoreLayerPtrs& lp = p.layer[l];
    lp.codes[0] = c[l].k_codes; lp.codes[1] = c[l].v_codes;
    lp.meta[0] = c[l].k_meta;   lp.meta[1] = c[l].v_meta;
    lp.in[0] = K[l]; lp.in[1] = V[l];
    lp.dense_limbs = c[l].dense_rot ? (const uint8_t*)c[l].dense_rot + kDenseLimbOffset : nullptr;
  }
  p.page_table = pt; p.slots = slots; p.append_lens = append_lens; p.append_bound = append_bound; p.T = T; p.token_stride = stride;
  p.n_seqs = n_seqs; p.max_pages = max_pages; p.num_pages = c->num_pages; p.n_kv_heads = c->n_kv_heads;
  p.had_block = c->had_block;
  p.rot[0] = (c->had_block > 1) && (c->rotate_mask & SAW_ROT_K);
  p.rot[1] = (c->had_block > 1) && (c->rotate_mask & SAW_ROT_V);
  for (int i = 0; i < 4; ++i) p.signs.w[i] = c->sign_bits[i];
  p.has_signs = (c->sign_bits[0] | c->sign_bits[1] | c->sign_bits[2] | c->sign_bits[3]) != 0;
  p.dense_on[0] = c->dense_rot && (c->rotate_mask & SAW_ROT_K);
  p.dense_on[1] = c->dense_rot && (c->rotate_mask & SAW_ROT_V);
  const int D = c->head_dim;
  const int tile_tokens = (p.dense_on[0] || p.dense_on[1]) ? 32 : 16;   // tokens per wavefront (the DENSE kernel takes two tiles)
  const int64_t tblocks = (T + tile_tokens - 1) / tile_tokens;
  if (tblocks > 0x7fffffffLL) return SAW_EINVAL;
  const bool pair64 = D == 64 && (c->n_kv_heads % 2) == 0;      // two 64-channel heads per wavefront
  const int kblocks = (2 * (c->n_kv_heads / (pair64 ? 2 : 1)) + 3) / 4;
  if (kblocks > 65535) return SAW_EINVAL;
  dim3 grid((unsigned)tblocks, kblocks, n_layers), block(256);
  // Block order.  With many (K|V, head) combinations per token (a token's K row of 4 KB or more: the MHA
  // shape with 32 heads of 64) the blocks of one token group run next to each other, so that blocks in
  // flight together read neighbouring pieces of the same input rows: 76.3 -> 69.7 us on the 32k-token MHA
  // prefill.  With 2 KB rows (8 heads of 128) the token groups are the fastest index: 34.0 against 34.7 us.
  p.kblocks = kblocks;
  p.kinds_fastest = 0;
  if (kblocks >= 8 && tblocks * kblocks < 0x7fffffffLL) {
    p.kinds_fastest = 1;
    grid = dim3((unsigned)(tblocks * kblocks), 1, n_layers);
  }
  const int h = c->had_block;
  int xs = -1;                                                  // static stage count when K and V agree
  if (p.rot[0] == p.rot[1]) xs = !p.rot[0] ? 0 : (h >= 128 ? 2 : (h >= 64 ? 1 : 0));
#define SAW_LAUNCH(DD, TT)                                                                             \
  switch (xs) {                                                                                        \
    case 0: rotate_quant_store_mfma_kernel<DD, TT, 0><<<grid, block, 0, st>>>(p); break;               \
    case 1: rotate_quant_store_mfma_kernel<DD, TT, 1><<<grid, block, 0, st>>>(p); break;               \
    case 2: rotate_quant_store_mfma_kernel<DD, TT, (DD == 128 ? 2 : 1)><<<grid, block, 0, st>>>(p); break; \
    default: rotate_quant_store_mfma_kernel<DD, TT, -1><<<grid, block, 0, st>>>(p); break;             \
  }
#define SAW_LAUNCH_PAIR(TT)                                                                             \
  switch (xs) {                                                                                        \
    case 0: rotate_quant_store_mfma_kernel<128, TT, 0, 2><<<grid, block, 0, st>>>(p); break;           \
    case 1: case 2: rotate_quant_store_mfma_kernel<128, TT, 1, 2><<<grid, block, 0, st>>>(p); break;   \
    default: rotate_quant_store_mfma_kernel<128, TT, -1, 2><<<grid, block, 0, st>>>(p); break;         \
  }
  if (p.dense_on[0] || p.dense_on[1]) {                         // head_dim 128 (checked by the caller)
    if (dt == SAW_BF16) rotate_quant_store_mfma_kernel<128, SAW_BF16, -1, 1, true><<<grid, block, 0, st>>>(p);
    else rotate_quant_store_mfma_kernel<128, SAW_F16, -1, 1, true><<<grid, block, 0, st>>>(p);
  }
  else if (pair64 && dt == SAW_BF16) { SAW_LAUNCH_PAIR(SAW_BF16) }
  else if (pair64) { SAW_LAUNCH_PAIR(SAW_F16) }
  else if (D == 128 && dt == SAW_BF16) { SAW_LAUNCH(128, SAW_BF16) }
  else if (D == 128) { SAW_LAUNCH(128, SAW_F16) }
  else if (dt == SAW_BF16) { SAW_LAUNCH(64, SAW_BF16) }
  else { SAW_LAUNCH(64, SAW_F16) }
#undef SAW_LAUNCH
#undef SAW_LAUNCH_PAIR
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

}  // namespace saw
