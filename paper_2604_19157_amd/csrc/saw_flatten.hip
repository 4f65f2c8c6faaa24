// Flatten-dequantise: a range of one sequence's INT4 pages -> a dense [n][kv_heads][d] K and/or V
// buffer in bf16 / fp16 / fp32, optionally rotated back (App. A.1: x^ = s (c - z); App. A.4:
// the block-diagonal Hadamard is symmetric and orthonormal, so the same matrix undoes it).
// This is the prefill-side consumer of the cache (App. B's flatten_dequant row): a chunked
// prefill attends over earlier chunks through this buffer.
//
// One wavefront takes one page (16 tokens) of one (K|V, kv head):
//   * the code tile (16 x d/2 bytes, contiguous) is read with coalesced 128-bit loads and passed
//     through LDS once (XOR chunk swizzle, conflict-free both ways) into the MFMA operand
//     layout, column = token;
//   * the nibbles become bf16 values 128 + c with one and-or per pair (exact), and the
//     Walsh-Hadamard transform over 32 contiguous channels is one pair of
//     v_mfma_f32_16x16x32_bf16 with a +/-1 matrix (block-diagonal for h = 16, identity when
//     nothing is to be rotated back), so every case runs the same instruction stream; orders
//     64 / 128 add register-to-register butterflies;
//   * everything up to here is exact integer arithmetic in fp32; the zero-point is taken out
//     afterwards: H (c + 128 - (z + 128)) = H (c + 128) - (z + 128) H 1, and H 1 is h at the
//     first channel of every block and 0 elsewhere, so a large zero-point cancels exactly
//     instead of through rounding;
//   * a lane ends up with eight contiguous output channels of one token for every 32-channel
//     group; 16-bit outputs are regrouped through LDS so that a store instruction writes whole
//     token rows (4 x 256 B for d = 128), fp32 outputs go out as two 16-byte stores per group.
#include "saw_common.h"

namespace saw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

struct FlattenParams {
  const uint8_t* codes[2];
  const float* meta[2];
  void* out[2];                 // null: tensor not wanted
  const int32_t* page_table;    // row of the sequence
  int64_t token_stride;         // output elements between tokens
  int32_t pos_begin, pos_end;
  int32_t first_page;           // pos_begin / 16
  int32_t num_pages, n_kv_heads, had_block;
  int32_t unrot[2];             // rotate this tensor back
  int32_t has_signs;            // any bit of `signs` set
  SignBits signs;               // R = diag(sigma) H_blk: rotating back ends with the signs
};

// HP = 2 ("head pair", for head_dim 64 with an even number of kv heads): the wavefront takes two
// neighbouring heads as one row of D = 128 values.  Their two code tiles are contiguous in the cache
// and their output rows are contiguous in the dense buffer; the tiles are re-ordered token-major
// on their way into LDS, after which everything runs as for head_dim 128 with per-head (scale, zero).
template <int D, int ODT, int HP = 1>
__global__ __launch_bounds__(256) void flatten_dequant_kernel(FlattenParams p) {
  constexpr int DH = D / HP;             // channels of one head
  constexpr int RB = D / 2;              // code bytes of one token's head vector or head pair (64 | 32)
  constexpr int XC = RB / 16;            // 16-byte chunks per vector (4 | 2)
  constexpr int NA = D / 32;             // 32-channel groups per vector (4 | 2)
  constexpr int FSH = (D == 128) ? 2 : 3;  // swizzle: chunk x of token t sits at x ^ ((t >> FSH) & (XC-1))
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n16 = lane & 15, rg = lane >> 4;
  const int n_heads_w = p.n_kv_heads / HP;                    // heads (or head pairs) of a tensor
  const int kind = blockIdx.x * 4 + wave;                     // (K|V, head or head pair)
  if (kind >= 2 * n_heads_w) return;
  const int which = kind >= n_heads_w ? 1 : 0;
  const int head = (kind - which * n_heads_w) * HP;           // (first) head of this wavefront
  if (p.out[which] == nullptr) return;
  const int lp = p.first_page + blockIdx.z * 65535 + blockIdx.y;   // logical page of the sequence
  if (16 * lp >= p.pos_end) return;
  const int pid = p.page_table[lp];
  if (pid < 0 || pid >= p.num_pages) return;                  // unmapped page: nothing written
  const bool unrot = p.unrot[which] != 0;

  __shared__ __attribute__((aligned(16))) uint8_t stage_all[4][16 * RB];
  __shared__ __attribute__((aligned(16))) uint8_t otile_all[(ODT == SAW_F32) ? 1 : 4][(ODT == SAW_F32) ? 16 : 16 * 2 * D];   // 16-bit outputs: a tile of output rows
  uint8_t* const stage = stage_all[wave];

  const uint8_t* tile = p.codes[which] + ((int64_t)pid * p.n_kv_heads + head) * (16 * (DH / 2));
  const float* mrow = p.meta[which] + ((int64_t)pid * p.n_kv_heads + head) * 32;
  if (lane < 16 * XC) {
    // 16-byte chunk `lane` of the tile(s): token tok, chunk x of the token's (pair) row
    int tok = lane / XC, x = lane % XC;
    if (HP == 2) {                                            // [head][token][32 B] -> token-major
      tok = (lane % 32) / 2;
      x = 2 * (lane / 32) + (lane % 2);
    }
    const u32x4 v = *(const u32x4*)(tile + 16 * lane);
    *(u32x4*)(stage + tok * RB + 16 * (x ^ ((tok >> FSH) & (XC - 1)))) = v;
  }
  float2 szh[HP];                                             // (scale, zero) of this lane's token, per head
#pragma unroll
  for (int hh = 0; hh < HP; ++hh) szh[hh] = *(const float2*)(mrow + 32 * hh + 2 * n16);

  // ---- the +/-1 matrix (see the store kernel): A[m][k], lane (m = n16, k-group = rg) ----
  // k runs over the nibble order the unpack produces: (n0, n4, n1, n5, n2, n6, n3, n7).
  const int hm = unrot ? min(p.had_block, 32) : 1;            // order handled inside the MFMA
  u32x4 ha1, ha2;
  {
    const int lo1 = 8 * (n16 >> 2) + (n16 & 3), lo2 = lo1 + 4;
    uint32_t e1[8], e2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int cl = 8 * rg + ((j & 1) ? 4 + (j >> 1) : (j >> 1));
      const bool on1 = (((lo1 ^ cl) & ~(hm - 1)) & 31) == 0;
      const bool on2 = (((lo2 ^ cl) & ~(hm - 1)) & 31) == 0;
      const uint32_t s1 = (__builtin_popcount(lo1 & cl & (hm - 1)) & 1) ? 0x8000u : 0u;
      const uint32_t s2 = (__builtin_popcount(lo2 & cl & (hm - 1)) & 1) ? 0x8000u : 0u;
      e1[j] = on1 ? (0x3F80u | s1) : 0u;
      e2[j] = on2 ? (0x3F80u | s2) : 0u;
    }
    ha1 = u32x4{e1[0] | (e1[1] << 16), e1[2] | (e1[3] << 16), e1[4] | (e1[5] << 16), e1[6] | (e1[7] << 16)};
    ha2 = u32x4{e2[0] | (e2[1] << 16), e2[2] | (e2[3] << 16), e2[4] | (e2[5] << 16), e2[6] | (e2[7] << 16)};
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  float y[8 * NA];                                             // y[8a + i]: channel 32a + 8rg + i of token n16
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    const uint32_t w = *(const uint32_t*)(stage + n16 * RB + 16 * (a ^ ((n16 >> FSH) & (XC - 1))) + 4 * rg);
    u32x4 bv;                                                  // eight bf16 values 128 + c
    bv.x = (w & 0x000F000Fu) | 0x43004300u;
    bv.y = ((w >> 4) & 0x000F000Fu) | 0x43004300u;
    bv.z = ((w >> 8) & 0x000F000Fu) | 0x43004300u;
    bv.w = ((w >> 12) & 0x000F000Fu) | 0x43004300u;
    const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
    const f32x4 d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ha1), __builtin_bit_cast(bf16x8, bv), zero, 0, 0, 0);
    const f32x4 d2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ha2), __builtin_bit_cast(bf16x8, bv), zero, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) { y[8 * a + i] = d1[i]; y[8 * a + 4 + i] = d2[i]; }
  }
  if (unrot && p.had_block >= 64) {
#pragma unroll
    for (int a = 0; a < NA; a += 2)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float u = y[8 * a + i], v = y[8 * a + 8 + i];
        y[8 * a + i] = u + v;
        y[8 * a + 8 + i] = u - v;
      }
  }
  if (D == 128 && unrot && p.had_block >= 128) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float u = y[8 * a + i], v = y[8 * a + 16 + i];
        y[8 * a + i] = u + v;
        y[8 * a + 16 + i] = u - v;
      }
  }

  // ---- zero-point and scale ----
  // un-rotated read-back: every channel carries (z + 128); rotated back: only the first channel
  // of each Hadamard block carries h (z + 128), the rest cancel exactly.
  const int h = unrot ? p.had_block : 1;
  float zoff_h[HP], sc_h[HP];
#pragma unroll
  for (int hh = 0; hh < HP; ++hh) {
    zoff_h[hh] = (szh[hh].y + 128.0f) * (float)h;
    sc_h[hh] = szh[hh].x * (unrot ? had_norm(p.had_block) : 1.0f);
  }
  constexpr int NAH = NA / HP;                                // 32-channel groups of one head
  const int pos = 16 * lp + n16;
  // Channel 32a + 8rg + i carries the zero-point term iff it is the first of its Hadamard block:
  // every channel when nothing is rotated back (h = 1), otherwise only i = 0 can be.
  if (ODT == SAW_F32) {
    if (pos < p.pos_begin || pos >= p.pos_end) return;
    const int64_t obase = (int64_t)(pos - p.pos_begin) * p.token_stride + head * DH;
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      const float zoff = zoff_h[a / NAH], sc = sc_h[a / NAH];
      float o[8];
      if (h == 1) {                                            // wavefront-uniform
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = sc * (y[8 * a + i] - zoff);
      } else {
        const bool first = ((32 * a + 8 * rg) & (h - 1)) == 0;
        o[0] = sc * (y[8 * a] - (first ? zoff : 0.0f));
#pragma unroll
        for (int i = 1; i < 8; ++i) o[i] = sc * y[8 * a + i];
      }
      if (p.has_signs && unrot) {                              // wavefront-uniform
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = apply_sign(p.signs, (32 * a + 8 * rg + i) % DH, o[i]);
      }
      float* dst = (float*)p.out[which] + obase + 32 * a + 8 * rg;
      *(f32x4*)dst = f32x4{o[0], o[1], o[2], o[3]};
      *(f32x4*)(dst + 4) = f32x4{o[4], o[5], o[6], o[7]};
    }
    return;
  }
  // 16-bit outputs: the tile's rows (one token's D values = 2 D bytes, contiguous in the output) are
  // put together in LDS, chunk c of row r at position c ^ (r & (NC - 1)), so that every store
  // instruction writes whole rows: 64 lanes x 16 bytes = 1 KiB = 1024 / (2 D) token rows.
  constexpr int NC = D / 8;                                    // 16-byte chunks per output row (16 | 8)
  constexpr int RPI = 64 / NC;                                 // rows per store instruction (4 | 8)
  uint8_t* const orow = otile_all[wave];
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    const float zoff = zoff_h[a / NAH], sc = sc_h[a / NAH];
    float o[8];
    if (h == 1) {                                              // wavefront-uniform
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = sc * (y[8 * a + i] - zoff);
    } else {
      const bool first = ((32 * a + 8 * rg) & (h - 1)) == 0;
      o[0] = sc * (y[8 * a] - (first ? zoff : 0.0f));
#pragma unroll
      for (int i = 1; i < 8; ++i) o[i] = sc * y[8 * a + i];
    }
    // round-to-nearest-even pairs: v_cvt_pk_bf16_f32, or two v_cvt_f16_f32 and a pack
    uint32_t w4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x2 pr = f32x2{o[2 * i], o[2 * i + 1]};
      if (ODT == SAW_BF16) w4[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
      else w4[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, f16x2));
    }
    if (p.has_signs && unrot) {                                // wavefront-uniform
      uint32_t sx[4];
      sign_pairs(p.signs, (32 * a + 8 * rg) % DH, sx);
#pragma unroll
      for (int i = 0; i < 4; ++i) w4[i] ^= sx[i];
    }
    const int c = 4 * a + rg;
    *(u32x4*)(orow + n16 * (2 * D) + 16 * (c ^ (n16 & (NC - 1)))) = u32x4{w4[0], w4[1], w4[2], w4[3]};
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int j = 0; j < 16 / RPI; ++j) {
    const int r = RPI * j + lane / NC, c = lane % NC;
    const int rpos = 16 * lp + r;
    const u32x4 v = *(const u32x4*)(orow + r * (2 * D) + 16 * (c ^ (r & (NC - 1))));
    if (rpos >= p.pos_begin && rpos < p.pos_end)
      *(u32x4*)((uint16_t*)p.out[which] + (int64_t)(rpos - p.pos_begin) * p.token_stride + head * DH + 8 * c) = v;
  }
}

int launch_flatten(const saw_cache_t* c, const int32_t* pt_row, int32_t pos_begin, int32_t pos_end,
                   int32_t unrotate, int32_t out_dtype, void* k_out, void* v_out, int64_t token_stride,
                   hipStream_t st) {
  FlattenParams p;
  p.codes[0] = c->k_codes; p.codes[1] = c->v_codes;
  p.meta[0] = c->k_meta;   p.meta[1] = c->v_meta;
  p.out[0] = k_out;        p.out[1] = v_out;
  p.page_table = pt_row;
  p.token_stride = token_stride;
  p.pos_begin = pos_begin; p.pos_end = pos_end;
  p.first_page = pos_begin / 16;
  p.num_pages = c->num_pages; p.n_kv_heads = c->n_kv_heads; p.had_block = c->had_block;
  const bool rot = unrotate && c->had_block > 1;
  p.unrot[0] = rot && (c->rotate_mask & SAW_ROT_K);
  p.unrot[1] = rot && (c->rotate_mask & SAW_ROT_V);
  for (int i = 0; i < 4; ++i) p.signs.w[i] = c->sign_bits[i];
  p.has_signs = (c->sign_bits[0] | c->sign_bits[1] | c->sign_bits[2] | c->sign_bits[3]) != 0;
  const int n_pages = (pos_end + 15) / 16 - p.first_page;
  // (K|V, head) groups vary fastest, so blocks that run together write neighbouring pieces of the
  // same token rows
  const bool pair64 = c->head_dim == 64 && (c->n_kv_heads % 2) == 0;   // two 64-channel heads per wavefront
  dim3 grid((2 * (c->n_kv_heads / (pair64 ? 2 : 1)) + 3) / 4, n_pages < 65535 ? n_pages : 65535, (n_pages + 65534) / 65535), block(256);
#define SAW_FLAT(DD, HH)                                                                          \
  switch (out_dtype) {                                                                            \
    case SAW_BF16: flatten_dequant_kernel<DD, SAW_BF16, HH><<<grid, block, 0, st>>>(p); break;     \
    case SAW_F16: flatten_dequant_kernel<DD, SAW_F16, HH><<<grid, block, 0, st>>>(p); break;       \
    default: flatten_dequant_kernel<DD, SAW_F32, HH><<<grid, block, 0, st>>>(p); break;            \
  }
  if (pair64) { SAW_FLAT(128, 2) } else if (c->head_dim == 128) { SAW_FLAT(128, 1) } else { SAW_FLAT(64, 1) }
#undef SAW_FLAT
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

}  // namespace saw
