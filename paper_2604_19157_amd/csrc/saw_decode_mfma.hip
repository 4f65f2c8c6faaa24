// INT4 paged decode attention for head_dim 128 on the gfx950 matrix cores.
// Paper: Sec. 2 (decode step), Sec. 4.1 / App. A.4 (rotated-space attention), App. A.1.
//
// One wavefront (a 64-thread block) owns one (sequence, kv head, context partition) and walks
// it in batches of four pages (64 tokens).  Per batch:
//   * the four K and four V code tiles (1 KiB each, contiguous in HBM) are fetched one
//     batch ahead into registers and dropped into LDS with a 16-byte-chunk swizzle
//     pos(t, Q) = 4t + ((Q + t/4) & 3) that makes every later LDS read bank-conflict free;
//   * nibbles become bf16 operands with two ALU ops per pair: (w >> 4i) & 0x000F000F | 0x43004300
//     is the bf16 pair (128 + c_lo, 128 + c_hi); the constant 128 joins the zero-point;
//   * logits: D[head][token] = q~ (heads x channels) . codes (channels x tokens) with
//     v_mfma_f32_16x16x32_bf16; q~ is carried as bf16 hi + lo limbs in separate rows of the
//     tile (~16 bits together), added after the gather below;
//   * the four pages' result rows are gathered with v_permlane16/32_swap so that lane =
//     token of the batch and registers = heads: the softmax runs on all 64 lanes;
//   * the running maximum is a lazily updated reference: it only moves (with a rescale of
//     the accumulators) when some logit exceeds it by more than 2^8;
//   * P.V needs tokens along the contraction: ds_read_b64_tr_b4 hands each lane the 16
//     tokens of one channel (a 16x16 nibble transpose inside LDS); P goes through LDS once as
//     bf16 hi/lo rows; O[head][channel] accumulates in eight 16x16 tiles.
// Zero-points never enter the loops:  q~.k^ = s (q~.(c+128) - (z+128) sum q~),
// sum_t w_t v^_t = sum_t w_t (c_t+128) - sum_t w_t (z_t+128),  w_t = p_t s_t.
#include "saw_decode.h"

namespace saw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define LDS_AS __attribute__((address_space(3)))

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

// In-place un-normalised block Walsh-Hadamard transform of n_vec vectors of 128 floats in LDS,
// run by one wavefront (the block is a single wave, so __syncthreads is a wave-level fence).
__device__ __forceinline__ void wave_lds_fwht128(float* x, int n_vec, int h, int lane) {
  for (int st = 1; st < h; st <<= 1) {
    for (int idx = lane; idx < n_vec * 64; idx += 64) {
      const int v = idx >> 6, r = idx & 63;
      const int i = v * 128 + (r / st) * 2 * st + (r % st);
      const float a = x[i], c = x[i + st];
      x[i] = a + c;
      x[i + st] = a - c;
    }
    __syncthreads();
  }
}

constexpr int kTileBytes = 1024;               // one (page, head) code tile: 16 tokens x 64 B
constexpr int kStageBytes = 8 * kTileBytes;    // four K tiles then four V tiles
constexpr int kProw = 72;                      // P row stride in bf16 (64 tokens + 8 pad: conflict-free b128 reads)
constexpr int kPbufBytes = 16 * kProw * 2;     // P as bf16 [16 rows][64 tokens]
constexpr float kLazyTau = 8.0f;               // reference max may lag the true max by 2^8

template <int G>
__global__ __launch_bounds__(64) void decode_int4_mfma_kernel(DecodeParams p) {
  constexpr int D = 128;
  constexpr int NS = (G > 4) ? 2 : 1;          // tokens per lane in the softmax layout
  constexpr int NH = (G > 4) ? 4 : G;          // heads per lane in the softmax layout
  constexpr int LO = (G > 4) ? 8 : 4;          // first row of the lo limbs of P
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  const int t_begin = split * p.chunk_tokens;
  const int64_t pt_row = (int64_t)b * p.max_pages;
  // Page ids: lane l of `pidv` holds the (clamped) physical page of logical page pg_first + l,
  // i.e. one vector load covers 16 batches; `pidv_nx` is the following 64 pages, loaded 16
  // batches ahead.  A batch takes its four ids with v_readlane, so no page-table latency sits
  // between consecutive batches.  The first load does not wait for the sequence length:
  // entries past the sequence's last page are read (inside the row) and clamped to a valid
  // page, and the tokens they stand for are masked out below.
  const int pg_first = t_begin >> 4;
#define SAW_LOAD_PIDS(dst, first)                                                               \
  {                                                                                             \
    int id = p.page_table[pt_row + min((first) + lane, p.max_pages - 1)];                       \
    dst = (id < 0 || id >= p.num_pages) ? 0 : id;                                               \
  }
  int pidv, pidv_nx;
  SAW_LOAD_PIDS(pidv, pg_first)
  const int L = min(p.seq_lens[b], p.bound);
  const int t_end = min(L, t_begin + p.chunk_tokens);
  if (t_begin >= t_end) {
    if (p.num_splits == 1)          // empty sequence and no merge pass: the output row is zero
      for (int i = lane; i < G * 128; i += 64)
        store_elem(p.out, p.out_dtype, ((int64_t)b * p.n_q_heads + kvh * G) * 128 + i, 0.f);
    return;
  }
  SAW_LOAD_PIDS(pidv_nx, pg_first + 64)

  __shared__ __attribute__((aligned(16))) uint8_t lds[kStageBytes + kPbufBytes];
  uint8_t* const pbuf = lds + kStageBytes;

  const int row16 = lane & 15, grp = lane >> 4;
  const int64_t head_tile = (int64_t)kvh * kTileBytes;
  const int64_t page_stride = (int64_t)p.n_kv_heads * kTileBytes;
  const int64_t head_meta = (int64_t)kvh * 32;                    // floats
  const int64_t page_meta = (int64_t)p.n_kv_heads * 32;

  // ---- staging registers: one batch ahead ----
  u32x4 kst[4], vst[4];
  f32x2 kmeta[NS], vmeta[NS];
#define SAW_FETCH(batch)                                                                        \
  {                                                                                             \
    if ((batch) > 0 && ((batch) & 15) == 0) {                                                   \
      pidv = pidv_nx;                                                                           \
      SAW_LOAD_PIDS(pidv_nx, pg_first + 4 * (batch) + 64)                                       \
    }                                                                                           \
    int pid_[4];                                                                                \
    _Pragma("unroll") for (int q = 0; q < 4; ++q)                                               \
      pid_[q] = __builtin_amdgcn_readlane(pidv, 4 * ((batch) & 15) + q);                        \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                             \
      const int64_t off = (int64_t)pid_[q] * page_stride + head_tile + lane * 16;               \
      kst[q] = *(const u32x4*)(p.k_codes + off);                                                \
      vst[q] = *(const u32x4*)(p.v_codes + off);                                                \
    }                                                                                           \
    _Pragma("unroll") for (int s = 0; s < NS; ++s) {                                            \
      const int pg = (G > 4) ? (2 * s + (lane >> 5)) : grp; /* page of this lane's token */     \
      const int id = pg == 0 ? pid_[0] : pg == 1 ? pid_[1] : pg == 2 ? pid_[2] : pid_[3];       \
      const int64_t moff = (int64_t)id * page_meta + head_meta + row16 * 2;                     \
      kmeta[s] = *(const f32x2*)(p.k_meta + moff);                                              \
      vmeta[s] = *(const f32x2*)(p.v_meta + moff);                                              \
    }                                                                                           \
  }
  SAW_FETCH(0)

  // ---- prologue: q~ = (q H_blk) sm_scale log2(e), as bf16 hi/lo MFMA operands ----
  // (the stage area doubles as fp32 scratch; nothing has been staged yet)
  float* const qs = (float*)lds;
  for (int i = lane; i < G * D; i += 64)
    qs[i] = load_elem(p.q, p.q_dtype, ((int64_t)b * p.n_q_heads + kvh * G) * D + i);
  __syncthreads();
  float qmul = p.q_scale;
  if (p.rot_k) {
    wave_lds_fwht128(qs, G, p.had_block, lane);
    qmul *= had_norm(p.had_block);
  }
  // A operand of the logit MFMA.  Rows m < LO carry the hi limbs of head m, rows LO + g the lo
  // limbs of head g; lane (row16 = m, grp = k-group) holds channels 32*grp + 8*kk + {0,4,1,5,2,6,3,7}.
  const bool is_lo = row16 >= LO;
  const int qhead = row16 - (is_lo ? LO : 0);
  const bool q_live = qhead < G;
  const float* qrow = qs + (q_live ? qhead : 0) * D + 32 * grp;
  u32x4 a_q[4];
  float qpart = 0.f;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    uint32_t limb[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float x = q_live ? qrow[8 * kk + j] * qmul : 0.f;
      uint32_t h16, l16;
      float sum;
      split_bf16(x, h16, l16, sum);
      limb[j] = is_lo ? l16 : h16;
      qpart += __uint_as_float(limb[j] << 16);
    }
    a_q[kk] = u32x4{limb[0] | (limb[4] << 16), limb[1] | (limb[5] << 16), limb[2] | (limb[6] << 16), limb[3] | (limb[7] << 16)};
  }
  qpart += __shfl_xor(qpart, 16, 64);
  qpart += __shfl_xor(qpart, 32, 64);            // every lane of row m: sum of the limbs it feeds
  __syncthreads();
  if (lane < 16) qs[lane] = qpart;
  __syncthreads();
  float qsum[NH];                                // sum over channels of (hi + lo), per head of this lane
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    const int hd = (G > 4) ? (4 * (grp & 1) + i) : i;
    qsum[i] = qs[hd] + qs[LO + hd];
  }
  __syncthreads();
  for (int i = lane; i < kPbufBytes / 4; i += 64) ((uint32_t*)pbuf)[i] = 0u;
  const uint32_t kbias = bf16_bias();

  // ---- per-lane constants ----
  const int st_off = 16 * (4 * (lane >> 2) + (((lane & 3) + (lane >> 4)) & 3));     // staging write: t = lane>>2, Q = lane&3
  const int kr_off = 16 * (4 * row16 + ((grp + (row16 >> 2)) & 3));                 // K read: t = row16, Q = grp
  int vr_off[8];
#pragma unroll
  for (int c = 0; c < 8; ++c)
    vr_off[c] = 4 * kTileBytes + grp * kTileBytes + 16 * (4 * row16 + (((c >> 1) + (row16 >> 2)) & 3)) + 8 * (c & 1);
  // P write column inside the batch: 16*page + 8*(t/8) + perm^-1(t%8),  perm^-1(u) = (u&3)<<1 | u>>2
  const int pcol_t = (row16 & 8) + (((row16 & 3) << 1) | ((row16 >> 2) & 1));
  const int head0 = (G > 4) ? 4 * (grp & 1) : 0;                                    // first head of this lane

  f32x4 oacc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) oacc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_ref[NH], lsum[NH], zs[NH];
#pragma unroll
  for (int i = 0; i < NH; ++i) { m_ref[i] = -INFINITY; lsum[i] = 0.f; zs[i] = 0.f; }

  const int nb = (t_end - t_begin + 63) >> 6;
  for (int bi = 0; bi < nb; ++bi) {
    // ---- stage the fetched batch, start the next fetch ----
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      *(u32x4*)(lds + q * kTileBytes + st_off) = kst[q];
      *(u32x4*)(lds + (4 + q) * kTileBytes + st_off) = vst[q];
    }
    f32x2 km[NS], vm[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) { km[s] = kmeta[s]; vm[s] = vmeta[s]; }
    if (bi + 1 < nb) SAW_FETCH(bi + 1)
    __syncthreads();

    // ---- logits: D_q[head][token of page q] ----
    f32x4 dq[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const u32x4 kw = *(const u32x4*)(lds + q * kTileBytes + kr_off);
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        acc = mfma_bf16(as_bf16x8(a_q[kk]), unpack8(kw[kk], kbias), acc);
      }
      dq[q] = acc;
    }
    // ---- gather: lane = token of the batch, registers = heads ----
    float sraw[NS][NH];
#pragma unroll
    for (int i = 0; i < NH; ++i) {
      float hi, lo, junk;
      if (G > 4) {      // tile rows: hi heads 0-3 | hi 4-7 | lo 0-3 | lo 4-7
        swap32(dq[0][i], dq[1][i], hi, lo);
        sraw[0][i] = hi + lo;
        swap32(dq[2][i], dq[3][i], hi, lo);
        sraw[NS - 1][i] = hi + lo;
      } else {          // tile rows: hi heads | lo heads | idle | idle
        float h01, l01, h23, l23;
        swap16(dq[0][i], dq[1][i], h01, l01);
        swap16(dq[2][i], dq[3][i], h23, l23);
        swap32(h01, h23, hi, junk);
        swap32(l01, l23, lo, junk);
        sraw[0][i] = hi + lo;
      }
    }
    // ---- softmax with a lazily updated reference maximum ----
    const int tok0 = t_begin + 64 * bi;
    float lg[NS][NH];
    bool valid[NS];
    bool need = false;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int pg = (G > 4) ? (2 * s + (lane >> 5)) : grp;
      valid[s] = (tok0 + 16 * pg + row16) < t_end;
      const float kz = km[s].y + 128.f;
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        const float v = km[s].x * fmaf(-kz, qsum[i], sraw[s][i]);
        lg[s][i] = valid[s] ? v : -INFINITY;
        need |= lg[s][i] > m_ref[i] + kLazyTau;
      }
    }
    if (__any(need)) {
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        float mx = lg[0][i];
        if (NS > 1) mx = fmaxf(mx, lg[NS - 1][i]);
        mx = row_allmax(mx);
        if (G > 4) {
          mx = fmaxf(mx, __shfl_xor(mx, 32, 64));      // lanes 32 apart share the head group
        } else {
          mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
          mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        }
        const float mnew = fmaxf(m_ref[i], mx);
        const float alpha = fast_exp2(m_ref[i] - mnew);      // 0 on the first batch
        lsum[i] *= alpha;
        zs[i] *= alpha;
#pragma unroll
        for (int c = 0; c < 8; ++c) oacc[c][i] *= alpha;
        m_ref[i] = mnew;
      }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int pg = (G > 4) ? (2 * s + (lane >> 5)) : grp;
      const int col = 16 * pg + pcol_t;
      const float vs = valid[s] ? vm[s].x : 0.f;
      const float vz = valid[s] ? vm[s].y + 128.f : 0.f;
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        const float pr = fast_exp2(lg[s][i] - m_ref[i]);     // exp2(-inf) = 0 for masked tokens
        lsum[i] += pr;
        uint32_t h16, l16;
        float wsum;
        split_bf16(pr * vs, h16, l16, wsum);
        zs[i] = fmaf(wsum, vz, zs[i]);
        ((uint16_t*)pbuf)[(head0 + i) * kProw + col] = (uint16_t)h16;
        ((uint16_t*)pbuf)[(LO + head0 + i) * kProw + col] = (uint16_t)l16;
      }
    }
    __syncthreads();
    // ---- O[row][channel] += P (rows x 64 tokens) . V codes ----
    const u32x4 pa0 = *(const u32x4*)(pbuf + (row16 * kProw + 16 * grp) * 2);
    const u32x4 pa1 = *(const u32x4*)(pbuf + (row16 * kProw + 16 * grp + 8) * 2);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const i32x2 tv = __builtin_amdgcn_ds_read_tr4_b64_v2i32((LDS_AS i32x2*)(lds + vr_off[c]));
      oacc[c] = mfma_bf16(as_bf16x8(pa0), unpack8((uint32_t)tv.x, kbias), oacc[c]);
      oacc[c] = mfma_bf16(as_bf16x8(pa1), unpack8((uint32_t)tv.y, kbias), oacc[c]);
    }
  }

  // ---- epilogue: reduce the per-lane sums, fold hi + lo rows, write the partial ----
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    lsum[i] = row_allsum(lsum[i]);
    zs[i] = row_allsum(zs[i]);
    if (G > 4) {
      lsum[i] += __shfl_xor(lsum[i], 32, 64);
      zs[i] += __shfl_xor(zs[i], 32, 64);
    } else {
      lsum[i] += __shfl_xor(lsum[i], 16, 64);
      lsum[i] += __shfl_xor(lsum[i], 32, 64);
      zs[i] += __shfl_xor(zs[i], 16, 64);
      zs[i] += __shfl_xor(zs[i], 32, 64);
    }
  }
  constexpr int LOSHIFT = (G > 4) ? 32 : 16;     // lanes holding the lo rows sit this far above the hi rows
  const bool writer = (G > 4) ? (grp < 2) : (grp == 0);
  if (p.num_splits == 1) {
    // The partition is the whole sequence: normalise, rotate back once for V, write the output.
    float* const fb = (float*)lds;               // [G][128]; every read of the stage area is done
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NH; ++i) {
      const float inv = 1.0f / lsum[i];
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float o = oacc[c][i] + __shfl_down(oacc[c][i], LOSHIFT, 64);
        if (writer && i < G) fb[(head0 + i) * D + 16 * c + row16] = (o - zs[i]) * inv;
      }
    }
    __syncthreads();
    float onorm = 1.0f;
    if (p.rot_v) {
      wave_lds_fwht128(fb, G, p.had_block, lane);
      onorm = had_norm(p.had_block);
    }
    const int64_t obase = ((int64_t)b * p.n_q_heads + kvh * G) * D;
    for (int i = lane; i < G * D; i += 64) store_elem(p.out, p.out_dtype, obase + i, fb[i] * onorm);
    return;
  }
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    const int head = head0 + i;
    float* dst = p.ws + (((int64_t)b * p.n_q_heads + kvh * G + head) * p.num_splits + split) * (D + 2);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float o = oacc[c][i] + __shfl_down(oacc[c][i], LOSHIFT, 64);
      if (writer && i < G) dst[2 + 16 * c + row16] = o - zs[i];
    }
    if (writer && row16 == 0 && i < G) { dst[0] = m_ref[i]; dst[1] = lsum[i]; }
  }
}

#undef SAW_FETCH
#undef SAW_LOAD_PIDS

int launch_decode_int4_mfma(const DecodeParams& p, int G, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: decode_int4_mfma_kernel<1><<<grid, dim3(64), 0, st>>>(p); break;
    case 2: decode_int4_mfma_kernel<2><<<grid, dim3(64), 0, st>>>(p); break;
    case 4: decode_int4_mfma_kernel<4><<<grid, dim3(64), 0, st>>>(p); break;
    case 8: decode_int4_mfma_kernel<8><<<grid, dim3(64), 0, st>>>(p); break;
    default: return SAW_EINVAL;
  }
  return SAW_OK;
}

}  // namespace saw
