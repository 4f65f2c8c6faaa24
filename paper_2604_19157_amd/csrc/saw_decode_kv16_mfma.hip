// 16-bit-KV paged decode attention for head_dim 128 on the gfx950 matrix cores: the unquantised
// comparison path (the cache the paper measures INT4 against, Sec. 2), written with the same
// machinery as the INT4 kernel so that the comparison is between formats, not between efforts.
//
// One wavefront owns one (sequence, kv head, partition) and walks it in batches of two pages
// (32 tokens).  Per batch:
//   * K needs no staging: lane (token = lane % 16, k-group = lane / 16) of the logit MFMA's B
//     operand wants 8 consecutive channels of its token, which is one 16-byte global load, so the
//     eight K operand registers of a batch are loaded straight from HBM one batch ahead;
//   * V is wanted with tokens along the contraction: its two page tiles (4 KiB each) go HBM -> LDS
//     directly (global_load_lds_dwordx4) into a double buffer, 16-byte chunks XOR-swizzled by row so
//     that ds_read_b64_tr_b16 (a 4x16 transpose of 16-bit elements inside each 16-lane group) reads
//     them without bank conflicts and hands each lane 4 tokens of one channel;
//   * logits: D[head][token] = q~ (heads x channels) . K (channels x tokens) with
//     v_mfma_f32_16x16x32, q~ carried as hi + lo 16-bit limbs in separate rows of the tile;
//   * softmax with a lazily updated reference maximum, P through LDS once as hi/lo rows,
//     O[head][channel] in eight 16x16 tiles.
// Group sizes up to 4 (rows: hi limbs of the heads, then lo limbs); larger groups use the
// vector-ALU kernel.
//
// PAIR = true gives this kernel the INT4 kernel's way of evening out a ragged batch when all of it
// is resident at once (one partition per sequence, 257..2048 (sequence, kv head) items): a block
// of two wavefronts owns the sequences at ranks r and B-1-r of the longest-first order and halves
// their 32-token batches: wavefront 0 streams the first part of the long sequence, wavefront 1 the
// short sequence and then the rest of the long one; the two leave their shares of the long
// sequence as (max, sum, accumulator) records in LDS, and whichever comes second combines them
// (wavefront 0's first) and writes the output.
#include "saw_decode.h"
#include "saw_wave_util.h"
#include "saw_rank.h"

namespace saw {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

namespace kv16 {

constexpr int kRowBytes = 256;                 // one token's head vector
constexpr int kPageBytes = 16 * kRowBytes;     // one (page, head) tile
constexpr int kVbufBytes = 2 * kPageBytes;     // a batch: 32 token rows
constexpr int kProw = 40;                      // P row stride in 16-bit elements (32 tokens + 8 pad)
constexpr int kPbufBytes = 8 * kProw * 2;      // hi rows of 4 heads, lo rows of 4 heads
constexpr int kWaveLds = 2 * kVbufBytes + kPbufBytes;
constexpr float kLazyTau = 8.0f;

template <int DT>
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  if (DT == SAW_BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// x = hi + lo as two 16-bit values of the cache's type (hi truncated / rounded, lo the rounded rest)
template <int DT>
__device__ __forceinline__ void split16(float x, uint32_t& hi16, uint32_t& lo16) {
  if (DT == SAW_BF16) {
    float sum;
    split_bf16(x, hi16, lo16, sum);
  } else {
    hi16 = f32_to_f16(x);
    lo16 = f32_to_f16(x - f16_to_f32(hi16));
  }
}

}  // namespace kv16

template <int G, int DT, bool PAIR>
__global__ __launch_bounds__(PAIR ? 128 : 64) void decode_kv16_mfma_kernel(DecodeParams p) {
  using namespace kv16;
  constexpr int D = 128;
  constexpr int NWV = PAIR ? 2 : 1;
  // (the partition index is rotated by kv head and sequence, so that no XCD serves a fixed set of partitions)
  const int split = (blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x, kvh = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row16 = lane & 15, grp = lane >> 4;
  // (one shared array for everything: see the INT4 kernel on why)
  __shared__ __attribute__((aligned(16))) uint8_t lds_all[NWV * kWaveLds + 16];
  uint8_t* const lds = lds_all + wave * kWaveLds;
  uint8_t* const vbuf_a = lds;
  uint8_t* const vbuf_b = lds + kVbufBytes;
  uint8_t* const pbuf = lds + 2 * kVbufBytes;
  int* const done_cnt = (int*)(lds_all + NWV * kWaveLds);      // PAIR: records left of the long sequence

  // ---- the ranges this wavefront streams ----
  int nseg = 1;
  int sg_b[2] = {(int)blockIdx.z, 0}, sg_t0[2] = {0, 0}, sg_t1[2] = {0, 0};
  bool sg_share[2] = {false, false};
  if (PAIR) {
    const int B = p.batch;
    if (threadIdx.x == 0) done_cnt[0] = 0;
    __syncthreads();
    const LenClasses lc = build_len_classes(p, B, lane, (int*)vbuf_a);
    const int r_long = blockIdx.z, r_short = B - 1 - r_long;
    const bool self = r_long == r_short;                // odd batch: the middle sequence pairs with itself
    const int b_long = seq_of_rank(lane, lc, r_long);
    const int b_short = self ? b_long : seq_of_rank(lane, lc, r_short);
    const int l_long = lc.lens[b_long];
    const int l_short = self ? 0 : lc.lens[b_short];
    const int nb_long = (l_long + 31) >> 5, nb_short = (l_short + 31) >> 5;
    // wavefront 1 pays a second prologue when the long sequence is shared: two batches in its favour
    const int cut = min(nb_long, (nb_long + nb_short + 2) >> 1);
    const bool shared = cut < nb_long;
    nseg = 0;
    if (wave == 0) {
      if (nb_long == 0) {                               // empty sequence: zero output row
        for (int i = lane; i < G * D; i += 64)
          store_elem(p.out, p.out_dtype, ((int64_t)b_long * p.n_q_heads + kvh * G) * D + i, 0.f);
      } else {
        sg_b[0] = b_long; sg_t0[0] = 0; sg_t1[0] = min(l_long, 32 * cut); sg_share[0] = shared;
        nseg = 1;
      }
    } else {
      if (nb_short > 0) {
        sg_b[0] = b_short; sg_t0[0] = 0; sg_t1[0] = l_short; sg_share[0] = false;
        nseg = 1;
      } else if (!self) {
        for (int i = lane; i < G * D; i += 64)
          store_elem(p.out, p.out_dtype, ((int64_t)b_short * p.n_q_heads + kvh * G) * D + i, 0.f);
      }
      if (shared) {                                     // last, so that its record can stay in this wavefront's buffers
        if (nseg == 0) { sg_b[0] = b_long; sg_t0[0] = 32 * cut; sg_t1[0] = l_long; sg_share[0] = true; }
        else           { sg_b[1] = b_long; sg_t0[1] = 32 * cut; sg_t1[1] = l_long; sg_share[1] = true; }
        ++nseg;
      }
    }
    wave_sync();                                        // the ranking's scratch lived in vbuf_a
  } else {
    const int L = min(p.seq_lens[sg_b[0]] + p.len_bias, p.bound);
    sg_t0[0] = split * p.chunk_tokens;
    sg_t1[0] = min(L, sg_t0[0] + p.chunk_tokens);
    if (sg_t0[0] >= sg_t1[0]) {
      if (p.num_splits == 1)
        for (int i = lane; i < G * D; i += 64)
          store_elem(p.out, p.out_dtype, ((int64_t)sg_b[0] * p.n_q_heads + kvh * G) * D + i, 0.f);
      return;
    }
  }

#pragma unroll 1
  for (int seg = 0; seg < nseg; ++seg) {
  const int b = seg == 0 ? sg_b[0] : sg_b[1];
  const int t_begin = seg == 0 ? sg_t0[0] : sg_t0[1];
  const int t_end = seg == 0 ? sg_t1[0] : sg_t1[1];
  const bool share = seg == 0 ? sg_share[0] : sg_share[1];

  const uint8_t* const kpages = p.k_codes;
  const uint8_t* const vpages = p.v_codes;
  const int64_t pt_row = (int64_t)b * p.max_pages;
  const int64_t page_stride = (int64_t)p.n_kv_heads * kPageBytes;
  const int64_t head_off = (int64_t)kvh * kPageBytes;
  const int pg_first = t_begin >> 4;
  const int nb = (t_end - t_begin + 31) >> 5;                       // batches of 32 tokens

  // ---- q~ = q sm_scale log2(e) as the logit MFMA's A operand: rows 0..3 hi limbs, 4..7 lo limbs ----
  u32x4 a_q[4];
  {
    const bool is_lo = (row16 & 4) != 0;
    const int qhead = row16 & 3;
    const bool live = row16 < 8 && qhead < G;
    const int64_t qbase = ((int64_t)b * p.n_q_heads + kvh * G + (live ? qhead : 0)) * D;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint32_t limb[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float x = live ? load_elem(p.q, p.q_dtype, qbase + 32 * kk + 8 * grp + j) * p.q_scale : 0.f;
        uint32_t h16, l16;
        split16<DT>(x, h16, l16);
        limb[j] = is_lo ? l16 : h16;
      }
      a_q[kk] = u32x4{limb[0] | (limb[1] << 16), limb[2] | (limb[3] << 16), limb[4] | (limb[5] << 16), limb[6] | (limb[7] << 16)};
    }
  }

  // ---- fetch ----
  // page ids of a batch: lanes 0 and 1 of `pidv`
  auto load_pids = [&](int batch) {
    const int lp = min(pg_first + 2 * batch + (lane & 1), p.max_pages - 1);
    const int id = p.page_table[pt_row + lp];
    return (id < 0 || id >= p.num_pages) ? 0 : id;
  };
  // K operand registers of a batch: kreg[page][kk] = channels 32kk + 8grp .. +7 of token row16
  u32x4 kreg[2][4];
#define KV16_LOAD_K(pid0, pid1)                                                                  \
  {                                                                                              \
    const uint8_t* k0 = kpages + (int64_t)(pid0) * page_stride + head_off + row16 * kRowBytes + 16 * grp; \
    const uint8_t* k1 = kpages + (int64_t)(pid1) * page_stride + head_off + row16 * kRowBytes + 16 * grp; \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                           \
      kreg[0][kk] = __builtin_nontemporal_load((const u32x4*)(k0 + 64 * kk));                    \
      kreg[1][kk] = __builtin_nontemporal_load((const u32x4*)(k1 + 64 * kk));                    \
    }                                                                                            \
  }
  // (all K and V reads are marked streaming, cache policy "nt", as in the INT4 kernel)
  // V tiles of a batch into VDST: transfer j covers token rows 4j .. 4j+3 (1 KiB of LDS); the lane
  // at chunk position c of row r brings source chunk c ^ (2 (r & 3))
  const int v_r4 = lane >> 4;                                        // row inside the transfer
  const int v_src = (v_r4 * kRowBytes) + 16 * ((lane & 15) ^ (2 * v_r4));
#define KV16_DMA_V(pid0, pid1, VDST)                                                             \
  {                                                                                              \
    const uint8_t* v0 = vpages + (int64_t)(pid0) * page_stride + head_off + v_src;               \
    const uint8_t* v1 = vpages + (int64_t)(pid1) * page_stride + head_off + v_src;               \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                              \
      __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(v0 + j * 4 * kRowBytes),          \
                                       (LDS_AS void*)(VDST + j * 1024), 16, 0, 2);               \
      __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(v1 + j * 4 * kRowBytes),          \
                                       (LDS_AS void*)(VDST + 4096 + j * 1024), 16, 0, 2);        \
    }                                                                                            \
  }
  int pid_nx;                                                        // ids of the batch after the one in flight
  {
    const int pv = load_pids(0);
    const int a = __builtin_amdgcn_readlane(pv, 0), c = __builtin_amdgcn_readlane(pv, 1);
    KV16_LOAD_K(a, c)
    KV16_DMA_V(a, c, vbuf_a)
    pid_nx = load_pids(min(1, nb - 1));
  }

  // ---- per-lane constants ----
  // V transpose reads: source lane (s = row16, g = grp), half h, addresses 4 channels (16c + 4(s&3) ..)
  // of token row r = 8g + 4h + s/4; the 16-byte chunk 2c + (s&3)/2 of that row sits at chunk position
  // (2c + (s&3)/2) ^ 2(r&3) = 2(c ^ (r&3)) + (s&3)/2
  const int v_rho = row16 >> 2;                                     // r & 3, the same for both halves
  const int vr_base = (8 * grp + v_rho) * kRowBytes + 16 * ((row16 & 3) >> 1) + 8 * (row16 & 1);
  // P: lane (token tk = lane % 32 of the batch, in lanes 0..31) writes column tk; the A operand read of
  // lane (row, g) takes tokens 8g .. 8g+7 of row & 7
  const uint32_t pa_addr = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)pbuf + ((row16 & 7) * kProw + 8 * grp) * 2;

  f32x4 oacc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) oacc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_ref[G], lsum[G];
#pragma unroll
  for (int i = 0; i < G; ++i) { m_ref[i] = -INFINITY; lsum[i] = 0.f; }

  auto two_batches = [&](const int bi0, uint8_t* __restrict__ const va, uint8_t* __restrict__ const vb,
                         uint8_t* __restrict__ const pb) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      if (half == 1 && bi0 + 1 >= nb) break;
      const int bi = bi0 + half;
      uint8_t* const vcur = half ? vb : va;
      uint8_t* const vnext = half ? va : vb;
      __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0): batch bi has landed (K registers, V in LDS)
      // ---- logits ----
      f32x4 dq[2];
#pragma unroll
      for (int pg = 0; pg < 2; ++pg) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) acc = mfma16<DT>(a_q[kk], kreg[pg][kk], acc);
        dq[pg] = acc;
      }
      // the next batch, if there is one: K into the registers just consumed, V into the other buffer
      if (bi + 1 < nb) {
        const int a = __builtin_amdgcn_readlane(pid_nx, 0), c = __builtin_amdgcn_readlane(pid_nx, 1);
        KV16_LOAD_K(a, c)
        KV16_DMA_V(a, c, vnext)
        pid_nx = load_pids(min(bi + 2, nb - 1));
      }
      // ---- gather: lanes 0..15 = tokens of page 0, 16..31 = page 1, registers = heads ----
      float lg[G];
      const int tok = t_begin + 32 * bi + (lane & 31);
      const bool valid = lane < 32 && tok < t_end;
      bool need = false;
#pragma unroll
      for (int i = 0; i < G; ++i) {
        float hi, lo;
        swap16(dq[0][i], dq[1][i], hi, lo);                  // hi: rows (p0.hi, p1.hi, ..), lo: rows (p0.lo, p1.lo, ..)
        lg[i] = valid ? hi + lo : -INFINITY;
        need |= lg[i] > m_ref[i] + kLazyTau;
      }
      if (__any(need)) {
#pragma unroll
        for (int i = 0; i < G; ++i) {
          float mx = row_allmax(lg[i]);
          mx = max_xor16(mx);
          mx = max_xor32(mx);
          const float mnew = fmaxf(m_ref[i], mx);
          const float alpha = fast_exp2(m_ref[i] - mnew);
          lsum[i] *= alpha;
#pragma unroll
          for (int c = 0; c < 8; ++c) oacc[c][i] *= alpha;
          m_ref[i] = mnew;
        }
      }
#pragma unroll
      for (int i = 0; i < G; ++i) {
        const float pr = fast_exp2(lg[i] - m_ref[i]);          // 0 for masked tokens and idle lanes
        lsum[i] += pr;
        uint32_t h16, l16;
        split16<DT>(pr, h16, l16);
        if (lane < 32) {
          ((uint16_t*)pb)[i * kProw + lane] = (uint16_t)h16;
          ((uint16_t*)pb)[(4 + i) * kProw + lane] = (uint16_t)l16;
        }
      }
      wave_sync();
      // ---- O[row][channel] += P (rows x 32 tokens) . V ----
      u32x4 pa;
      asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(pa) : "v"(pa_addr) : "memory");
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int voff = vr_base + 32 * (c ^ v_rho);
        const i16x4 t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS i16x4*)(vcur + voff));
        const i16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS i16x4*)(vcur + voff + 4 * kRowBytes));
        const u32x4 bv = u32x4{(uint32_t)(uint16_t)t0[0] | ((uint32_t)(uint16_t)t0[1] << 16),
                               (uint32_t)(uint16_t)t0[2] | ((uint32_t)(uint16_t)t0[3] << 16),
                               (uint32_t)(uint16_t)t1[0] | ((uint32_t)(uint16_t)t1[1] << 16),
                               (uint32_t)(uint16_t)t1[2] | ((uint32_t)(uint16_t)t1[3] << 16)};
        oacc[c] = mfma16<DT>(pa, bv, oacc[c]);
      }
      wave_sync();                                           // P is rewritten by the next batch
    }
  };
  for (int bi = 0; bi < nb; bi += 2) two_batches(bi, vbuf_a, vbuf_b, pbuf);
  __builtin_amdgcn_s_waitcnt(0x0F70);                        // nothing this wavefront requested is still on its way

  // ---- epilogue ----
#pragma unroll
  for (int i = 0; i < G; ++i) {
    lsum[i] = row_allsum(lsum[i]);
    lsum[i] = add_xor16(lsum[i]);
    lsum[i] = add_xor32(lsum[i]);
  }
  // oacc[c][i] of lane (grp, row16) = O[row 4 grp + i][channel 16c + row16]: rows 0..3 (grp 0) hi, 4..7 (grp 1) lo
  const bool writer = grp == 0;
  if (PAIR && share) {
    // this wavefront's share of the long sequence as a record in its own V buffer (every read of
    // it is done and nothing is in flight): acc[G][128] un-normalised, then (max, sum) per head
    float* const rec = (float*)vbuf_a;
    wave_sync();
#pragma unroll
    for (int i = 0; i < G; ++i) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float o = add_xor16(oacc[c][i]);     // hi rows + lo rows
        if (writer) rec[i * D + 16 * c + row16] = o;
      }
      if (writer && row16 == 0) { rec[G * D + 2 * i] = m_ref[i]; rec[G * D + 2 * i + 1] = lsum[i]; }
    }
    // LDS operations of a wavefront complete in order, so the record is in place before the count;
    // the wavefront that finds the other already counted does the rest for both (a shared range
    // is always a wavefront's last).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    int before = 0;
    if (lane == 0) before = __hip_atomic_fetch_add(done_cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    before = __builtin_amdgcn_readfirstlane(before);
    if (before == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const float* const rec0 = (const float*)lds_all;                  // wavefront 0's record is always the first operand
    const float* const rec1 = (const float*)(lds_all + kWaveLds);
    const int64_t obase = ((int64_t)b * p.n_q_heads + kvh * G) * D;
    for (int idx = lane; idx < G * D; idx += 64) {
      const int h = idx >> 7;
      const float m0 = rec0[G * D + 2 * h], m1 = rec1[G * D + 2 * h];
      const float mm = fmaxf(m0, m1);
      const float a0 = fast_exp2(m0 - mm), a1 = fast_exp2(m1 - mm);
      const float v = fmaf(a1, rec1[idx], a0 * rec0[idx]);
      const float l = fmaf(a1, rec1[G * D + 2 * h + 1], a0 * rec0[G * D + 2 * h + 1]);
      store_elem(p.out, p.out_dtype, obase + idx, v / l);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < G; ++i) {
    const int head = kvh * G + i;
    float* part = p.ws + (((int64_t)b * p.n_q_heads + head) * p.num_splits + split) * (D + 2);
    const float inv = 1.0f / lsum[i];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float o = add_xor16(oacc[c][i]);       // hi rows + lo rows
      if (writer) {
        if (p.num_splits == 1)
          store_elem(p.out, p.out_dtype, ((int64_t)b * p.n_q_heads + head) * D + 16 * c + row16, o * inv);
        else
          part[2 + 16 * c + row16] = o;
      }
    }
    if (p.num_splits != 1 && writer && row16 == 0) { part[0] = m_ref[i]; part[1] = lsum[i]; }
  }
  wave_sync();                                   // the next range's prologue reuses the buffers
  }  // ranges of this wavefront
}

#undef KV16_LOAD_K
#undef KV16_DMA_V

// head_dim 128, group size <= 4; returns false when this kernel does not cover the case.
bool launch_decode_kv16_mfma(const DecodeParams& p, int G, int kv_dtype, dim3 grid, hipStream_t st) {
#define KV16_GO(GG)                                                                              \
  if (p.pair) {                                                                                  \
    const dim3 pgrid(1, grid.y, (p.batch + 1) / 2);                                              \
    if (kv_dtype == SAW_BF16) decode_kv16_mfma_kernel<GG, SAW_BF16, true><<<pgrid, dim3(128), 0, st>>>(p); \
    else decode_kv16_mfma_kernel<GG, SAW_F16, true><<<pgrid, dim3(128), 0, st>>>(p);             \
  } else if (kv_dtype == SAW_BF16) decode_kv16_mfma_kernel<GG, SAW_BF16, false><<<grid, dim3(64), 0, st>>>(p); \
  else decode_kv16_mfma_kernel<GG, SAW_F16, false><<<grid, dim3(64), 0, st>>>(p);
  switch (G) {
    case 1: KV16_GO(1) return true;
    case 2: KV16_GO(2) return true;
    case 4: KV16_GO(4) return true;
    default: return false;
  }
#undef KV16_GO
}

}  // namespace saw
