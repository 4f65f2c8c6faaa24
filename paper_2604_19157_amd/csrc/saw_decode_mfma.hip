// INT4 paged decode attention for head_dim 128 on the gfx950 matrix cores.
// Paper: Sec. 2 (decode step), Sec. 4.1 / App. A.4 (rotated-space attention), App. A.1.
//
// A wavefront walks a range of one (sequence, kv head)'s tokens in batches of four pages (64
// tokens); which ranges a wavefront gets (a whole partition, every NW-th batch of one, or an even
// share of a long/short sequence pair) is described at the kernel.  Per batch:
//   * the four K and four V code tiles (1 KiB each, contiguous in HBM) and the tokens' (scale,
//     zero) pairs go straight from global memory into LDS (global_load_lds_dwordx4, no staging
//     registers): V and the metadata one batch ahead into double buffers, K into a single buffer
//     that is refilled as soon as its operand reads are done.  Each lane fetches the 16-byte chunk that belongs at its LDS
//     position under the swizzle pos(t, Q) = 4t + ((Q + t/4) & 3), which makes every later
//     LDS read bank-conflict free while a lane quad still reads one whole 64-byte row;
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
// When one partition covers the sequence the kernel also normalises, rotates the output back and
// writes it (no merge launch), and it can append the step's new token itself (append_token).
#include "saw_decode.h"
#include "saw_wave_util.h"
#include "saw_rank.h"

namespace saw {

constexpr int kTileBytes = 1024;               // one (page, head) code tile: 16 tokens x 64 B
constexpr int kProw = 72;                      // P row stride in bf16 (64 tokens + 8 pad: conflict-free b128 reads)
constexpr int kPbufBytes = 16 * kProw * 2;     // P as bf16 [16 rows][64 tokens]
constexpr float kLazyTau = 8.0f;               // reference max may lag the true max by 2^8

// ---------------------------------------------------------------------------------------
// q~ = (q H_blk) sm_scale log2(e) for the G query heads of one kv head, in the lane layout of the
// logit MFMA's A operand, as bf16 hi and lo limbs (Sec. 4.1: the query is rotated once and
// consumed by the q.K loop).  Rows m < LO carry the hi limbs of head m, rows LO + g the lo limbs
// of head g; lane (row16 = m, grp = k-group) holds channels 32*grp + 8*kk + {0,4,1,5,2,6,3,7}.
// qsum[i] is the sum over channels of hi + lo for the i-th head of this lane's softmax layout.
// `qraw` holds this lane's share of q (element lane + 64 j), loaded by the caller ahead of time;
// `qs` is LDS scratch of G*128 floats.  It is a __restrict__ parameter on purpose: that keeps
// these LDS accesses in an alias scope of their own, so the compiler does not make them wait for
// the LDS-DMA transfers the caller already has in flight into other buffers.
// HP (two 64-channel heads per row, see the kernel): `qraw[j]`, j < G, is channel `lane` of the j-th
// query head of the pair; its row gets the 64 values in the half of its own kv head and zeros in
// the other half, so that the 128-channel products below are the 64-channel ones.
// DN: a learned rotation R_l follows the Hadamard (App. A.3); a compile-time flag, so that the kernels
// of caches without one carry none of its code.
template <int G, int NH, bool HP, bool DN>
__device__ __forceinline__ void prepare_q(const DecodeParams& p, const float (&qraw)[2 * G], int lane,
                                          float* __restrict__ qs, u32x4 (&a_q)[4],
                                          float (&qsum)[NH], float& qmul_out) {
  constexpr int D = 128;
  constexpr int LO = (G > 4) ? 8 : 4;
  const int row16 = lane & 15, grp = lane >> 4;
  if (HP) {
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int kv = j / (G / 2 > 0 ? G / 2 : 1);
      qs[j * D + 64 * kv + lane] = qraw[j];
      qs[j * D + 64 * (1 - kv) + lane] = 0.f;
    }
  } else {
    // a lane holds channels `lane` and `lane + 64` of every head: the butterflies of stride 64
    // (h = 128) are done here, in registers, and the LDS transform only goes up to order 64
    const bool top = p.rot_k && p.had_block > 64;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float a = qraw[2 * g], b = qraw[2 * g + 1];
      qs[lane + 128 * g] = top ? a + b : a;
      qs[lane + 128 * g + 64] = top ? a - b : b;
    }
  }
  wave_sync();
  float qmul = p.q_scale;
  if (p.rot_k) {
    wave_lds_fwht128<G>(qs, min(p.had_block, 64), lane);
    qmul *= had_norm(p.had_block);
  }
  // learned rotation after the Hadamard (App. A.3: q^ = (q H_b) R_l)
  if constexpr (DN) {
    if (p.dense_k) wave_lds_matvec128<G>(qs, p.dense, lane);
  }
  const bool is_lo = row16 >= LO;
  const int qhead = row16 - (is_lo ? LO : 0);
  const bool q_live = qhead < G;
  const float* qrow = qs + (q_live ? qhead : 0) * D + 32 * grp;
  const float qm = q_live ? qmul : 0.f;                      // idle rows of the tile carry zeros
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const f32x4 va = *(const f32x4*)(qrow + 8 * kk), vb = *(const f32x4*)(qrow + 8 * kk + 4);
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {                            // dword j packs channels j (low half) and j + 4
      const float x0 = va[j] * qm, x1 = vb[j] * qm;
      const uint32_t u0 = __float_as_uint(x0), u1 = __float_as_uint(x1);
      // hi limbs: the top 16 bits of both values in one byte permute
      const uint32_t hi = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
      // lo limbs: the remainders, rounded to nearest even (v_cvt_pk_bf16_f32)
      const f32x2 rem = f32x2{x0 - __uint_as_float(u0 & 0xffff0000u), x1 - __uint_as_float(u1 & 0xffff0000u)};
      typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
      const uint32_t lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(rem, bf16x2_t));
      w[j] = is_lo ? lo : hi;
    }
    a_q[kk] = u32x4{w[0], w[1], w[2], w[3]};
  }
  // qsum = sum over channels of the limbs as the matrix cores will see them: one product per k-step
  // with a matrix of ones leaves row m's sum in every column; lane (grp, .) holds rows 4 grp + i,
  // and the hi and lo rows of a head sit one (G <= 4) or two (G = 8) lane groups apart
  f32x4 rs = f32x4{0.f, 0.f, 0.f, 0.f};
  const bf16x8 ones = as_bf16x8(u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) rs = mfma_bf16(as_bf16x8(a_q[kk]), ones, rs);
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    float t = rs[i];
    if (G <= 4) t = add_xor16(t);                            // rows 0-3 (hi) + rows 4-7 (lo); groups 2, 3 hold zeros
    qsum[i] = add_xor32(t);                                  // G = 8: rows 4 (grp & 1) + i (hi) + 8 more (lo)
  }
  wave_sync();
  qmul_out = qmul;
}

constexpr int kMetaBytesOf(bool hp) { return hp ? 2048 : 1024; }   // one batch's (scale, zero) pairs: K, then V

// (what append_token leaves for append_store: this lane's code byte and (scale, zero) pair of K and of V,
// the token's vector index in the pools, and whether its page is mapped)
struct NewToken {
  uint32_t byte[2];
  f32x2 meta[2];
  int64_t vec;
  bool place;
};
// The stores of the new token to the cache pools.  They are issued after the batch that attends to the
// token (which needs nothing from memory), so that no part of the step waits for them.
template <bool HP>
__device__ __forceinline__ void append_store(const DecodeParams& p, int lane, const NewToken& nt) {
  constexpr int DH = HP ? 64 : 128;
  if (!nt.place) return;
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    uint8_t* codes = const_cast<uint8_t*>(w ? p.v_codes : p.k_codes);
    float* meta = const_cast<float*>(w ? p.v_meta : p.k_meta);
    codes[nt.vec * (DH / 2) + (lane & (DH / 2 - 1))] = (uint8_t)nt.byte[w];
    if ((lane & (DH / 2 - 1)) == 0) *(f32x2*)(meta + nt.vec * 2) = nt.meta[w];
  }
}
// The decode step's own token (fused append, Sec. 4.1's "new KV entries are rotated, quantised
// and written" folded into the attention launch): rotate and quantise the new K and V vectors of
// (sequence b, kv head kvh) for position L exactly as the store kernel would (Sec. 3 eqs. 1-3,
// App. A.1; append_store writes them to the pools), and place its codes and (scale, zero) pairs in LDS as token 0 of page 0 of a
// batch, in the layout the transfers produce.  The caller then runs one more batch in which only that
// token is valid, so the new token goes through the very code path of the cached ones (same q~ limbs,
// same softmax update) and nothing this launch writes to the cache is read back by it.  All of this
// happens at the END of the range that starts the sequence, when every transfer of the range has
// landed: at the start of a launch all wavefronts of the chip run their prologues at once and are
// bound by instruction issue, while later the vector ALU has slack under the memory traffic.
// One wavefront, two channels per lane.
//   pid, wk, wv  page id of position L and this lane's two channels of the new K and V vectors,
//         loaded by the caller at the start of the range
//   scr   LDS scratch of 256 floats (16-byte aligned) that no buffer below overlaps
//   kdst, vdst, mdst  the K buffer, a V buffer and its metadata buffer
// HP: the 128 values are the new vectors of two neighbouring 64-channel kv heads (lanes 0-31 hold
// the first head's channels), quantised and stored per head; `kvh` counts pairs.
template <int G, bool HP, bool DN>
__device__ __forceinline__ void append_token(const DecodeParams& p, int kvh, int lane, int L, int pid,
                                             uint32_t wk, uint32_t wv, float* __restrict__ scr,
                                             uint8_t* __restrict__ kdst, uint8_t* __restrict__ vdst,
                                             uint8_t* __restrict__ mdst, NewToken& nt) {
  constexpr int D = 128;
  constexpr int DH = HP ? 64 : 128;  // channels of one head
  float* const yb = scr;            // [2][128]: K and V for the rotation
  const int slot = L & 15;
  nt.place = pid >= 0 && pid < p.num_pages;                  // otherwise attended to but not stored
  const int head = HP ? 2 * kvh + (lane >> 5) : kvh;         // kv head of this lane's two channels
  nt.vec = ((int64_t)pid * p.n_kv_heads + head) * 16 + slot;
  // K and V go through every step together (index 0: K, 1: V): one two-vector transform instead of
  // two single ones, and reductions that overlap each other
  const bool rot[2] = {p.rot_k != 0, p.rot_v != 0};                                // block Hadamard
  const bool dns[2] = {DN && p.dense_k != 0, DN && p.dense_v != 0};                  // learned rotation after it
  float x[2][2];
  if (p.kv_new_dtype == SAW_BF16) { widen2<SAW_BF16>(wk, x[0][0], x[0][1]); widen2<SAW_BF16>(wv, x[1][0], x[1][1]); }
  else                            { widen2<SAW_F16>(wk, x[0][0], x[0][1]);  widen2<SAW_F16>(wv, x[1][0], x[1][1]); }
  if (p.has_signs) {                                         // x diag(sigma), as the store kernel does
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      if (rot[w]) {
        x[w][0] = apply_sign(p.signs, (2 * lane) & (DH - 1), x[w][0]);
        x[w][1] = apply_sign(p.signs, (2 * lane + 1) & (DH - 1), x[w][1]);
      }
    }
  }
  if (rot[0] || rot[1] || dns[0] || dns[1]) {
    *(f32x2*)(yb + 2 * lane) = f32x2{x[0][0], x[0][1]};
    *(f32x2*)(yb + D + 2 * lane) = f32x2{x[1][0], x[1][1]};
    wave_sync();
    if (rot[0] && rot[1]) wave_lds_fwht128<2>(yb, p.had_block, lane);
    else if (rot[0]) wave_lds_fwht128<1>(yb, p.had_block, lane);
    else if (rot[1]) wave_lds_fwht128<1>(yb + D, p.had_block, lane);
    if constexpr (DN) {                                    // k^ = (k H_b) R_l, the same for V (App. A.3)
      if (dns[0] && dns[1]) wave_lds_matvec128<2>(yb, p.dense, lane);
      else if (dns[0]) wave_lds_matvec128<1>(yb, p.dense, lane);
      else if (dns[1]) wave_lds_matvec128<1>(yb + D, p.dense, lane);
    }
    const f32x2 yk = *(const f32x2*)(yb + 2 * lane), yv = *(const f32x2*)(yb + D + 2 * lane);
    x[0][0] = yk.x; x[0][1] = yk.y; x[1][0] = yv.x; x[1][1] = yv.y;
    wave_sync();
  }
  // min and max over each head's values (128: all lanes, 64: half of them): reductions of
  // (max, -min) pairs, rows first (DPP)
  float mx[2], nmn[2];
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    mx[w] = row_allmax(fmaxf(x[w][0], x[w][1]));
    nmn[w] = row_allmax(-fminf(x[w][0], x[w][1]));
  }
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    mx[w] = max_xor16(mx[w]);
    nmn[w] = max_xor16(nmn[w]);
    if (!HP) {
      mx[w] = max_xor32(mx[w]);
      nmn[w] = max_xor32(nmn[w]);
    }
  }
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const float norm = rot[w] ? had_norm(p.had_block) : 1.0f;
    const float mn = -nmn[w];
    const float range = mx[w] - mn;
    float inv, zq, s_store, z_store;
    if (range > 0.0f) {
      inv = 15.0f / range;
      s_store = range * (norm * (1.0f / 15.0f));
      zq = rintf(-mn * inv);
      z_store = zq;
    } else {  // constant vector
      inv = 0.0f;
      zq = 0.0f;
      s_store = (mn != 0.0f) ? fabsf(mn) * norm : 1.0f;
      z_store = (mn > 0.0f) ? -1.0f : ((mn < 0.0f) ? 1.0f : 0.0f);
    }
    const float c0 = __builtin_amdgcn_fmed3f(rintf(x[w][0] * inv) + zq, 0.0f, 15.0f);
    const float c1 = __builtin_amdgcn_fmed3f(rintf(x[w][1] * inv) + zq, 0.0f, 15.0f);
    const uint8_t byte = (uint8_t)((uint32_t)c0 | ((uint32_t)c1 << 4));
    const bool meta_lane = (lane & (DH / 2 - 1)) == 0;        // lane 0 (and lane 32 for the pair's second head)
    nt.byte[w] = byte;
    nt.meta[w] = f32x2{s_store, z_store};
    // token 0 of page 0 of the batch: its 64 code bytes are the first 64 bytes of the tile (chunk Q of
    // token 0 sits at chunk position Q), its pairs the first of the metadata block (head pair: one per head)
    (w ? vdst : kdst)[lane] = byte;
    if (meta_lane)
      *(f32x2*)(mdst + (w ? kMetaBytesOf(HP) / 2 : 0) + (HP ? 128 * (lane >> 5) : 0)) = f32x2{s_store, z_store};
  }
  wave_sync();
}

// one batch's (scale, zero) pairs: K 4 pages x 128 B, then V (twice that for a pair of 64-channel heads)
template <bool HP> constexpr int kMetaBytes = HP ? 2048 : 1024;
// The P buffer is never a transfer target.  Up to G = 4 it also serves, at the start of a range, as the
// query preparation's scratch (the rotated query rows, at most 2 KB), so that this work touches no
// memory a transfer may be writing.
template <int G, bool HP> constexpr int kWaveLdsG = 12 * kTileBytes + kPbufBytes + 2 * kMetaBytes<HP>;   // per wavefront: K buffer, two V buffers, P buffer, two metadata buffers

// Two ways of giving wavefronts their work.
//
// PAIR = false: NW wavefronts share one (sequence, kv head, partition): wavefront w takes batches
// w, w + NW, ... and the block folds their running (max, sum, accumulator) states together in LDS
// at the end; with several partitions the result goes to the workspace for the merge kernel.
//
// PAIR = true (one partition per sequence, batch too large for every wavefront to need help):
// a block of NW = 2 or 4 wavefronts owns the sequences at ranks r and B-1-r of the longest-first
// order and splits their batches, laid end to end (long, then short), into NW equal shares: a
// wavefront gets a stretch of the long sequence, of the short one, or - one wavefront per block
// at most - the end of the long one and the start of the short one.  A sequence that one
// wavefront covers alone is finished by it; otherwise each wavefront leaves its share as a
// (max, sum, accumulator) record in LDS and counts itself in with an LDS atomic, and whichever
// comes last combines the records (always in wavefront order) and writes the output, so nobody
// waits for anybody.  The wavefront with two stretches takes the short sequence's first, so the
// record it leaves in its own buffers is its last act; the short sequence's record, if that one
// is shared too (NW = 4 only), goes to a spare slot of the block.  Every wavefront of the launch
// then streams the same number of tokens (give or take a batch) however ragged the batch is,
// with no partial results in global memory.  NW = 4 keeps the chip's 2048 wavefront slots busy
// when there are only 512 to 1024 (sequence, kv head) items.
enum SegMode : int { kSegSplitKV = 0, kSegAlone = 1, kSegShare = 2 };

//
// HP = true ("head pair") serves head_dim 64 with an even number of kv heads: the block's kv "head" is
// a pair of neighbouring 64-channel heads, whose code tiles ([head][token][32 B]) and metadata are
// contiguous in a page.  The transfers re-order a pair's tiles into rows of 128 channels (head 2j's
// 64, then head 2j+1's), the G query rows (G/2 per kv head) carry zeros in the other head's half,
// and everything between the transfers and the epilogue runs exactly as for head_dim 128; only the
// (scale, zero) pairs are per (token, kv head), and a row's own 64 output channels are kept.
// PK (pair mode): sequences per block, 2 (ranks r and B-1-r) or 3 (ranks r, 2n-1-r and 2n+r with
// n = ceil(B/3): the first two add up alike, the third makes the totals differ by up to a third of
// the spread of the lengths).  Four wavefronts over three sequences put 4/3 wavefronts on a (sequence,
// kv head) item, which fills the chip when there are 1025 to 1536 items - too many for four
// wavefronts per pair, and with two per pair a quarter to a half of the slots would stay empty.
template <int G, int NW, bool PAIR, bool HP = false, int PK = 2, bool DN = false>
// (a launch of this kernel puts at most 8 wavefronts on a compute unit, 2 per SIMD: let the
// register allocator use the 256 registers that leaves each of them)
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void decode_int4_mfma_kernel(DecodeParams p) {
  static_assert(!PAIR || NW == 2 || NW == 4, "a pair block has two or four wavefronts");
  static_assert(!HP || G >= 2, "a head pair has at least one query head per kv head");
  static_assert(!(HP && DN), "the learned rotation is built for head_dim 128");
  constexpr int D = 128;                       // channels of a row (a head, or a pair of 64-channel heads)
  constexpr int DH = HP ? 64 : 128;            // channels of one head
  constexpr int GK = HP ? G / 2 : G;           // query heads per kv head
  constexpr int KV = (HP && G <= 4) ? 2 : 1;   // kv heads whose metadata one lane needs (G = 8: its own only)
  constexpr int NS = (G > 4) ? 2 : 1;          // tokens per lane in the softmax layout
  constexpr int NH = (G > 4) ? 4 : G;          // heads per lane in the softmax layout
  constexpr int LO = (G > 4) ? 8 : 4;          // first row of the lo limbs of P
  constexpr int STEP = PAIR ? 1 : NW;          // batch stride of a wavefront inside its range
  // (which partition a block takes is rotated by its kv head and sequence: blocks go to the XCDs round
  // robin in launch order, and with the partition index as the fastest grid index and a partition count
  // that shares a factor with 8 every XCD would serve a fixed set of partition indices - of a ragged
  // batch the later partitions are mostly empty, so some XCDs got most of the work: 33 sequences x 8
  // partitions 41 us against 28-32 us with 7 or 9 partitions)
  const int split = (blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x;
  const int kvh = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int first_batch = PAIR ? 0 : wave;     // first batch of this wavefront inside its range

  constexpr int kWaveLds = kWaveLdsG<G, HP>;
  // One shared array for everything, the pair counter included: with a single LDS object the
  // compiler keeps the restrict scopes of the helpers' pointer arguments, which is what lets their LDS
  // accesses proceed while transfers are in flight (with two objects it replaces those scopes by
  // per-object ones and then orders every LDS access behind every transfer).
  constexpr int kRecFloats = G * 128 + 2 * G;                   // a record: accumulator rows, then (max, sum) per row
  constexpr int K = PAIR ? PK : 1;                              // sequences of a pair-mode block
  static_assert(PK == 2 || PK == 3, "a block takes two or three sequences");
  // (a wavefront can hold the head of a shared sequence and, after it, an earlier sequence of the block
  // only when the block has more than two wavefronts or more than two sequences: then that record
  // needs a slot outside the wavefront's own buffers)
  constexpr bool kSpare = PAIR && (NW > 2 || K > 2);
  constexpr int kSpareBytes = kSpare ? (K - 1) * kRecFloats * 4 : 0;
  __shared__ __attribute__((aligned(16))) uint8_t lds_all[NW * kWaveLds + 16 + kSpareBytes];
  uint8_t* const kbuf = lds_all + wave * kWaveLds;
  uint8_t* const vbuf_a = kbuf + 4 * kTileBytes;
  uint8_t* const vbuf_b = kbuf + 8 * kTileBytes;
  uint8_t* const pbuf = kbuf + 12 * kTileBytes;
  uint8_t* const mbuf_a = pbuf + kPbufBytes;   // metadata of the batch in vbuf_a / vbuf_b
  uint8_t* const mbuf_b = mbuf_a + kMetaBytes<HP>;
  int* const done_cnt = (int*)(lds_all + NW * kWaveLds);        // PAIR: records left so far of the block's sequences [k]
  float* const spare_rec = (float*)(lds_all + NW * kWaveLds + 16);   // PAIR, NW = 4: spare record of sequence k >= 1 at (k - 1) * kRecFloats

  // ---- the ranges this wavefront streams: (sequence, first token, end token, what to do with the result) ----
  int nseg = 1;
  // (a wavefront has at most one range per sequence of its block; the arrays are read with
  // select chains, never indexed at run time)
  constexpr int MS = (K > 2) ? K : 2;
  int sg_t0[MS], sg_t1[MS], sg_mode[MS], sg_seq[MS];   // per range: tokens, mode, which of the block's sequences
  int bk[MS], lk[MS];                                   // per sequence of the block: index in the batch, cached tokens
#pragma unroll
  for (int i = 0; i < MS; ++i) { sg_t0[i] = 0; sg_t1[i] = 0; sg_mode[i] = kSegAlone; sg_seq[i] = 0; bk[i] = 0; lk[i] = 0; }
  bk[0] = (int)blockIdx.z; sg_t0[0] = split * p.chunk_tokens; sg_mode[0] = kSegSplitKV;
  uint32_t part_mask[MS];                      // PAIR: wavefronts with a share of sequence k of the block
#pragma unroll
  for (int i = 0; i < MS; ++i) part_mask[i] = 0u;
  if (PAIR) {
    const int B = p.batch;
    if (threadIdx.x < 4) done_cnt[threadIdx.x] = 0;
    __syncthreads();                                    // nothing in flight yet: a plain barrier is fine here
    // the block's sequences by length rank, longest first; rank >= B: no such sequence
    int rk[K], nbk[K], stk[K];
    bool present[K];
    if (K == 2) {
      rk[0] = blockIdx.z; rk[1] = B - 1 - rk[0];
      present[0] = true; present[1] = rk[1] != rk[0];   // odd batch: the middle sequence is alone
    } else {
      const int n3 = (B + 2) / 3;
      rk[0] = blockIdx.z; rk[1] = 2 * n3 - 1 - rk[0]; rk[K - 1] = 2 * n3 + rk[0];
      present[0] = true; present[1] = rk[1] < B; present[K - 1] = rk[K - 1] < B;
    }
    if (p.order) {
      // the caller supplied the longest-first order: two dependent loads per sequence instead of the ranking
      int oi[K], raw[K];
#pragma unroll
      for (int k = 0; k < K; ++k) oi[k] = present[k] ? p.order[rk[k]] : 0;
#pragma unroll
      for (int k = 0; k < K; ++k) bk[k] = min(max(oi[k], 0), B - 1);
#pragma unroll
      for (int k = 0; k < K; ++k) raw[k] = present[k] ? p.seq_lens[bk[k]] : 0;
#pragma unroll
      for (int k = 0; k < K; ++k) lk[k] = present[k] ? max(min(raw[k] + p.len_bias, p.bound), 0) : 0;
    } else {
      const LenClasses lc = build_len_classes(p, B, lane, (int*)kbuf);
#pragma unroll
      for (int k = 0; k < K; ++k) {
        bk[k] = present[k] ? seq_of_rank(lane, lc, rk[k]) : 0;
        lk[k] = present[k] ? lc.lens[bk[k]] : 0;
      }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) nbk[k] = (lk[k] + 63) >> 6;
    // Shares of the sequences' batches laid end to end: wavefront w takes [T w / NW, T (w+1) / NW).
    // A wavefront that gets the end of one sequence and the start of the next pays another
    // prologue, about the time of two or three batches: that cost sits in front of every sequence
    // but the first as kGap batches nobody streams (stk[k] is where sequence k starts; 2 and 3
    // measured 1-2 % better than their neighbours for blocks of two and of four).
    constexpr int kGap = (NW > 2) ? 3 : 2;
    int T = 0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      stk[k] = T + ((k > 0 && nbk[k] > 0) ? kGap : 0);
      T = stk[k] + nbk[k];
    }
#pragma unroll
    for (int w = 0; w < NW; ++w) {       // (T < 2^27 batches: the products fit 32 bits)
      const int lo_w = (int)(((uint32_t)T * (uint32_t)w) / NW), hi_w = (int)(((uint32_t)T * (uint32_t)(w + 1)) / NW);
#pragma unroll
      for (int k = 0; k < K; ++k)
        if (max(lo_w, stk[k]) < min(hi_w, stk[k] + nbk[k])) part_mask[k] |= 1u << w;
    }
    const int lo = (int)(((uint32_t)T * (uint32_t)wave) / NW), hi = (int)(((uint32_t)T * (uint32_t)(wave + 1)) / NW);
    nseg = 0;
    // Last sequence first: what a wavefront streams last is then the sequence it shares with the
    // wavefronts before it, whose record can stay in its own buffers.  A sequence without cached
    // tokens has no share: its zero row - or, with a fused append, an empty range that still
    // attends to the new token - goes to the last wavefront (the first, for the block's longest).
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      const int p0 = max(lo, stk[k]), p1 = min(hi, stk[k] + nbk[k]);
      bool add = false;
      int t0 = 0, t1 = 0, mode_k = kSegAlone;
      if (p0 < p1) {
        add = true;
        t0 = 64 * (p0 - stk[k]); t1 = min(lk[k], 64 * (p1 - stk[k]));
        mode_k = __popc(part_mask[k]) > 1 ? kSegShare : kSegAlone;
      } else if (present[k] && nbk[k] == 0 && wave == (k == 0 ? 0 : NW - 1)) {
        if (p.append) {
          add = true;
        } else {
          for (int i = lane; i < G * DH; i += 64)
            store_elem(p.out, p.out_dtype, ((int64_t)bk[k] * p.n_q_heads + kvh * G) * DH + i, 0.f);
        }
      }
      if (add) {
#pragma unroll
        for (int i = 0; i < MS; ++i)
          if (i == nseg) { sg_t0[i] = t0; sg_t1[i] = t1; sg_mode[i] = mode_k; sg_seq[i] = k; }
        ++nseg;
      }
    }
    wave_sync();                                        // the ranking's scratch lived in kbuf (and on into vbuf_a)
  } else if (p.sorted) {
    // one block per (sequence, kv head), more blocks than fit the chip at once: blocks are dispatched
    // in index order as earlier ones finish, so taking the sequences longest first leaves the
    // shortest for the end of the launch
    if (p.order) {
      bk[0] = min(max(p.order[blockIdx.z], 0), p.batch - 1);
    } else {
      const LenClasses lc = build_len_classes(p, p.batch, lane, (int*)kbuf);
      bk[0] = seq_of_rank(lane, lc, blockIdx.z);
    }
    wave_sync();
  }

  // The bookkeeping above is wavefront-uniform, but it is read once per range only: parked in vector
  // registers on purpose (the set-up code is short of scalar ones) and brought back when needed.
#pragma unroll
  for (int i = 0; i < MS; ++i) {
    asm volatile("" : "+v"(sg_t0[i]), "+v"(sg_t1[i]), "+v"(sg_mode[i]), "+v"(sg_seq[i]));
    asm volatile("" : "+v"(bk[i]), "+v"(lk[i]), "+v"(part_mask[i]));
  }
  const int row16 = lane & 15, grp = lane >> 4;
  const int64_t head_tile = (int64_t)kvh * kTileBytes;
  const int64_t page_stride = (int64_t)p.n_kv_heads * (HP ? kTileBytes / 2 : kTileBytes);
  const int64_t head_meta = (int64_t)kvh * (HP ? 64 : 32);        // floats
  const int64_t page_meta = (int64_t)p.n_kv_heads * 32;
  // lane l fills LDS chunk l of a tile = token t = l/4, stored quarter (l & 3) = (Q + t/4) & 3;
  // quarter Q of a row is 16 source bytes: of the token's 64 (head_dim 128), or half Q & 1 of the
  // token's 32 in head Q >> 1 of the pair, whose tiles follow each other
  const int q_src = ((lane & 3) - (lane >> 4)) & 3;
  const int g_swz = HP ? 512 * (q_src >> 1) + 32 * (lane >> 2) + 16 * (q_src & 1) : 64 * (lane >> 2) + 16 * q_src;
  const uint32_t kbias = bf16_bias();
  // ---- per-lane constants ----
  const int kr_off = 16 * (4 * row16 + ((grp + (row16 >> 2)) & 3));                 // K read: t = row16, Q = grp
  int vr_off[8];
#pragma unroll
  for (int c = 0; c < 8; ++c)
    vr_off[c] = grp * kTileBytes + 16 * (4 * row16 + (((c >> 1) + (row16 >> 2)) & 3)) + 8 * (c & 1);
  // P write column inside the batch: 16*page + 8*(t/8) + perm^-1(t%8),  perm^-1(u) = (u&3)<<1 | u>>2
  const int pcol_t = (row16 & 8) + (((row16 & 3) << 1) | ((row16 >> 2) & 1));
  const int head0 = (G > 4) ? 4 * (grp & 1) : 0;                                    // first head of this lane
  const uint32_t pa_addr = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)pbuf + (row16 * kProw + 16 * grp) * 2;   // LDS byte address

#pragma unroll 1
  for (int seg = 0; seg < nseg; ++seg) {
#define SAW_SEG(a) (seg == 0 ? a[0] : (seg == 1 || MS == 2) ? a[1] : a[MS - 1])
#define SAW_SEQ(a) (sq == 0 ? a[0] : (sq == 1 || MS == 2) ? a[1] : a[MS - 1])
  const int sq = __builtin_amdgcn_readfirstlane(SAW_SEG(sg_seq));
  const int b = __builtin_amdgcn_readfirstlane(SAW_SEQ(bk));
  const int t_begin = __builtin_amdgcn_readfirstlane(SAW_SEG(sg_t0));
  const int mode = __builtin_amdgcn_readfirstlane(SAW_SEG(sg_mode));
  const int64_t pt_row = (int64_t)b * p.max_pages;
  // Page ids: lane l of `pidv` holds the (clamped) physical page of logical page
  // pg_first + 64*window + l, i.e. one vector load covers a window of 16 batches; `pidv_nx` is
  // the following window, loaded a window ahead.  A batch takes its four ids with v_readlane, so
  // no page-table latency sits between consecutive batches.  The first load does not wait for
  // the sequence length: entries past the sequence's last page are read (inside the row) and
  // clamped to a valid page, and the tokens they stand for are masked out below.
  const int pg_first = t_begin >> 4;
#define SAW_LOAD_PIDS(dst, first) dst = p.page_table[pt_row + min((first) + lane, p.max_pages - 1)];
#define SAW_CLAMP_PID(id) (((id) < 0 || (id) >= p.num_pages) ? 0 : (id))
  int pidv, pidv_nx;                 // pidv_nx stays unclamped until it becomes pidv
  int window = 0;                    // 16-batch window pidv covers
  SAW_LOAD_PIDS(pidv, pg_first)
  int t_end, seq_len_b;                // seq_len_b: cached tokens of the sequence (= position of an appended token)
  if (PAIR) {
    t_end = __builtin_amdgcn_readfirstlane(SAW_SEG(sg_t1));
    seq_len_b = __builtin_amdgcn_readfirstlane(SAW_SEQ(lk));
  } else {
    seq_len_b = max(min(p.seq_lens[b] + p.len_bias, p.bound), 0);
    t_end = min(seq_len_b, t_begin + p.chunk_tokens);
    if (t_begin >= t_end && !(p.append && t_begin == 0)) {            // block-uniform
      if (p.num_splits == 1)           // empty sequence and no merge pass: the output row is zero
        for (int i = threadIdx.x; i < G * DH; i += 64 * NW)
          store_elem(p.out, p.out_dtype, ((int64_t)b * p.n_q_heads + kvh * G) * DH + i, 0.f);
      return;
    }
  }
  SAW_LOAD_PIDS(pidv_nx, pg_first + 64)
  // this lane's share of the G query vectors (element lane + 64 j), issued ahead of the code transfers
  uint32_t qbits[2 * G];
  {
    // (the block's G query heads are contiguous: G x 128 values, or G x 64 for a head pair)
    constexpr int NQ = HP ? G : 2 * G;
    const int64_t qoff = ((int64_t)b * p.n_q_heads + kvh * G) * DH + lane;
    if (p.q_dtype == SAW_F32) {
#pragma unroll
      for (int j = 0; j < 2 * G; ++j) qbits[j] = (j < NQ) ? ((const uint32_t*)p.q)[qoff + 64 * j] : 0u;
    } else {
#pragma unroll
      for (int j = 0; j < 2 * G; ++j) qbits[j] = (j < NQ) ? ((const uint16_t*)p.q)[qoff + 64 * j] : 0u;
    }
  }

  // fused append: the range that starts the sequence also takes the step's new token (wavefront
  // 0 of the block when several share the range); its inputs are requested here, with the query
  const bool takes_new = p.append && t_begin == 0 && first_batch == 0;
  uint32_t new_wk = 0, new_wv = 0;
  int new_pid = -1;
  if (takes_new) {
    // (the block's new K|V values are 128 contiguous elements: one head, or a pair of 64-channel heads)
    const int64_t e = ((int64_t)b * p.n_kv_heads * DH + (int64_t)kvh * D) / 2 + lane;
    new_wk = ((const uint32_t*)p.k_new)[e];
    new_wv = ((const uint32_t*)p.v_new)[e];
    // (a length beyond the caller's bound was clamped for the attention; storing at the clamped
    // position would overwrite a cached token, so such a token is attended to but not stored)
    if ((seq_len_b >> 4) < p.max_pages && p.seq_lens[b] <= p.bound) new_pid = p.page_table[pt_row + (seq_len_b >> 4)];
  }

  // (first use of the page ids: only here, so that the query and new-token loads above are in
  // flight while this waits for them)
  pidv = SAW_CLAMP_PID(pidv);
  const int nb = max(t_end - t_begin + 63, 0) >> 6;               // batches of the range (0: only an appended token)
  // last batch of this wavefront (below first_batch if it has none)
  const int my_last = nb - 1 - ((nb - 1 - first_batch) % STEP + STEP) % STEP;

  // ---- fetch: LDS-DMA for the code tiles, registers for this lane's token metadata ----
#define SAW_ROTATE_PIDS(batch)                                                                  \
  if (((batch) >> 4) != window) {                                                               \
    window = (batch) >> 4;                                                                      \
    pidv = SAW_CLAMP_PID(pidv_nx);                                                              \
    SAW_LOAD_PIDS(pidv_nx, pg_first + 64 * window + 64)                                         \
  }
#define SAW_PID(batch, q) __builtin_amdgcn_readlane(pidv, 4 * ((batch) & 15) + (q))
  // (cache policy 2 = "nt": the cache is read once per launch, and marking the transfers as
  // streaming is worth 8-10 % of the whole launch: 150 -> 138 us on the ragged 256-sequence batch)
#define SAW_DMA(gptr, ldsptr)                                                                   \
  __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(gptr), (LDS_AS void*)(ldsptr), 16, 0, 2)
  // V tiles of `batch` into VDST and the batch's metadata into MDST: lanes 0-31 bring the K
  // (scale, zero) pairs, lanes 32-63 the V pairs, 16 bytes (two tokens) each, so the metadata
  // also goes HBM -> LDS and no register is the target of a load that is still in flight
#define SAW_FETCH_V(batch, VDST, MDST)                                                          \
  {                                                                                             \
    SAW_ROTATE_PIDS(batch)                                                                      \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                             \
      const uint8_t* vp = p.v_codes + (int64_t)SAW_PID(batch, q) * page_stride + head_tile;     \
      SAW_DMA(vp + g_swz, VDST + q * kTileBytes);                                               \
    }                                                                                           \
    const int mq = HP ? (lane >> 4) : (lane >> 3) & 3;                                          \
    const int id = mq == 0 ? SAW_PID(batch, 0) : mq == 1 ? SAW_PID(batch, 1)                    \
                 : mq == 2 ? SAW_PID(batch, 2) : SAW_PID(batch, 3);                             \
    if (HP) { /* a page's pairs for both heads are 256 contiguous bytes: one transfer for K, one for V */ \
      const int64_t mo = (int64_t)id * page_meta + head_meta + 4 * (lane & 15);                 \
      SAW_DMA(p.k_meta + mo, MDST);                                                             \
      SAW_DMA(p.v_meta + mo, MDST + 1024);                                                      \
    } else {                                                                                    \
      const float* mp = (lane < 32 ? p.k_meta : p.v_meta) + (int64_t)id * page_meta + head_meta + 4 * (lane & 7); \
      SAW_DMA(mp, MDST);                                                                        \
    }                                                                                           \
  }
  // K tiles of `batch` into KDST (the ids were rotated by the V fetch of the same batch)
#define SAW_FETCH_K(batch, KDST)                                                                \
  {                                                                                             \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                             \
      const uint8_t* kp = p.k_codes + (int64_t)SAW_PID(batch, q) * page_stride + head_tile;     \
      SAW_DMA(kp + g_swz, KDST + q * kTileBytes);                                               \
    }                                                                                           \
  }

  // ---- the first transfers, then the q~ operands ----
  // The first batch's tiles leave as soon as the page ids are here, and the q~ preparation runs while
  // they travel.  For that, two things must hold.  Every load issued so far (page ids, query, new
  // token) is waited for before the transfers go out: the ids are needed now anyway, and with nothing
  // else outstanding no later wait for one of these loads can fall on the transfers.  And the
  // preparation's LDS scratch is memory no transfer of the first batch targets, reached through
  // restrict-qualified pointers: the compiler then orders none of its LDS accesses behind them.
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0)
  if (nb > 0) {
    // issued unconditionally: a wavefront without a batch of its own shadows the last batch
    const int first = min(first_batch, nb - 1);
    SAW_FETCH_V(first, vbuf_a, mbuf_a)
    SAW_FETCH_K(first, kbuf)
  }
  // query scratch: up to G = 4 in the P buffer (no transfer ever targets it), else the second V
  // buffer for the rows (first written by the second batch's transfers, which leave after this)
  float* const qrows = (G <= 4) ? (float*)pbuf : (float*)vbuf_b;
  u32x4 a_q[4];
  float qsum[NH];
  float qmul;
  {
    float qraw[2 * G];
    const bool q_is_f32 = p.q_dtype == SAW_F32, q_is_bf16 = p.q_dtype == SAW_BF16;
#pragma unroll
    for (int j = 0; j < 2 * G; ++j) {                       // all three widenings, then selects
      const float as_f32 = __uint_as_float(qbits[j]);
      const float as_bf16 = __uint_as_float(qbits[j] << 16);
      const float as_f16 = f16_to_f32(qbits[j] & 0xffffu);
      qraw[j] = q_is_f32 ? as_f32 : (q_is_bf16 ? as_bf16 : as_f16);
      // randomised Hadamard: q diag(sigma) first (element lane + 64 j is channel lane + 64 (j & 1))
      if (p.rot_k && p.has_signs) qraw[j] = apply_sign(p.signs, HP ? lane : lane + 64 * (j & 1), qraw[j]);
    }
    prepare_q<G, NH, HP, DN>(p, qraw, lane, qrows, a_q, qsum, qmul);
  }

  f32x4 oacc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) oacc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_ref[NH], lsum[NH], zs[NH];
#pragma unroll
  for (int i = 0; i < NH; ++i) { m_ref[i] = -INFINITY; lsum[i] = 0.f; zs[i] = 0.f; }

  // One batch, whose first token is position tok0 of the sequence.  On entry the transfers of batch bi
  // (V into vcur, K into kb, metadata) are the only ones this wavefront has in flight.
  // The buffers come in as __restrict__ parameters: after inlining that gives the LDS accesses
  // and the LDS-DMA transfers distinct alias scopes, so the compiler's own wait-count insertion
  // does not drain the prefetch before reading a buffer no transfer is writing.  Correctness
  // does not rest on that analysis: the explicit vmcnt(0) below covers everything batch bi needs.
  auto body = [&](const int bi, const int tok0, uint8_t* __restrict__ const kb, uint8_t* __restrict__ const vcur,
                  uint8_t* __restrict__ const vnext, uint8_t* __restrict__ const pb,
                  uint8_t* __restrict__ const mcur, uint8_t* __restrict__ const mnext) __attribute__((always_inline)) {
    // (issued through the builtin, not inline asm, so that the compiler's wait-count pass sees it
    // and stops guarding earlier loads, e.g. the q~ operands, with waits of its own further down)
    __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0): batch bi has landed (codes in LDS, metadata)
    f32x2 km[NS][KV], vm[NS][KV];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int pg = (G > 4) ? (2 * s + (lane >> 5)) : grp;        // page of this lane's token
#pragma unroll
      for (int kv = 0; kv < KV; ++kv) {
        // head pair: [page][kv head][token]; with G = 8 a lane's four heads belong to kv head grp & 1
        const int mo = HP ? 256 * pg + 128 * (G > 4 ? (grp & 1) : kv) + 8 * row16 : 128 * pg + 8 * row16;
        km[s][kv] = *(const f32x2*)(mcur + mo);
        vm[s][kv] = *(const f32x2*)(mcur + kMetaBytes<HP> / 2 + mo);
      }
    }
    // K operand reads first, before the next transfers are issued.
    u32x4 kw[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) kw[q] = *(const u32x4*)(kb + q * kTileBytes + kr_off);
    __builtin_amdgcn_s_waitcnt(0xC07F);                    // lgkmcnt(0): ... and they have returned: kb is free
    // The next batch of this wavefront, if it has one (the branch is wavefront-uniform and the
    // wait at the top of a batch is a full vmcnt(0), so the number of transfers in flight may
    // depend on the path).  vnext was last read two batches ago.
    const int nxt = min(bi + STEP, my_last);
    if (bi + STEP <= my_last) {
      SAW_FETCH_V(nxt, vnext, mnext)
      SAW_FETCH_K(nxt, kb)
    }

    // ---- logits: D_q[head][token of page q] ----
    f32x4 dq[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        acc = mfma_bf16(as_bf16x8(a_q[kk]), unpack8(kw[q][kk], kbias), acc);
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
    float lg[NS][NH];
    bool valid[NS];
    bool need = false;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int pg = (G > 4) ? (2 * s + (lane >> 5)) : grp;
      valid[s] = (tok0 + 16 * pg + row16) < t_end;
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        const int kv = (KV == 2 && i >= G / 2) ? 1 : 0;
        const float kz = km[s][kv].y + 128.f;
        const float v = km[s][kv].x * fmaf(-kz, qsum[i], sraw[s][i]);
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
          mx = max_xor32(mx);      // lanes 32 apart share the head group
        } else {
          mx = max_xor16(mx);
          mx = max_xor32(mx);
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
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        const int kv = (KV == 2 && i >= G / 2) ? 1 : 0;
        const float vs = valid[s] ? vm[s][kv].x : 0.f;
        const float vz = valid[s] ? vm[s][kv].y + 128.f : 0.f;
        const float pr = fast_exp2(lg[s][i] - m_ref[i]);     // exp2(-inf) = 0 for masked tokens
        lsum[i] += pr;
        uint32_t h16, l16;
        float wsum;
        split_bf16(pr * vs, h16, l16, wsum);
        zs[i] = fmaf(wsum, vz, zs[i]);
        ((uint16_t*)pb)[(head0 + i) * kProw + col] = (uint16_t)h16;
        ((uint16_t*)pb)[(LO + head0 + i) * kProw + col] = (uint16_t)l16;
      }
    }
    wave_sync();
    // ---- O[row][channel] += P (rows x 64 tokens) . V codes ----
    // The two P operand reads are issued by hand: written as ordinary LDS loads, the compiler's
    // wait insertion cannot tell them from the buffers the LDS-DMA prefetch is filling and would
    // drain every transfer in flight (s_waitcnt vmcnt(0)) right here.
    u32x4 pa0, pa1;
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(pa0), "=&v"(pa1)
                 : "v"(pa_addr)
                 : "memory");
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const i32x2 tv = __builtin_amdgcn_ds_read_tr4_b64_v2i32((LDS_AS i32x2*)(vcur + vr_off[c]));
      oacc[c] = mfma_bf16(as_bf16x8(pa0), unpack8((uint32_t)tv.x, kbias), oacc[c]);
      oacc[c] = mfma_bf16(as_bf16x8(pa1), unpack8((uint32_t)tv.y, kbias), oacc[c]);
    }
  };
  for (int bi = first_batch; bi < nb; bi += 2 * STEP) {
    body(bi, t_begin + 64 * bi, kbuf, vbuf_a, vbuf_b, pbuf, mbuf_a, mbuf_b);
    if (bi + STEP < nb) body(bi + STEP, t_begin + 64 * (bi + STEP), kbuf, vbuf_b, vbuf_a, pbuf, mbuf_b, mbuf_a);
  }

  // A wavefront without a batch of its own (first_batch >= nb) still has the prologue's transfers of
  // the last batch in flight.  Everything below reuses those buffers as scratch, so they have to
  // have landed first: without this wait a transfer can arrive after the scratch has been written
  // and overwrite it.
  __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0)

  // Fused append: the step's new token is quantised and stored now, placed in the (idle) buffers as
  // token 0 of a batch, and attended to by one more pass of the batch code in which only that token is
  // valid (tok0 = t_end - 1: only position tok0 + 0 lies below t_end; the batch index is past the range,
  // so nothing is requested).
  if (takes_new) {
    NewToken nt;
    append_token<G, HP, DN>(p, kvh, lane, seq_len_b, new_pid, new_wk, new_wv, (float*)vbuf_b, kbuf, vbuf_a, mbuf_a, nt);
    body(0x3fffffff, t_end - 1, kbuf, vbuf_a, vbuf_b, pbuf, mbuf_a, mbuf_b);
    append_store<HP>(p, lane, nt);                         // (nobody waits for these: see append_store)
  }

  // ---- fold the wavefronts of the block together (wavefront 0 keeps the result) ----
  // Every wavefront leaves its state in its own buffers; then all of them work on the fold together:
  // each works out the common reference maximum and the NW weights per head, combines its own slice of
  // the accumulator tiles over all wavefronts into wavefront 0's copy, and wavefront 0 combines the
  // sums.  Two block barriers whatever NW is, instead of one pass per wavefront by wavefront 0 alone.
  if (!PAIR && NW > 1) {
    static_assert(8 % NW == 0, "the accumulator tiles are dealt out evenly");
    constexpr int CPW = 8 / NW;                             // accumulator tiles per wavefront
    float* const st = (float*)kbuf;                         // this wavefront's state: [j][lane]
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) st[(4 * c + i) * 64 + lane] = oacc[c][i];
#pragma unroll
    for (int i = 0; i < NH; ++i) {
      st[(32 + i) * 64 + lane] = m_ref[i];
      st[(36 + i) * 64 + lane] = lsum[i];
      st[(40 + i) * 64 + lane] = zs[i];
    }
    __syncthreads();
    float aw[NW][NH];
#pragma unroll
    for (int i = 0; i < NH; ++i) {
      float mw[NW];
      float mm = -INFINITY;                                 // (wavefront 0 always has a batch: the maximum is finite)
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        mw[w] = ((const float*)(lds_all + w * kWaveLds))[(32 + i) * 64 + lane];
        mm = fmaxf(mm, mw[w]);
      }
#pragma unroll
      for (int w = 0; w < NW; ++w) aw[w][i] = fast_exp2(mw[w] - mm);   // 0 for a wavefront that had no batch
      m_ref[i] = mm;
    }
    float* const st0 = (float*)lds_all;                     // wavefront 0's state
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int c = wave * CPW + cc;
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v = fmaf(aw[w][i], ((const float*)(lds_all + w * kWaveLds))[(4 * c + i) * 64 + lane], v);
        st0[(4 * c + i) * 64 + lane] = v;                   // (only this wavefront touches tile c of that copy now)
      }
    }
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < NH; ++i) {
        float l = 0.f, z = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const float* so = (const float*)(lds_all + w * kWaveLds);
          l = fmaf(aw[w][i], so[(36 + i) * 64 + lane], l);
          z = fmaf(aw[w][i], so[(40 + i) * 64 + lane], z);
        }
        lsum[i] = l;
        zs[i] = z;
      }
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int i = 0; i < NH; ++i) oacc[c][i] = st[(4 * c + i) * 64 + lane];
  }

  // ---- epilogue: reduce the per-lane sums, fold hi + lo rows ----
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    lsum[i] = row_allsum(lsum[i]);
    zs[i] = row_allsum(zs[i]);
    if (G > 4) {
      lsum[i] = add_xor32(lsum[i]);
      zs[i] = add_xor32(zs[i]);
    } else {
      lsum[i] = add_xor16(lsum[i]);
      lsum[i] = add_xor32(lsum[i]);
      zs[i] = add_xor16(zs[i]);
      zs[i] = add_xor32(zs[i]);
    }
  }
  // (the lanes holding the lo rows sit 16 lanes above the hi rows, 32 for G = 8)
  const bool writer = (G > 4) ? (grp < 2) : (grp == 0);
  const int emode = PAIR ? mode : (p.num_splits == 1 ? (int)kSegAlone : (int)kSegSplitKV);
  if (emode == kSegSplitKV) {
    // one of several partitions: (max, sum, un-normalised accumulator) for the merge kernel
#pragma unroll
    for (int i = 0; i < NH; ++i) {
      const int head = head0 + i;
      float* dst = p.ws + (((int64_t)b * p.n_q_heads + kvh * G + head) * p.num_splits + split) * (DH + 2);
      const int own = head / GK;                  // head pair: the half of the row that is this head's
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float o = (G > 4) ? add_xor32(oacc[c][i]) : add_xor16(oacc[c][i]);   // hi rows + lo rows
        if (writer && i < G && (!HP || (c >> 2) == own)) dst[2 + 16 * (HP ? (c & 3) : c) + row16] = o - zs[i];
      }
      if (writer && row16 == 0 && i < G) { dst[0] = m_ref[i]; dst[1] = lsum[i]; }
    }
    return;
  }
  // The range's result as a record (every read of this wavefront's V buffers is done):
  // acc[G][128] (un-normalised, zero-point term removed), then (max, sum) per head.  It lives at the
  // start of the V buffers (with G = 8 the pairs land at the start of the second one), or in the
  // block's spare slot when this wavefront still has its share of the long sequence to stream.
  float* const fb = (float*)vbuf_a;
  // (a shared range that is not this wavefront's last is the start of sequence sq >= 1)
  const bool to_spare = kSpare && emode == kSegShare && seg != nseg - 1;
  float* const rec = to_spare ? spare_rec + (sq - 1) * kRecFloats : fb;
  float* const ml = rec + G * D;
  wave_sync();
#pragma unroll
  for (int i = 0; i < NH; ++i) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float o = (G > 4) ? add_xor32(oacc[c][i]) : add_xor16(oacc[c][i]);   // hi rows + lo rows
      if (writer && i < G) rec[(head0 + i) * D + 16 * c + row16] = o - zs[i];
    }
    if (writer && row16 == 0 && i < G) {
      ml[2 * (head0 + i)] = m_ref[i];
      ml[2 * (head0 + i) + 1] = lsum[i];
    }
  }
  // the records that make up the sequence's result: this one, or with a shared sequence those of
  // every wavefront that has a share, in wavefront order (so the sum does not depend on who
  // happens to come last)
  const float* recs[NW];
#pragma unroll
  for (int k = 0; k < NW; ++k) recs[k] = rec;
  int nrec = 1;
  if (PAIR && emode == kSegShare) {
    // LDS operations of a wavefront complete in order, so the record is in place before the
    // count; the wavefront that finds all others counted does the rest for everybody.
    // the sequence's wavefronts, and those of them that also hold a share of an earlier sequence of
    // the block (at most one: its record is the one in the spare slot)
    uint32_t mask = part_mask[0], lower = 0u;
#pragma unroll
    for (int k = 1; k < K; ++k)
      if (k == sq) { mask = part_mask[k]; } else if (k < sq) { lower |= part_mask[k]; }
    if (sq > 0) lower |= part_mask[0];
    mask = (uint32_t)__builtin_amdgcn_readfirstlane((int)mask);
    lower = (uint32_t)__builtin_amdgcn_readfirstlane((int)lower);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    int before = 0;
    if (lane == 0) before = __hip_atomic_fetch_add(done_cnt + sq, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    before = __builtin_amdgcn_readfirstlane(before);
    if (before != __popc(mask) - 1) {
      // (a record in this wavefront's own buffers is its last act; after one in the spare slot
      // the next range's prologue reuses the buffers)
      wave_sync();
      continue;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    nrec = 0;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
      if ((mask >> k) & 1u) {
        const float* rk = ((lower >> k) & 1u) ? spare_rec + (sq - 1) * kRecFloats
                                              : (const float*)(lds_all + k * kWaveLds + 4 * kTileBytes);
#pragma unroll
        for (int r = 0; r < NW; ++r)
          if (r == nrec) recs[r] = rk;
        ++nrec;
      }
    }
  }
  wave_sync();
  // combine and normalise into this wavefront's buffer.  The weight of record r for head h, the
  // denominator already divided in, is the same in every lane and is worked out first (the (max, sum)
  // pairs sit behind the rows of a record and are read before anything is overwritten); then element by
  // element, in place where the record lives in this buffer.
  float wgt[NW][G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mr[NW], lr[NW];
#pragma unroll
    for (int r = 0; r < NW; ++r) {
      mr[r] = (r < nrec) ? recs[r][G * D + 2 * h] : -INFINITY;
      lr[r] = (r < nrec) ? recs[r][G * D + 2 * h + 1] : 0.f;
    }
    float mm = mr[0];
#pragma unroll
    for (int r = 1; r < NW; ++r) mm = fmaxf(mm, mr[r]);
    float den = 0.f;
#pragma unroll
    for (int r = 0; r < NW; ++r) {
      wgt[r][h] = (PAIR && nrec > 1) ? ((r < nrec) ? fast_exp2(mr[r] - mm) : 0.f) : (r == 0 ? 1.f : 0.f);
      den = fmaf(wgt[r][h], lr[r], den);
    }
    const float inv = __builtin_amdgcn_rcpf(den);
#pragma unroll
    for (int r = 0; r < NW; ++r) wgt[r][h] *= inv;
  }
  wave_sync();
#pragma unroll
  for (int it = 0; it < G * D / 64; ++it) {
    const int idx = lane + 64 * it;
    constexpr int kPerHead = D / 64;                          // iterations per head
    const int h = it / kPerHead;                              // compile-time after unrolling
    float v = wgt[0][h] * recs[0][idx];
    if (PAIR) {
#pragma unroll
      for (int r = 1; r < NW; ++r)
        if (r < nrec) v = fmaf(wgt[r][h], recs[r][idx], v);
    }
    fb[idx] = v;
  }
  wave_sync();
  // rotate back once for V (App. A.4; a learned rotation's transpose first, App. A.3), write the output
  float onorm = 1.0f;
  if constexpr (DN) {
    if (p.dense_v) wave_lds_matvec128<G>(fb, p.dense + kDenseD * kDenseD, lane);
  }
  if (p.rot_v) {
    wave_lds_fwht128<G>(fb, p.had_block, lane);
    onorm = had_norm(p.had_block);
  }
  const int64_t obase = ((int64_t)b * p.n_q_heads + kvh * G) * DH;
  if (HP) {
    for (int i = lane; i < G * D; i += 64) {
      float o = fb[i] * onorm;
      if (p.rot_v && p.has_signs) o = apply_sign(p.signs, i & (DH - 1), o);    // (o~ H_blk) diag(sigma) = o~ R^T
      const int h = i >> 7, c = i & 127;           // a row's own 64 channels; the other half is cross terms
      if ((c >> 6) == h / GK) store_elem(p.out, p.out_dtype, obase + h * 64 + (c & 63), o);
    }
  } else {
    // four consecutive channels per lane: 16-byte (fp32) or 8-byte (16-bit) stores, whole rows per instruction
#pragma unroll
    for (int it = 0; it < (G * D + 255) / 256; ++it) {
      const int i = 4 * (lane + 64 * it);
      if (G * D % 256 != 0 && i >= G * D) break;             // (one query head: 32 lanes hold its row)
      const f32x4 o4 = *(const f32x4*)(fb + i);
      float o[4] = {o4.x * onorm, o4.y * onorm, o4.z * onorm, o4.w * onorm};
      if (p.rot_v && p.has_signs) {                                            // (o~ H_blk) diag(sigma) = o~ R^T
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = apply_sign(p.signs, (i + e) & (DH - 1), o[e]);
      }
      if (p.out_dtype == SAW_F32) {
        *(f32x4*)((float*)p.out + obase + i) = f32x4{o[0], o[1], o[2], o[3]};
      } else {
        uint32_t w0, w1;
        if (p.out_dtype == SAW_BF16) {
          w0 = f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16);
          w1 = f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16);
        } else {
          w0 = f32_to_f16(o[0]) | ((uint32_t)f32_to_f16(o[1]) << 16);
          w1 = f32_to_f16(o[2]) | ((uint32_t)f32_to_f16(o[3]) << 16);
        }
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        *(u32x2_t*)((uint16_t*)p.out + obase + i) = u32x2_t{w0, w1};
      }
    }
  }
  wave_sync();                                   // the next range's prologue reuses these buffers
  }  // ranges of this wavefront
}

#undef SAW_FETCH_V
#undef SAW_FETCH_K
#undef SAW_DMA
#undef SAW_PID
#undef SAW_ROTATE_PIDS
#undef SAW_LOAD_PIDS
#undef SAW_CLAMP_PID
#undef SAW_SEG
#undef SAW_SEQ

template <int G, bool HP, bool DN>
static void launch_g(const DecodeParams& p, int B, int nw, dim3 grid, hipStream_t st) {
  if constexpr (!(HP && G == 8)) {       // (two such blocks of head pairs with eight query rows would not fit LDS)
    if (p.pair == 4 && p.pair_seqs == 3) {
      decode_int4_mfma_kernel<G, 4, true, HP, 3, DN><<<dim3(1, grid.y, (B + 2) / 3), dim3(256), 0, st>>>(p);
      return;
    }
    if (p.pair == 2 && p.pair_seqs == 3) {
      decode_int4_mfma_kernel<G, 2, true, HP, 3, DN><<<dim3(1, grid.y, (B + 2) / 3), dim3(128), 0, st>>>(p);
      return;
    }
  }
  if (p.pair == 4) {
    decode_int4_mfma_kernel<G, 4, true, HP, 2, DN><<<dim3(1, grid.y, (B + 1) / 2), dim3(256), 0, st>>>(p);
    return;
  }
  if (p.pair) {
    decode_int4_mfma_kernel<G, 2, true, HP, 2, DN><<<dim3(1, grid.y, (B + 1) / 2), dim3(128), 0, st>>>(p);
    return;
  }
  if (nw >= 8) decode_int4_mfma_kernel<G, 8, false, HP, 2, DN><<<grid, dim3(512), 0, st>>>(p);
  else if (nw >= 4) decode_int4_mfma_kernel<G, 4, false, HP, 2, DN><<<grid, dim3(256), 0, st>>>(p);
  else if (nw == 2) decode_int4_mfma_kernel<G, 2, false, HP, 2, DN><<<grid, dim3(128), 0, st>>>(p);
  else decode_int4_mfma_kernel<G, 1, false, HP, 2, DN><<<grid, dim3(64), 0, st>>>(p);
}

// `G`: query heads per kv head.  `nw`: wavefronts per (sequence, kv head, partition) block: 1, 2 or
// 4 (ignored in pair mode).  `head_pairs`: head_dim 64, grid.y = n_kv_heads / 2 blocks of two kv
// heads each (2 G rows), G <= 4; otherwise head_dim 128 and grid.y = n_kv_heads.
int launch_decode_int4_mfma(const DecodeParams& p, int G, int B, int nw, bool head_pairs, dim3 grid, hipStream_t st) {
  if (head_pairs) {
    switch (G) {
      case 1: launch_g<2, true, false>(p, B, nw, grid, st); break;
      case 2: launch_g<4, true, false>(p, B, nw, grid, st); break;
      case 4: launch_g<8, true, false>(p, B, nw, grid, st); break;
      default: return SAW_EINVAL;
    }
    return SAW_OK;
  }
  if (p.dense) {                        // a learned rotation after the Hadamard: the kernels that carry its code
    switch (G) {
      case 1: launch_g<1, false, true>(p, B, nw, grid, st); break;
      case 2: launch_g<2, false, true>(p, B, nw, grid, st); break;
      case 4: launch_g<4, false, true>(p, B, nw, grid, st); break;
      case 8: launch_g<8, false, true>(p, B, nw, grid, st); break;
      default: return SAW_EINVAL;
    }
    return SAW_OK;
  }
  switch (G) {
    case 1: launch_g<1, false, false>(p, B, nw, grid, st); break;
    case 2: launch_g<2, false, false>(p, B, nw, grid, st); break;
    case 4: launch_g<4, false, false>(p, B, nw, grid, st); break;
    case 8: launch_g<8, false, false>(p, B, nw, grid, st); break;
    default: return SAW_EINVAL;
  }
  return SAW_OK;
}

}  // namespace saw
