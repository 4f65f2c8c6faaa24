// Kernel argument block shared by the decode kernels.
#pragma once

#include "saw_common.h"

namespace saw {

struct DecodeParams {
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const float* k_meta;
  const float* v_meta;
  const void* q;
  const int32_t* page_table;
  const int32_t* seq_lens;
  float* ws;            // [B][Hq][S][D + 2]: (m, l, acc[D])
  void* out;
  float q_scale;        // sm_scale * log2(e)
  int32_t q_dtype, out_dtype;
  int32_t n_q_heads, n_kv_heads, max_pages, num_pages;
  int32_t had_block, rot_k, rot_v;
  int32_t num_splits, chunk_tokens, bound;
  const void* k_new;    // fused append (matrix-core INT4 path): the step's K, V [B][Hkv][d], else null
  const void* v_new;
  int32_t kv_new_dtype, append;
  int32_t len_bias;     // added to every seq_lens entry (1 when a separate store launch appended a token)
  int32_t sorted;           // matrix-core path, one block per (sequence, kv head): block z takes the sequence of length rank z
  int32_t pair;             // matrix-core path: blocks of this many wavefronts (2 or 4) over (long, short) sequence pairs; 0: off
  int32_t pair_seqs;        // matrix-core path, pair mode: sequences per block, 2 or (with pair == 4) 3
  const int32_t* order;     // matrix-core INT4 path: the caller's longest-first order of the sequences, or null (ranked in the kernel)
  int32_t batch;
  int32_t waves_per_item;   // matrix-core path: wavefronts sharing one partition (1, 2, 4 or 8)
  const float* dense;       // learned rotation R_l (App. A.3): fp32 [128][128], its transpose right behind it; null: none
  int32_t dense_k, dense_v; // R_l applies to K and the query / to V and the output
  int32_t has_signs;        // any bit of `signs` set
  SignBits signs;           // R = diag(sigma) H_blk for every rotated tensor and the query; outputs take R^T
};

// Length classes of the in-kernel longest-first ranking (saw_rank.h), shared with the host-side
// mirror saw_decode_rank_order.  `nbmax` is the batch's longest (clamped) sequence in 64-token
// units.  Class 63 is for sequences without cached tokens only; the others spread over classes
// 0 (longest) to 62 in proportion to their length.
__host__ __device__ inline float rank_scale(int nbmax) { return 63.0f / (float)(nbmax > 1 ? nbmax : 1); }
__host__ __device__ inline int rank_class(int len, float kscale) {
  const int nb = (len + 63) >> 6;
  if (nb == 0) return 63;
  const int c = 62 - (int)((float)(nb - 1) * kscale);
  return c < 0 ? 0 : c;
}

// MFMA INT4 decode (saw_decode_mfma.hip) for head_dim 128, grid = (splits, kv heads, batch), and
// with `head_pairs` for head_dim 64, grid = (splits, kv heads / 2, batch): see decode_head_pairs().
int launch_decode_int4_mfma(const DecodeParams& p, int G, int B, int nw, bool head_pairs, dim3 grid, hipStream_t st);

// head_dim 64 runs on the matrix cores when the kv heads can be taken two at a time (rows of 128
// channels again) and the pair's query heads fit the 16-row tile as hi and lo limbs.
inline bool decode_head_pairs(int head_dim, int n_kv_heads, int G) {
  return head_dim == 64 && n_kv_heads % 2 == 0 && (G == 1 || G == 2 || G == 4);
}
// (sequence, kv head) work items per sequence as the INT4 decode kernels see them
inline int decode_items_per_seq(int head_dim, int n_kv_heads) {
  return (head_dim == 64 && n_kv_heads % 2 == 0) ? n_kv_heads / 2 : n_kv_heads;
}

// MFMA 16-bit-KV decode for head_dim 128 and group sizes up to 4 (saw_decode_kv16_mfma.hip); false: not covered.
bool launch_decode_kv16_mfma(const DecodeParams& p, int G, int kv_dtype, dim3 grid, hipStream_t st);

inline size_t partial_bytes(int B, int Hq, int splits, int D) {
  return (((size_t)B * Hq * splits * (D + 2) * sizeof(float)) + 15) & ~(size_t)15;
}

}  // namespace saw
