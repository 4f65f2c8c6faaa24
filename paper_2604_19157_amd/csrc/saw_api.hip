// C ABI entry points: argument validation on the host, then kernel launches on the
// caller's stream.  No allocation, no synchronisation, no global state.
#include <math.h>

#include <mutex>

#include "saw_decode.h"

// Split-KV scratch of saw_paged_decode_attn_static, the entry point for callers that cannot
// allocate: one array per GPU the library runs on, held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[SAW_STATIC_SCRATCH_BYTES];

namespace saw {


int launch_store(const saw_cache_t*, const void*, const void*, int, int64_t, int64_t, const int32_t*,
                 int32_t, int32_t, const int32_t*, const int32_t*, int32_t, hipStream_t);
int launch_prepare_dense(const float*, void*, hipStream_t);
int launch_decode_order(const int32_t*, int, int, int32_t*, hipStream_t);
int launch_read_probe(const saw_cache_t*, const int32_t*, int64_t, void*, int32_t, hipStream_t);
int launch_plain_store_valu(const saw_cache_t*, const void*, const void*, int, int64_t, int64_t, const int32_t*, int32_t,
                            int32_t, const int32_t*, hipStream_t);
int launch_store_layers(const saw_cache_t*, const void* const*, const void* const*, int, int, int64_t, int64_t,
                        const int32_t*, int32_t, int32_t, const int32_t*, hipStream_t);
int launch_flatten(const saw_cache_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, void*, void*, int64_t,
                   hipStream_t);
int launch_dequant(const saw_cache_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, int32_t,
                   float*, float*, hipStream_t);
int launch_kv16_store(const saw_cache_t*, void*, void*, const void*, const void*, int64_t, int64_t,
                      const int32_t*, int32_t, int32_t, const int32_t*, hipStream_t);
int run_decode(const saw_cache_t* c, bool kv16, const void* k_pages, const void* v_pages, int kv_dtype,
               const void* q, int q_dtype, int B, int Hq, const int32_t* pt, int max_pages,
               const int32_t* seq_lens, float sm_scale, void* out, int out_dtype, void* ws,
               const SplitPlan& plan, const void* k_new, const void* v_new, int kv_new_dtype, int len_bias,
               const int32_t* order, hipStream_t st);

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

static bool shape_ok(const saw_cache_t* c) {
  if (c->page_size != 16) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->n_kv_heads < 1 || c->num_pages < 1) return false;
  return true;
}

static bool block_ok(const saw_cache_t* c) {
  const int h = c->had_block;
  if (!(h == 1 || h == 16 || h == 32 || h == 64 || h == 128)) return false;
  if (h > c->head_dim) return false;
  if (c->rotate_mask & ~(SAW_ROT_K | SAW_ROT_V)) return false;
  // sign bits exist for the head's channels only
  if (c->head_dim == 64 && (c->sign_bits[2] | c->sign_bits[3])) return false;
  // the learned rotation is built for head_dim 128, its prepared buffer read with 16-byte loads
  if (c->dense_rot && (c->head_dim != kDenseD || !aligned16(c->dense_rot))) return false;
  return true;
}


// Split-KV plan.  Partitions are whole multiples of 64 tokens so every wavefront pass
// starts on a page boundary.  The automatic choice aims at about 2048 wavefronts (8 per compute
// unit): one partition per sequence once the batch alone provides them, otherwise partitions of
// at least 256 tokens, and 2 or 4 wavefronts per partition when even those are too few.
// The INT4 kernels (`kv16` false) stay with one partition from 512 (sequence, kv head) items on:
// their pair mode evens out ragged lengths inside the launch at any occupancy, and the merge
// pass costs more than the extra wavefronts bring (256 sequences x 4 kv heads, 2304 tokens each:
// 61 us against 66 us with two partitions; ragged 80 against 84; at 320 items partitions win).
static bool make_plan(const saw_cache_t* c, int B, int max_pages, int max_seq_len, int num_splits,
                      bool kv16, SplitPlan* plan) {
  const int64_t cap = (int64_t)max_pages * c->page_size;
  if (cap <= 0 || cap > 0x7fffffffLL) return false;
  int bound = (max_seq_len <= 0) ? (int)cap : max_seq_len;
  if (bound > cap) return false;
  if (num_splits < 0 || num_splits > 1024) return false;
  const int units = (bound + 63) / 64;                    // 64-token units
  int S = num_splits;
  bool block_of_eight = false;
  if (S == 0) {
    const int64_t items = (int64_t)B * decode_items_per_seq(c->head_dim, c->n_kv_heads);
    // one wavefront per (item, partition), about 8 per compute unit; a quarter more for 257 to 511 items,
    // the zone of mid-size ragged batches, where many partitions of the shorter sequences are empty
    // (48 ragged sequences x 8 kv heads: 6 partitions 37.1 us, 7: 34.4 us, 8: 34.2 us; 33 x 8: 8 partitions
    // 30.3 us, 10: 27.7 us)
    const int64_t slots = (items > 256 && items < 512) ? 2560 : 2048;
    int64_t s = (slots + items - 1) / items;
    const int64_t max_by_min_chunk = (units + 3) / 4;      // partitions of >= 256 tokens
    if (s > max_by_min_chunk) s = max_by_min_chunk;
    if (!kv16 && items >= 512 && B <= 1024) s = 1;
    // Very many partitions (a single long sequence): a quarter of them, each shared by four wavefronts
    // that fold their states in LDS, leaves the merge pass a quarter of the partial records to write
    // and read - as long as every wavefront keeps its 512 tokens (131072 tokens x 8 kv heads: 256
    // partitions 40.0 us, 64 partitions of four wavefronts 37.8 us).
    if (!kv16 && s > 64 && units / (s / 4) >= 32) s /= 4;
    // Small batches of short contexts: ONE block of eight wavefronts per (sequence, kv head) - a compute
    // unit's worth, the wavefronts taking every eighth 64-token batch and folding their states in LDS -
    // covers the whole sequence, so the call is a single launch without partial results in memory and
    // without a merge pass (with a fused append: the whole decode step in one launch).  It pays while
    // every wavefront has at most five batches, or eight when the blocks fill most of the chip
    // (32 sequences x 8 kv heads x 2304 tokens: 26.0 -> 21.8 us, x 4096 tokens: 35.0 -> 31.7 us;
    // 16 x 1024: 20.7 -> 18.0 us; 4 x 2304: 20.5 -> 18.8 us; with longer contexts or fewer blocks the
    // partitions win: 16 x 4096: 23.6 against 27.2 us, 1 x 8192: 20.3 against 42.4 us).
    const int64_t per_wave = (units + 7) / 8;
    const bool matrix_core_shape = c->head_dim == 128 || c->n_kv_heads % 2 == 0;
    if (!kv16 && matrix_core_shape && items <= 256 && (per_wave <= 5 || (items >= 192 && per_wave <= 8))) {
      s = 1;
      block_of_eight = true;
    }
    if (s < 1) s = 1;
    if (s > 1024) s = 1024;
    S = (int)s;
  }
  if (S > units) S = units;
  if (S < 1) S = 1;
  const int chunk_units = (units + S - 1) / S;
  plan->chunk_tokens = chunk_units * 64;
  plan->num_splits = (units + chunk_units - 1) / chunk_units;
  plan->bound = bound;
  // wavefronts per partition: only when the partitions alone cannot fill the chip (about 2560
  // wavefront slots), and while every wavefront keeps at least 8 batches (512 tokens) of its own
  const int64_t blocks = (int64_t)B * decode_items_per_seq(c->head_dim, c->n_kv_heads) * plan->num_splits;
  int nw = 1;
  while (nw < 4 && blocks * nw * 2 <= 2560 && plan->chunk_tokens / (nw * 2) >= 512) nw *= 2;
  if (block_of_eight && plan->num_splits == 1) nw = 8;
  plan->waves_per_item = nw;
  return true;
}

}  // namespace saw

using namespace saw;

extern "C" {

int saw_version(void) { return SAW_VERSION; }

const char* saw_strerror(int code) {
  switch (code) {
    case SAW_OK: return "ok";
    case SAW_EINVAL: return "invalid argument (shape, Hadamard block, dtype, stride or alignment)";
    case SAW_ENULL: return "null pointer";
    case SAW_EWORKSPACE: return "workspace too small";
    case SAW_ELAUNCH: return "kernel launch failed";
    case SAW_ESCRATCH: return "the split-KV partial results of this call exceed the static scratch of the no-allocation entry point";
    default: return "unknown error";
  }
}

size_t saw_dense_rotation_bytes(int32_t head_dim) { return head_dim == kDenseD ? kDenseBytes : 0; }

int saw_prepare_dense_rotation(const float* R, int32_t head_dim, void* prepared, size_t prepared_bytes,
                               saw_stream_t stream) {
  if (!R || !prepared) return SAW_ENULL;
  if (head_dim != kDenseD || prepared_bytes < kDenseBytes || !aligned16(R) || !aligned16(prepared)) return SAW_EINVAL;
  return launch_prepare_dense(R, prepared, (hipStream_t)stream);
}

int saw_rotate_quant_store(const saw_cache_t* c, const void* K, const void* V, int32_t in_dtype,
                           int64_t T, int64_t token_stride_elems, const int32_t* page_table,
                           int32_t n_seqs, int32_t max_pages_per_seq, const int32_t* slots,
                           saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || !block_ok(c)) return SAW_EINVAL;
  if (in_dtype != SAW_F16 && in_dtype != SAW_BF16) return SAW_EINVAL;
  if (T < 0 || n_seqs < 1 || max_pages_per_seq < 1) return SAW_EINVAL;
  if (T == 0) return SAW_OK;
  if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !K || !V || !page_table || !slots)
    return SAW_ENULL;
  if (token_stride_elems < (int64_t)c->n_kv_heads * c->head_dim || (token_stride_elems & 7)) return SAW_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(c->k_codes) || !aligned16(c->v_codes) ||
      (((uintptr_t)c->k_meta) & 7u) || (((uintptr_t)c->v_meta) & 7u) || (((uintptr_t)slots) & 7u))
    return SAW_EINVAL;
  return launch_store(c, K, V, in_dtype, T, token_stride_elems, page_table, n_seqs, max_pages_per_seq,
                      slots, nullptr, 0, (hipStream_t)stream);
}

int saw_rotate_quant_store_layers(const saw_cache_t* caches, const void* const* K, const void* const* V,
                                  int32_t n_layers, int32_t in_dtype, int64_t T, int64_t token_stride_elems,
                                  const int32_t* page_table, int32_t n_seqs, int32_t max_pages_per_seq,
                                  const int32_t* slots, saw_stream_t stream) {
  if (!caches || !K || !V) return SAW_ENULL;
  if (n_layers < 1) return SAW_EINVAL;
  if (in_dtype != SAW_F16 && in_dtype != SAW_BF16) return SAW_EINVAL;
  if (T < 0 || n_seqs < 1 || max_pages_per_seq < 1) return SAW_EINVAL;
  const saw_cache_t* c0 = caches;
  if (!shape_ok(c0) || !block_ok(c0)) return SAW_EINVAL;
  if (token_stride_elems < (int64_t)c0->n_kv_heads * c0->head_dim || (token_stride_elems & 7)) return SAW_EINVAL;
  if (!page_table || !slots) return T == 0 ? SAW_OK : SAW_ENULL;
  if (((uintptr_t)slots) & 7u) return SAW_EINVAL;
  for (int l = 0; l < n_layers; ++l) {
    const saw_cache_t* c = caches + l;
    // one launch, one shape: the layers of a model agree in everything but their pools, inputs and learned rotation
    if (c->num_pages != c0->num_pages || c->n_kv_heads != c0->n_kv_heads || c->page_size != c0->page_size ||
        c->head_dim != c0->head_dim || c->had_block != c0->had_block || c->rotate_mask != c0->rotate_mask ||
        c->sign_bits[0] != c0->sign_bits[0] || c->sign_bits[1] != c0->sign_bits[1] ||
        c->sign_bits[2] != c0->sign_bits[2] || c->sign_bits[3] != c0->sign_bits[3] ||
        (c->dense_rot != nullptr) != (c0->dense_rot != nullptr))
      return SAW_EINVAL;
    if (!block_ok(c)) return SAW_EINVAL;
    if (T == 0) continue;
    if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !K[l] || !V[l]) return SAW_ENULL;
    if (!aligned16(K[l]) || !aligned16(V[l]) || !aligned16(c->k_codes) || !aligned16(c->v_codes) ||
        (((uintptr_t)c->k_meta) & 7u) || (((uintptr_t)c->v_meta) & 7u))
      return SAW_EINVAL;
  }
  if (T == 0) return SAW_OK;
  for (int l0 = 0; l0 < n_layers; l0 += SAW_MAX_STORE_LAYERS) {       // 32 layers per launch
    const int n = n_layers - l0 < SAW_MAX_STORE_LAYERS ? n_layers - l0 : SAW_MAX_STORE_LAYERS;
    const int rc = launch_store_layers(caches + l0, K + l0, V + l0, n, in_dtype, T, token_stride_elems, page_table,
                                       n_seqs, max_pages_per_seq, slots, (hipStream_t)stream);
    if (rc != SAW_OK) return rc;
  }
  return SAW_OK;
}

int saw_read_probe(const saw_cache_t* c, const int32_t* page_ids, int64_t n_pages, void* sink, size_t sink_bytes,
                   saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || c->head_dim != 128 || n_pages < 1) return SAW_EINVAL;
  if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !page_ids || !sink) return SAW_ENULL;
  if (!aligned16(c->k_codes) || !aligned16(c->v_codes) || !aligned16(c->k_meta) || !aligned16(c->v_meta)) return SAW_EINVAL;
  const int32_t n_waves = (2048 / c->n_kv_heads) * c->n_kv_heads;       // as many as the chip holds of the decode kernel
  if (n_waves < c->n_kv_heads || sink_bytes < (size_t)n_waves * 4) return SAW_EINVAL;
  return launch_read_probe(c, page_ids, n_pages, sink, n_waves, (hipStream_t)stream);
}

int saw_plain_quant_store_valu(const saw_cache_t* c, const void* K, const void* V, int32_t in_dtype, int64_t T,
                               int64_t token_stride_elems, const int32_t* page_table, int32_t n_seqs,
                               int32_t max_pages_per_seq, const int32_t* slots, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || c->head_dim != 128) return SAW_EINVAL;
  if (in_dtype != SAW_F16 && in_dtype != SAW_BF16) return SAW_EINVAL;
  if (T < 0 || n_seqs < 1 || max_pages_per_seq < 1) return SAW_EINVAL;
  if (T == 0) return SAW_OK;
  if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !K || !V || !page_table || !slots) return SAW_ENULL;
  if (token_stride_elems < (int64_t)c->n_kv_heads * c->head_dim || (token_stride_elems & 7)) return SAW_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(c->k_codes) || !aligned16(c->v_codes) ||
      (((uintptr_t)c->k_meta) & 7u) || (((uintptr_t)c->v_meta) & 7u) || (((uintptr_t)slots) & 7u))
    return SAW_EINVAL;
  return launch_plain_store_valu(c, K, V, in_dtype, T, token_stride_elems, page_table, n_seqs, max_pages_per_seq, slots,
                                 (hipStream_t)stream);
}

size_t saw_decode_workspace_bytes(const saw_cache_t* c, int32_t B, int32_t n_q_heads,
                                  int32_t max_seq_len, int32_t num_splits) {
  if (!c || !shape_ok(c) || B < 1 || n_q_heads < 1 || max_seq_len < 1) return 0;
  SplitPlan plan;
  const int max_pages = (max_seq_len + c->page_size - 1) / c->page_size;
  // (the INT4 and the 16-bit calls may choose different partition counts: enough for either)
  SplitPlan plan16;
  if (!make_plan(c, B, max_pages, max_seq_len, num_splits, false, &plan) ||
      !make_plan(c, B, max_pages, max_seq_len, num_splits, true, &plan16))
    return 0;
  return partial_bytes(B, n_q_heads, plan.num_splits > plan16.num_splits ? plan.num_splits : plan16.num_splits,
                       c->head_dim);
}

int saw_decode_plan(const saw_cache_t* c, int32_t B, int32_t max_seq_len, int32_t num_splits,
                    int32_t* splits_out, int32_t* chunk_tokens_out) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || B < 1 || max_seq_len < 1) return SAW_EINVAL;
  SplitPlan plan;
  const int max_pages = (max_seq_len + c->page_size - 1) / c->page_size;
  if (!make_plan(c, B, max_pages, max_seq_len, num_splits, false, &plan)) return SAW_EINVAL;
  if (splits_out) *splits_out = plan.num_splits;
  if (chunk_tokens_out) *chunk_tokens_out = plan.chunk_tokens;
  return SAW_OK;
}

int saw_decode_rank_order(const int32_t* seq_lens_host, int32_t B, int32_t max_seq_len, int32_t* order_out) {
  if (!seq_lens_host || !order_out) return SAW_ENULL;
  if (B < 1 || B > 1024) return SAW_EINVAL;
  const int bound = max_seq_len <= 0 ? 0x7fffffff : max_seq_len;
  int nbmax = 0;
  int cls[1024];
  for (int b = 0; b < B; ++b) {
    const int len = seq_lens_host[b] < 0 ? 0 : (seq_lens_host[b] > bound ? bound : seq_lens_host[b]);
    cls[b] = len;
    const int nb = (int)(((int64_t)len + 63) >> 6);
    if (nb > nbmax) nbmax = nb;
  }
  const float kscale = rank_scale(nbmax);
  for (int b = 0; b < B; ++b) cls[b] = rank_class(cls[b], kscale);
  int n = 0;
  for (int c = 0; c < 64; ++c)                       // class 0 first; inside a class by sequence index
    for (int b = 0; b < B; ++b)
      if (cls[b] == c) order_out[n++] = b;
  return SAW_OK;
}

int saw_decode_order(const int32_t* seq_lens, int32_t B, int32_t max_seq_len, int32_t* order_out, saw_stream_t stream) {
  if (!seq_lens || !order_out) return SAW_ENULL;
  if (B < 1 || B > 1024) return SAW_EINVAL;
  return launch_decode_order(seq_lens, B, max_seq_len <= 0 ? 0x7fffffff : max_seq_len, order_out, (hipStream_t)stream);
}

static int decode_common(const saw_cache_t* c, bool kv16, const void* kp, const void* vp, int kv_dtype,
                         const void* q, int32_t q_dtype, int32_t B, int32_t Hq, const int32_t* pt,
                         int32_t max_pages, const int32_t* seq_lens, int32_t max_seq_len, float sm_scale,
                         void* out, int32_t out_dtype, void* ws, size_t ws_bytes, int32_t num_splits,
                         const saw_decode_hints_t* hints, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c)) return SAW_EINVAL;
  if (!kv16 && !block_ok(c)) return SAW_EINVAL;
  if (kv16 && kv_dtype != SAW_F16 && kv_dtype != SAW_BF16) return SAW_EINVAL;
  if (q_dtype != SAW_F16 && q_dtype != SAW_BF16 && q_dtype != SAW_F32) return SAW_EINVAL;
  if (out_dtype != SAW_F16 && out_dtype != SAW_BF16 && out_dtype != SAW_F32) return SAW_EINVAL;
  if (B < 1 || Hq < 1 || max_pages < 1) return SAW_EINVAL;
  if (B > 65535 || c->n_kv_heads > 65535) return SAW_EINVAL;
  if (Hq % c->n_kv_heads) return SAW_EINVAL;
  const int G = Hq / c->n_kv_heads;
  if (!(G == 1 || G == 2 || G == 4 || G == 8)) return SAW_EINVAL;
  if (!kp || !vp || !q || !pt || !seq_lens || !out || !ws) return SAW_ENULL;
  if (!kv16 && (!c->k_meta || !c->v_meta)) return SAW_ENULL;
  if (!aligned16(kp) || !aligned16(vp) || !aligned16(ws) || !aligned16(out)) return SAW_EINVAL;
  // (the INT4 kernels fetch the (scale, zero) pairs with 16-byte transfers)
  if (!kv16 && (!aligned16(c->k_meta) || !aligned16(c->v_meta))) return SAW_EINVAL;
  if (!isfinite(sm_scale)) return SAW_EINVAL;
  SplitPlan plan;
  if (!make_plan(c, B, max_pages, max_seq_len, num_splits, kv16, &plan)) return SAW_EINVAL;
  const size_t need = partial_bytes(B, Hq, plan.num_splits, c->head_dim);
  if (ws_bytes < need) return SAW_EWORKSPACE;
  return run_decode(c, kv16, kp, vp, kv_dtype, q, q_dtype, B, Hq, pt, max_pages, seq_lens, sm_scale, out,
                    out_dtype, ws, plan, nullptr, nullptr, 0, 0, hints ? hints->order : nullptr, (hipStream_t)stream);
}

int saw_paged_decode_attn(const saw_cache_t* c, const void* q, int32_t q_dtype, int32_t B,
                          int32_t n_q_heads, const int32_t* page_table, int32_t max_pages_per_seq,
                          const int32_t* seq_lens, int32_t max_seq_len, float sm_scale, void* out,
                          int32_t out_dtype, void* workspace, size_t workspace_bytes,
                          int32_t num_splits, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  return decode_common(c, false, c->k_codes, c->v_codes, 0, q, q_dtype, B, n_q_heads, page_table,
                       max_pages_per_seq, seq_lens, max_seq_len, sm_scale, out, out_dtype, workspace,
                       workspace_bytes, num_splits, nullptr, stream);
}

int saw_paged_decode_attn_hinted(const saw_cache_t* c, const void* q, int32_t q_dtype, int32_t B,
                                 int32_t n_q_heads, const int32_t* page_table, int32_t max_pages_per_seq,
                                 const int32_t* seq_lens, int32_t max_seq_len, float sm_scale, void* out,
                                 int32_t out_dtype, void* workspace, size_t workspace_bytes,
                                 int32_t num_splits, const saw_decode_hints_t* hints, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  return decode_common(c, false, c->k_codes, c->v_codes, 0, q, q_dtype, B, n_q_heads, page_table,
                       max_pages_per_seq, seq_lens, max_seq_len, sm_scale, out, out_dtype, workspace,
                       workspace_bytes, num_splits, hints, stream);
}

// The device address of `scratch` on the current device, resolved once per device with that device
// current (every GPU holds its own copy of the array at its own address).
static int static_scratch_ptr(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptrs[kMaxDevices] = {nullptr};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SAW_ELAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SAW_ELAUNCH;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return SAW_OK;
}

int saw_paged_decode_attn_static(const saw_cache_t* c, const void* q, int32_t q_dtype, int32_t B,
                                 int32_t n_q_heads, const int32_t* page_table, int32_t max_pages_per_seq,
                                 const int32_t* seq_lens, int32_t max_seq_len, float sm_scale, void* out,
                                 int32_t out_dtype, int32_t num_splits, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || B < 1 || n_q_heads < 1 || max_pages_per_seq < 1) return SAW_EINVAL;
  // the scratch the plan needs, before anything else: too large is an error of its own
  SplitPlan plan;
  if (!make_plan(c, B, max_pages_per_seq, max_seq_len, num_splits, false, &plan)) return SAW_EINVAL;
  if (partial_bytes(B, n_q_heads, plan.num_splits, c->head_dim) > (size_t)SAW_STATIC_SCRATCH_BYTES) return SAW_ESCRATCH;
  void* ws = nullptr;
  const int rc = static_scratch_ptr(&ws);
  if (rc != SAW_OK) return rc;
  // (nothing in the scratch has to start at zero: every partial record the merge pass reads was
  // written by the decode pass of the same call)
  return decode_common(c, false, c->k_codes, c->v_codes, 0, q, q_dtype, B, n_q_heads, page_table,
                       max_pages_per_seq, seq_lens, max_seq_len, sm_scale, out, out_dtype, ws,
                       (size_t)SAW_STATIC_SCRATCH_BYTES, num_splits, nullptr, stream);
}

static int append_common(const saw_cache_t* c, const void* K_new, const void* V_new, int32_t kv_dtype,
                         const void* q, int32_t q_dtype, int32_t B, int32_t Hq,
                         const int32_t* page_table, int32_t max_pages, const int32_t* seq_lens,
                         int32_t max_seq_len, float sm_scale, void* out, int32_t out_dtype,
                         void* ws, size_t ws_bytes, const saw_decode_hints_t* hints, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || !block_ok(c)) return SAW_EINVAL;
  if (kv_dtype != SAW_F16 && kv_dtype != SAW_BF16) return SAW_EINVAL;
  if (q_dtype != SAW_F16 && q_dtype != SAW_BF16 && q_dtype != SAW_F32) return SAW_EINVAL;
  if (out_dtype != SAW_F16 && out_dtype != SAW_BF16 && out_dtype != SAW_F32) return SAW_EINVAL;
  if (B < 1 || Hq < 1 || max_pages < 1 || B > 65535 || c->n_kv_heads > 65535) return SAW_EINVAL;
  if (Hq % c->n_kv_heads) return SAW_EINVAL;
  const int G = Hq / c->n_kv_heads;
  if (!(G == 1 || G == 2 || G == 4 || G == 8)) return SAW_EINVAL;
  if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !K_new || !V_new || !q || !page_table ||
      !seq_lens || !out || !ws)
    return SAW_ENULL;
  if (!aligned16(K_new) || !aligned16(V_new) || !aligned16(c->k_codes) || !aligned16(c->v_codes) ||
      !aligned16(ws) || !aligned16(out) || !aligned16(c->k_meta) || !aligned16(c->v_meta))
    return SAW_EINVAL;
  if (!isfinite(sm_scale) || max_seq_len < 0) return SAW_EINVAL;
  // the plan covers the lengths after the append (max_seq_len + 1 tokens)
  const int64_t cap = (int64_t)max_pages * c->page_size;
  const int64_t after = (max_seq_len <= 0 ? cap - 1 : (int64_t)max_seq_len) + 1;
  if (after > cap) return SAW_EINVAL;
  SplitPlan plan;
  const bool fused_kernel = c->head_dim == 128 || decode_head_pairs(c->head_dim, c->n_kv_heads, G);
  if (!make_plan(c, B, max_pages, (int)after, 0, false, &plan)) return SAW_EINVAL;
  const size_t need = partial_bytes(B, Hq, plan.num_splits, c->head_dim);
  if (ws_bytes < need) return SAW_EWORKSPACE;
  if (fused_kernel) {
    // the decode kernel stores the new token itself and attends to it from registers (with several
    // partitions per sequence the one that starts the sequence does, and the merge kernel follows);
    // the cached range is [0, seq_lens[b]), bounded by max_seq_len as given
    plan.bound = (int)(after - 1);
    return run_decode(c, false, c->k_codes, c->v_codes, 0, q, q_dtype, B, Hq, page_table, max_pages, seq_lens,
                      sm_scale, out, out_dtype, ws, plan, K_new, V_new, kv_dtype, 0, hints ? hints->order : nullptr,
                      (hipStream_t)stream);
  }
  // head_dim 64 outside the head-pair kernel: two launches from the same call: append (token b -> sequence b at seq_lens[b]),
  // then decode over seq_lens[b] + 1 tokens
  const int rc = launch_store(c, K_new, V_new, kv_dtype, B, (int64_t)c->n_kv_heads * c->head_dim, page_table, B,
                              max_pages, nullptr, seq_lens, (int32_t)(after - 1), (hipStream_t)stream);
  if (rc != SAW_OK) return rc;
  return run_decode(c, false, c->k_codes, c->v_codes, 0, q, q_dtype, B, Hq, page_table, max_pages, seq_lens,
                    sm_scale, out, out_dtype, ws, plan, nullptr, nullptr, 0, 1, hints ? hints->order : nullptr,
                    (hipStream_t)stream);
}

int saw_append_decode_attn(const saw_cache_t* c, const void* K_new, const void* V_new, int32_t kv_dtype,
                           const void* q, int32_t q_dtype, int32_t B, int32_t Hq,
                           const int32_t* page_table, int32_t max_pages, const int32_t* seq_lens,
                           int32_t max_seq_len, float sm_scale, void* out, int32_t out_dtype,
                           void* ws, size_t ws_bytes, saw_stream_t stream) {
  return append_common(c, K_new, V_new, kv_dtype, q, q_dtype, B, Hq, page_table, max_pages, seq_lens, max_seq_len,
                       sm_scale, out, out_dtype, ws, ws_bytes, nullptr, stream);
}

int saw_append_decode_attn_hinted(const saw_cache_t* c, const void* K_new, const void* V_new, int32_t kv_dtype,
                                  const void* q, int32_t q_dtype, int32_t B, int32_t Hq,
                                  const int32_t* page_table, int32_t max_pages, const int32_t* seq_lens,
                                  int32_t max_seq_len, float sm_scale, void* out, int32_t out_dtype,
                                  void* ws, size_t ws_bytes, const saw_decode_hints_t* hints, saw_stream_t stream) {
  return append_common(c, K_new, V_new, kv_dtype, q, q_dtype, B, Hq, page_table, max_pages, seq_lens, max_seq_len,
                       sm_scale, out, out_dtype, ws, ws_bytes, hints, stream);
}

int saw_dequant_pages(const saw_cache_t* c, const int32_t* page_table, int32_t max_pages_per_seq,
                      int32_t seq, int32_t pos_begin, int32_t pos_end, int32_t unrotate, float* k_out,
                      float* v_out, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || !block_ok(c)) return SAW_EINVAL;
  if (seq < 0 || pos_begin < 0 || pos_end < pos_begin || max_pages_per_seq < 1) return SAW_EINVAL;
  if ((int64_t)pos_end > (int64_t)max_pages_per_seq * c->page_size) return SAW_EINVAL;
  if (pos_end == pos_begin) return SAW_OK;
  if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !page_table) return SAW_ENULL;
  if (!k_out && !v_out) return SAW_OK;
  if ((k_out && !aligned16(k_out)) || (v_out && !aligned16(v_out))) return SAW_EINVAL;
  return launch_dequant(c, page_table, max_pages_per_seq, seq, pos_begin, pos_end, unrotate, k_out, v_out,
                        (hipStream_t)stream);
}

int saw_flatten_dequant(const saw_cache_t* c, const int32_t* page_table, int32_t max_pages_per_seq,
                        int32_t seq, int32_t pos_begin, int32_t pos_end, int32_t unrotate,
                        int32_t out_dtype, void* k_out, void* v_out, int64_t token_stride_elems,
                        saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c) || !block_ok(c)) return SAW_EINVAL;
  if (out_dtype != SAW_F16 && out_dtype != SAW_BF16 && out_dtype != SAW_F32) return SAW_EINVAL;
  if (seq < 0 || pos_begin < 0 || pos_end < pos_begin || max_pages_per_seq < 1) return SAW_EINVAL;
  if ((int64_t)pos_end > (int64_t)max_pages_per_seq * c->page_size) return SAW_EINVAL;
  if (token_stride_elems < (int64_t)c->n_kv_heads * c->head_dim || (token_stride_elems % 8)) return SAW_EINVAL;
  if (unrotate && c->dense_rot && (c->rotate_mask & (SAW_ROT_K | SAW_ROT_V))) return SAW_EINVAL;   // not built here
  if (pos_end == pos_begin) return SAW_OK;
  if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !page_table) return SAW_ENULL;
  if (!k_out && !v_out) return SAW_OK;
  if ((k_out && !aligned16(k_out)) || (v_out && !aligned16(v_out))) return SAW_EINVAL;
  return launch_flatten(c, page_table + (int64_t)seq * max_pages_per_seq, pos_begin, pos_end, unrotate,
                        out_dtype, k_out, v_out, token_stride_elems, (hipStream_t)stream);
}

int saw_kv16_store(const saw_cache_t* c, void* k_pages, void* v_pages, int32_t dtype, const void* K,
                   const void* V, int64_t T, int64_t token_stride_elems, const int32_t* page_table,
                   int32_t n_seqs, int32_t max_pages_per_seq, const int32_t* slots, saw_stream_t stream) {
  if (!c) return SAW_ENULL;
  if (!shape_ok(c)) return SAW_EINVAL;
  if (dtype != SAW_F16 && dtype != SAW_BF16) return SAW_EINVAL;
  if (T < 0 || n_seqs < 1 || max_pages_per_seq < 1) return SAW_EINVAL;
  if (T == 0) return SAW_OK;
  if (!k_pages || !v_pages || !K || !V || !page_table || !slots) return SAW_ENULL;
  if (token_stride_elems < (int64_t)c->n_kv_heads * c->head_dim || (token_stride_elems & 7)) return SAW_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(k_pages) || !aligned16(v_pages)) return SAW_EINVAL;
  return launch_kv16_store(c, k_pages, v_pages, K, V, T, token_stride_elems, page_table, n_seqs,
                           max_pages_per_seq, slots, (hipStream_t)stream);
}

int saw_kv16_paged_decode_attn(const saw_cache_t* c, const void* k_pages, const void* v_pages,
                               int32_t dtype, const void* q, int32_t q_dtype, int32_t B,
                               int32_t n_q_heads, const int32_t* page_table, int32_t max_pages_per_seq,
                               const int32_t* seq_lens, int32_t max_seq_len, float sm_scale, void* out,
                               int32_t out_dtype, void* workspace, size_t workspace_bytes,
                               int32_t num_splits, saw_stream_t stream) {
  return decode_common(c, true, k_pages, v_pages, dtype, q, q_dtype, B, n_q_heads, page_table,
                       max_pages_per_seq, seq_lens, max_seq_len, sm_scale, out, out_dtype, workspace,
                       workspace_bytes, num_splits, nullptr, stream);
}

}  // extern "C"
