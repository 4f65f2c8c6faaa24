/*
 * saw.h -- C ABI of the SAW-INT4 KV-cache hot path for AMD MI355X (gfx950).
 *
 * Two stages (paper Sec. 3 and Sec. 4.1):
 *   1. saw_rotate_quant_store: block-diagonal Hadamard rotation, token-wise asymmetric
 *      INT4 quantisation and paged store of new K/V tokens, fused in one kernel;
 *   2. saw_paged_decode_attn: one decode step o = softmax(q K^T / sqrt(d)) V read
 *      straight from the INT4 pages, with q rotated instead of un-rotating K and the
 *      output rotated back once for V.
 * plus saw_append_decode_attn (both stages of a decode step in one call, one kernel launch
 * for large batches), saw_flatten_dequant (the prefill-side read-back into dense 16-bit
 * buffers), saw_dequant_pages (fp32 read-back for inspection), and a 16-bit-KV paged
 * decode (saw_kv16_*) that serves as the same-run unquantised comparison.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or keeps them.  `saw_cache_t` itself is a host struct.
 *   - Calls only validate arguments on the host and enqueue kernels on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream); they never
 *     synchronise.  Return 0 on success, a negative SAW_E* code otherwise; on error
 *     nothing was launched.
 *   - Cache layout (one layer):
 *       codes  [num_pages][n_kv_heads][page_size][head_dim/2]  uint8
 *              byte j of a vector = code(2j) | code(2j+1) << 4          (App. A.1)
 *       meta   [num_pages][n_kv_heads][page_size][2]            float32 (scale, zero)
 *     separately for K and V.  A vector is dequantised as scale * (code - zero)
 *     (App. A.1) and lives in the rotated space when its rotate_mask bit is set.
 *   - page_table is [n_seqs][max_pages_per_seq] int32: logical page i of sequence b
 *     is physical page page_table[b][i]; logical position p sits in logical page
 *     p / page_size at slot p % page_size.
 *   - Query head j reads kv head j / (n_q_heads / n_kv_heads).
 *   - Alignment: code pools, K/V inputs, attention and read-back outputs and workspaces 16 bytes; the metadata
 *     pools 8 bytes for the store and 16 bytes for the decode calls (which fetch the pairs with
 *     16-byte transfers); anything else is SAW_EINVAL.
 *   - Supported: page_size 16; head_dim 64 or 128; had_block 1 (no rotation), 16, 32,
 *     64 or 128 with had_block <= head_dim; n_q_heads / n_kv_heads in {1, 2, 4, 8}.
 *   - Randomised Hadamard (Sec. 3): with sign_bits set in the cache descriptor the rotation of
 *     every rotated tensor is R = diag(sigma) H_blk (sigma = +/-1 per channel, one vector for all
 *     heads); the query is multiplied by R as well, outputs and rotated-back read-backs by R^T.
 */
#ifndef SAW_H_
#define SAW_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAW_VERSION 100

/* element types */
#define SAW_F16  1
#define SAW_BF16 2
#define SAW_F32  3

/* rotate_mask bits (Sec. 3: K~ = quant(K H), V~ = quant(V H); the K-only variant clears bit 1) */
#define SAW_ROT_K 1
#define SAW_ROT_V 2

/* error codes */
#define SAW_OK          0
#define SAW_EINVAL     -1   /* unsupported shape, block size, dtype, stride or alignment */
#define SAW_ENULL      -2   /* a required pointer is NULL                               */
#define SAW_EWORKSPACE -3   /* workspace smaller than saw_decode_workspace_bytes(...)   */
#define SAW_ELAUNCH    -4   /* the HIP runtime refused the launch                       */
#define SAW_ESCRATCH   -5   /* saw_paged_decode_attn_static: the call needs more than SAW_STATIC_SCRATCH_BYTES */

/* size of the per-GPU scratch array behind saw_paged_decode_attn_static */
#define SAW_STATIC_SCRATCH_BYTES (16u << 20)

typedef void* saw_stream_t;

typedef struct saw_cache {
  uint8_t* k_codes;     /* device, layout above */
  uint8_t* v_codes;
  float*   k_meta;
  float*   v_meta;
  int32_t  num_pages;
  int32_t  n_kv_heads;
  int32_t  page_size;   /* 16 */
  int32_t  head_dim;    /* 64 | 128 */
  int32_t  had_block;   /* h of BDR-h (Sec. 3 eq. 2-3): 1 | 16 | 32 | 64 | 128 */
  int32_t  rotate_mask; /* SAW_ROT_K | SAW_ROT_V */
  uint32_t sign_bits[4]; /* randomised Hadamard (Sec. 3): bit c (word c / 32, bit c % 32) set = channel c is
                            negated before the block Hadamard, i.e. R = diag(sigma) H_blk; every rotated
                            tensor uses R, the query R as well, outputs and read-backs R^T.  All zero = the
                            plain Hadamard.  Bits at or above head_dim must be zero (SAW_EINVAL). */
  const void* dense_rot; /* learned per-layer rotation R_l (Sec. 3 "Hessian-Aware Quantization", App. A.3): a
                            device buffer filled by saw_prepare_dense_rotation, or NULL for none.  Every tensor
                            whose rotate_mask bit is set is then stored as ((x diag(sigma)) H_blk) R_l (with
                            had_block 1: x R_l), the query takes the same transform and outputs / read-backs its
                            transpose R_l^T first, then the Hadamard's.  head_dim 128 only (SAW_EINVAL otherwise). */
} saw_cache_t;

int saw_version(void);
const char* saw_strerror(int code);

/*
 * Learned per-layer rotation (App. A.3, runtime application: q^ = (q H_b) R_l, k^ = (k H_b) R_l, the same
 * for V).  The calibration that produces R_l is not part of this library: the caller supplies the
 * orthogonal matrix.  saw_prepare_dense_rotation turns it, once per layer, into the operand layouts the
 * kernels read (R_l and its transpose in fp32 for the query / output / read-back products, and three
 * bf16 limbs of R_l in matrix-core operand order for the store kernel, whose product is accurate to
 * fp32 so that the stored codes still follow the rounding-boundary rule):
 *   R         device, [head_dim][head_dim] float32 row-major, y = x R (x a row vector); 16-byte aligned.
 *   prepared  device, at least saw_dense_rotation_bytes(head_dim) bytes, 16-byte aligned; this pointer goes
 *             into saw_cache_t.dense_rot and must stay valid while the cache is used.
 * saw_dense_rotation_bytes returns 0 for an unsupported head_dim (only 128 is supported).
 */
size_t saw_dense_rotation_bytes(int32_t head_dim);
int saw_prepare_dense_rotation(const float* R, int32_t head_dim, void* prepared, size_t prepared_bytes,
                               saw_stream_t stream);

/*
 * Fused rotate -> quantise -> pack -> paged store (Sec. 3 eqs. 1-3, App. A.1, App. A.4).
 *
 * For each new token t < T and kv head g: y = x H_blk (H_blk = diag of orthonormal
 * order-h Sylvester Hadamard blocks; skipped when h == 1 or the tensor's rotate_mask
 * bit is clear), then s = (max y - min y)/15, z = round(-min y / s),
 * c_i = clip(round(y_i/s) + z, 0, 15) over all head_dim channels (one (s, z) per
 * token and head), round = half to even.  A constant vector stores s = |y_0|
 * (1 if zero), z = -sign(y_0), codes 0.  Arithmetic is fp32 on exactly widened inputs.
 *
 *   K, V        device, [T][n_kv_heads][head_dim] of in_dtype (SAW_F16 | SAW_BF16); the
 *               distance between tokens is token_stride_elems (>= n_kv_heads*head_dim,
 *               multiple of 8); base pointers 16-byte aligned.
 *   page_table  device, [n_seqs][max_pages_per_seq].
 *   slots       device, [T][2] int32 = (sequence index, logical position), 8-byte aligned.  Slots must be
 *               unique within a call.  A token whose sequence index, position or page id
 *               is out of range (seq outside [0, n_seqs), position outside
 *               [0, max_pages_per_seq*page_size), page outside [0, num_pages)) is skipped.
 * T == 0 is a no-op.
 */
int saw_rotate_quant_store(const saw_cache_t* cache, const void* K, const void* V,
                           int32_t in_dtype, int64_t T, int64_t token_stride_elems,
                           const int32_t* page_table, int32_t n_seqs, int32_t max_pages_per_seq,
                           const int32_t* slots, saw_stream_t stream);

/*
 * The same store for several layers in ONE kernel launch (App. B: at decode the per-layer KV write is a few
 * microseconds of launch latency, not bandwidth; a caller that has several layers' new K/V at hand - a
 * prefill chunk, a draft model's burst, a cache import - pays that latency once per SAW_MAX_STORE_LAYERS
 * layers instead of once per layer).  Results are those of n_layers calls of saw_rotate_quant_store.
 *
 *   caches      HOST array of n_layers descriptors.  The layers share page_table and slots and must agree in
 *               num_pages, n_kv_heads, page_size, head_dim, had_block, rotate_mask and sign_bits (SAW_EINVAL
 *               otherwise); the pools and the learned rotation (all layers with one, or none) are per layer.
 *   K, V        HOST arrays of n_layers device pointers, each as in saw_rotate_quant_store, with one
 *               token_stride_elems for all.
 * Any n_layers >= 1; more than SAW_MAX_STORE_LAYERS layers go out as several launches.
 */
#define SAW_MAX_STORE_LAYERS 32
int saw_rotate_quant_store_layers(const saw_cache_t* caches, const void* const* K, const void* const* V,
                                  int32_t n_layers, int32_t in_dtype, int64_t T, int64_t token_stride_elems,
                                  const int32_t* page_table, int32_t n_seqs, int32_t max_pages_per_seq,
                                  const int32_t* slots, saw_stream_t stream);

/*
 * Bytes of scratch the decode calls need for these arguments (split-KV partial
 * results [B][n_q_heads][splits][head_dim + 2] float32, rounded up to 16 bytes).  max_seq_len and num_splits
 * have the meaning below; returns 0 on invalid arguments.
 */
size_t saw_decode_workspace_bytes(const saw_cache_t* cache, int32_t B, int32_t n_q_heads,
                                  int32_t max_seq_len, int32_t num_splits);

/*
 * The split-KV geometry saw_paged_decode_attn will use for these arguments (host-side helper
 * for reporting): partitions per sequence and tokens per partition.  Either output may be NULL.
 * (The 16-bit comparison call may choose more partitions for the same arguments;
 * saw_decode_workspace_bytes covers both.)
 */
int saw_decode_plan(const saw_cache_t* cache, int32_t B, int32_t max_seq_len, int32_t num_splits,
                    int32_t* splits_out, int32_t* chunk_tokens_out);

/*
 * Host-side mirror of the longest-first order in which the decode kernels take a large batch's
 * sequences (they derive it themselves from seq_lens on the device; nothing has to be passed in).
 * For inspection and tests: seq_lens_host and order_out are HOST arrays of B <= 1024 entries;
 * order_out[r] = index of the sequence at rank r.  Sequences are ranked by 64 length classes scaled
 * to the longest sequence of the batch (after clamping to max_seq_len; <= 0: no clamp), ties in
 * index order; sequences without cached tokens form the last class alone, so none of them ranks
 * ahead of a non-empty sequence whatever the bound.
 */
int saw_decode_rank_order(const int32_t* seq_lens_host, int32_t B, int32_t max_seq_len, int32_t* order_out);

/*
 * One decode step over the INT4 cache (Sec. 2: o = softmax(q K^T/sqrt(d)) V; Sec. 4.1 and
 * App. A.4: logits (q H_blk) dequant(K~)^T, output Score dequant(V~) H_blk).
 *
 *   q           device, [B][n_q_heads][head_dim] of q_dtype (SAW_F16 | SAW_BF16 | SAW_F32), dense.
 *   seq_lens    device, [B] int32: tokens of sequence b to attend to, positions [0, len).
 *               Lengths are clamped to the bound below.  len == 0 gives a zero output row.
 *   max_seq_len host-side upper bound on seq_lens (sizes the split grid); <= 0 means
 *               max_pages_per_seq * page_size.  Must not exceed that product.
 *   sm_scale    logit scale; <= 0 selects 1/sqrt(head_dim).
 *   out         device, [B][n_q_heads][head_dim] of out_dtype (SAW_F32 | SAW_F16 | SAW_BF16).
 *   workspace   device scratch of at least saw_decode_workspace_bytes(...) bytes, 16-byte
 *               aligned; contents are overwritten; concurrent calls need separate workspaces.
 *   num_splits  split-KV factor (partitions of the context per sequence, merged by
 *               log-sum-exp); 0 picks one from the shape.  Max 1024.
 */
int saw_paged_decode_attn(const saw_cache_t* cache, const void* q, int32_t q_dtype,
                          int32_t B, int32_t n_q_heads,
                          const int32_t* page_table, int32_t max_pages_per_seq,
                          const int32_t* seq_lens, int32_t max_seq_len, float sm_scale,
                          void* out, int32_t out_dtype,
                          void* workspace, size_t workspace_bytes, int32_t num_splits,
                          saw_stream_t stream);

/*
 * Optional hints for the decode calls.  `order`: a device array of B int32, a permutation of 0..B-1 that
 * lists the sequences longest first (ties in any order; sequences without cached tokens LAST - the
 * schedule of a large batch relies on that).  A serving engine knows its lengths on the host and can keep
 * this order at no cost; with it the kernels of a large batch skip their own length ranking (the first
 * microseconds of every wavefront).  Entries outside [0, B) are clamped; an order that is not a permutation
 * or not sorted gives unbalanced work or wrong rows, never an out-of-bounds access.  The order is only
 * read where the launch needs one (one partition per sequence and more than 256 (sequence, kv head)
 * items); hints == NULL or order == NULL: the kernels rank the sequences themselves, which is what
 * saw_paged_decode_attn / saw_append_decode_attn do.  Everything else as in those calls.
 */
/*
 * saw_decode_order computes such an order on the device from the device-resident lengths (exactly
 * longest first after clamping to max_seq_len, <= 0: no clamp; ties in index order, so empty sequences
 * come last), without a host read: one small launch per decode step, whose result serves the hinted
 * call of every layer of the step.  seq_lens, order_out: device, B int32 each; B <= 1024 (larger
 * batches do not use an order).
 */
int saw_decode_order(const int32_t* seq_lens, int32_t B, int32_t max_seq_len, int32_t* order_out,
                     saw_stream_t stream);

typedef struct saw_decode_hints {
  const int32_t* order;
} saw_decode_hints_t;

int saw_paged_decode_attn_hinted(const saw_cache_t* cache, const void* q, int32_t q_dtype,
                                 int32_t B, int32_t n_q_heads,
                                 const int32_t* page_table, int32_t max_pages_per_seq,
                                 const int32_t* seq_lens, int32_t max_seq_len, float sm_scale,
                                 void* out, int32_t out_dtype,
                                 void* workspace, size_t workspace_bytes, int32_t num_splits,
                                 const saw_decode_hints_t* hints, saw_stream_t stream);

int saw_append_decode_attn_hinted(const saw_cache_t* cache, const void* K_new, const void* V_new,
                                  int32_t kv_dtype, const void* q, int32_t q_dtype, int32_t B,
                                  int32_t n_q_heads, const int32_t* page_table, int32_t max_pages_per_seq,
                                  const int32_t* seq_lens, int32_t max_seq_len, float sm_scale, void* out,
                                  int32_t out_dtype, void* workspace, size_t workspace_bytes,
                                  const saw_decode_hints_t* hints, saw_stream_t stream);

/*
 * saw_paged_decode_attn without a workspace argument, for callers that cannot allocate device
 * memory or carry a workspace around: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same kernels, same arguments and same results as saw_paged_decode_attn;
 * the split-KV partial results live in a static device array of SAW_STATIC_SCRATCH_BYTES (16 MiB)
 * that every GPU the library runs on holds until the process ends.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine); its first use on a device resolves the
 * array's address there (hipGetSymbolAddress), so make that first call outside a graph capture.
 *   - A call whose partial results ([B][n_q_heads][splits][head_dim + 2] float32, see
 *     saw_decode_workspace_bytes / saw_decode_plan) exceed the array returns SAW_ESCRATCH and
 *     launches nothing; a smaller num_splits (1 needs 520 B per query row) makes it fit.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it.  Nothing in it has to start at zero and nothing is kept
 *     from one call to the next.
 */
int saw_paged_decode_attn_static(const saw_cache_t* cache, const void* q, int32_t q_dtype,
                                 int32_t B, int32_t n_q_heads,
                                 const int32_t* page_table, int32_t max_pages_per_seq,
                                 const int32_t* seq_lens, int32_t max_seq_len, float sm_scale,
                                 void* out, int32_t out_dtype, int32_t num_splits,
                                 saw_stream_t stream);

/*
 * One whole decode step for a layer in a single call: append this step's K/V token of every
 * sequence to the cache, then attend over the cache including it (Sec. 4.1: "new KV entries
 * are rotated, quantised and written" followed by the rotated-space attention).  The result is
 * that of saw_rotate_quant_store(slots = (b, seq_lens[b])) followed by saw_paged_decode_attn
 * over seq_lens[b] + 1 tokens.  With head_dim 128, and with head_dim 64 when n_kv_heads is even
 * and a kv head serves at most 4 query heads, the decode kernel does the append itself: the
 * wavefront that starts a sequence also quantises the new token, attends to it from on-chip memory
 * (nothing the call writes is read back by it) and stores it, which makes the step ONE kernel launch
 * when there is one partition per sequence (large batches, and small batches of short contexts), and
 * the decode and merge kernels otherwise.  For the remaining head_dim 64 shapes the
 * call enqueues the store and the decode kernels back to back.
 *
 *   K_new, V_new device, dense [B][n_kv_heads][head_dim] of kv_dtype (SAW_F16 | SAW_BF16),
 *               16-byte aligned: token b belongs to sequence b.
 *   seq_lens    device, [B] int32: tokens cached BEFORE this call; the new token goes to
 *               position seq_lens[b] (its page must be mapped in page_table; if it is not, the
 *               token is still attended to but not stored).  A sequence whose length exceeds
 *               max_seq_len breaks the bound: nothing is stored for it and its output row covers a
 *               clamped range only.  Not modified: the caller advances its lengths afterwards.
 *   max_seq_len host-side upper bound on seq_lens (before the append); <= 0 means
 *               max_pages_per_seq * page_size - 1.  max_seq_len + 1 must fit the page table row.
 *   workspace   at least saw_decode_workspace_bytes(cache, B, n_q_heads, max_seq_len + 1, 0) bytes.
 * Everything else as in saw_paged_decode_attn.
 */
int saw_append_decode_attn(const saw_cache_t* cache, const void* K_new, const void* V_new,
                           int32_t kv_dtype, const void* q, int32_t q_dtype, int32_t B,
                           int32_t n_q_heads, const int32_t* page_table, int32_t max_pages_per_seq,
                           const int32_t* seq_lens, int32_t max_seq_len, float sm_scale, void* out,
                           int32_t out_dtype, void* workspace, size_t workspace_bytes,
                           saw_stream_t stream);

/*
 * Dequantise positions [pos_begin, pos_end) of sequence `seq` into dense fp32
 * [pos_end - pos_begin][n_kv_heads][head_dim] buffers: x^ = s (c - z) (App. A.1).  With
 * unrotate != 0 the rotated tensors are multiplied by H_blk once more, which returns them
 * to the original space (H is symmetric and orthonormal, App. A.4; with sign_bits set the factor
 * is R^T = H_blk diag(sigma), the inverse of R).  Either output may be
 * NULL to skip it.  The caller guarantees the positions are backed by valid pages.
 */
int saw_dequant_pages(const saw_cache_t* cache, const int32_t* page_table,
                      int32_t max_pages_per_seq, int32_t seq, int32_t pos_begin, int32_t pos_end,
                      int32_t unrotate, float* k_out, float* v_out, saw_stream_t stream);

/*
 * Flatten-dequantise (the flatten_dequant step of App. B's prefill breakdown; arithmetic of
 * App. A.1 and A.4): positions [pos_begin, pos_end) of sequence `seq` are gathered from the
 * INT4 pages into dense buffers for a prefill / chunked-prefill attention consumer,
 * x^ = s (c - z), multiplied by H_blk once more when unrotate != 0 (by R^T = H_blk diag(sigma) when
 * sign_bits are set; tensors the cache holds rotated return to the original space; with
 * unrotate == 0 they stay in the rotated space).
 *
 *   k_out, v_out  device, [pos_end - pos_begin][n_kv_heads][head_dim] of out_dtype
 *                 (SAW_BF16 | SAW_F16 | SAW_F32), 16-byte aligned, token_stride_elems elements
 *                 between tokens (>= n_kv_heads*head_dim, multiple of 8).  Either may be NULL.
 *   Positions whose page-table entry is outside [0, num_pages) are left unwritten.  A cache with a learned
 *   rotation (dense_rot) can be flattened as stored (unrotate == 0) only: rotating back is SAW_EINVAL here
 *   (saw_dequant_pages does it).
 * pos_end == pos_begin is a no-op.  Errors: SAW_EINVAL for a bad range (negative, reversed,
 * beyond max_pages_per_seq * page_size), dtype, stride or alignment; SAW_ENULL for a null
 * cache / page table.
 */
int saw_flatten_dequant(const saw_cache_t* cache, const int32_t* page_table,
                        int32_t max_pages_per_seq, int32_t seq, int32_t pos_begin, int32_t pos_end,
                        int32_t unrotate, int32_t out_dtype, void* k_out, void* v_out,
                        int64_t token_stride_elems, saw_stream_t stream);

/*
 * 16-bit-KV comparison path (the unquantised cache the paper measures INT4 against):
 * pages are [num_pages][n_kv_heads][page_size][head_dim] of `dtype` (SAW_F16 | SAW_BF16),
 * no rotation, no metadata.  Same argument meaning as the INT4 calls; `cache` supplies
 * only the shape fields (pointers and had_block / rotate_mask are ignored).
 */
int saw_kv16_store(const saw_cache_t* shape, void* k_pages, void* v_pages, int32_t dtype,
                   const void* K, const void* V, int64_t T, int64_t token_stride_elems,
                   const int32_t* page_table, int32_t n_seqs, int32_t max_pages_per_seq,
                   const int32_t* slots, saw_stream_t stream);

int saw_kv16_paged_decode_attn(const saw_cache_t* shape, const void* k_pages, const void* v_pages,
                               int32_t dtype, const void* q, int32_t q_dtype,
                               int32_t B, int32_t n_q_heads,
                               const int32_t* page_table, int32_t max_pages_per_seq,
                               const int32_t* seq_lens, int32_t max_seq_len, float sm_scale,
                               void* out, int32_t out_dtype,
                               void* workspace, size_t workspace_bytes, int32_t num_splits,
                               saw_stream_t stream);

/*
 * Measurement aids (they compute nothing of the method; bench.py reports them next to the kernels' figures).
 *
 * saw_read_probe: a kernel that only READS the cache, in the decode kernel's access pattern - as many
 * single-wavefront blocks as the chip holds of the decode kernel (2048), each walking an equal share of
 * `page_ids` for one kv head in batches of four pages: the K and V code tiles (1 KiB pieces) and the
 * (scale, zero) pairs, one batch ahead, streaming cache policy - and folds what it read into one word per
 * wavefront.  Bytes read: n_pages * n_kv_heads * 2304 (head_dim 128 only).  Timing it gives the read-only
 * streaming ceiling of the memory system for this pattern; with page_ids = 0, 1, 2, ... the plain
 * contiguous read.  `sink`: device, at least 8192 bytes.
 *
 * saw_plain_quant_store_valu: saw_rotate_quant_store restricted to "no rotation" (had_block and
 * rotate_mask are ignored; head_dim 128) on a plain vector-ALU kernel without matrix cores or LDS staging:
 * the leanest plain INT4 store (App. A.1's quantiser, same bytes as the fused kernel with had_block 1), as
 * the comparator for what the fused rotation costs.
 */
int saw_read_probe(const saw_cache_t* cache, const int32_t* page_ids, int64_t n_pages, void* sink,
                   size_t sink_bytes, saw_stream_t stream);
int saw_plain_quant_store_valu(const saw_cache_t* cache, const void* K, const void* V, int32_t in_dtype,
                               int64_t T, int64_t token_stride_elems, const int32_t* page_table,
                               int32_t n_seqs, int32_t max_pages_per_seq, const int32_t* slots,
                               saw_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* SAW_H_ */
