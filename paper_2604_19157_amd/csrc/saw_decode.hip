// Paged decode attention over the INT4 cache (and over a 16-bit cache for comparison),
// split-KV with a log-sum-exp merge.  Paper: Sec. 2 (decode step), Sec. 4.1 and App. A.4
// (q is rotated once, K is consumed in the rotated space, the output is rotated back
// once for V), App. A.1 (x^ = s (c - z)).
//
// The zero-point never enters the inner loop:
//   q~ . k^_t      = s_t (q~ . c_t) - s_t z_t sum(q~)
//   sum_t p_t v^_t = sum_t (p_t s_t) c_t - sum_t p_t s_t z_t
// Logits are kept in base-2 units (log2 e folded into q~) so the softmax uses exp2.
#include "saw_decode.h"
#include "saw_wave_util.h"

namespace saw {


// In-place un-normalised block Walsh-Hadamard over `n_vec` vectors of length D held in LDS.
template <int D>
__device__ __forceinline__ void lds_fwht(float* x, int n_vec, int h, int tid, int nthreads) {
  for (int st = 1; st < h; st <<= 1) {
    for (int idx = tid; idx < n_vec * (D / 2); idx += nthreads) {
      const int v = idx / (D / 2);
      const int r = idx % (D / 2);
      const int i = v * D + (r / st) * 2 * st + (r % st);
      const float a = x[i], b = x[i + st];
      x[i] = a + b;
      x[i + st] = a - b;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// INT4 decode, VALU formulation.  One 256-thread block per (sequence, kv head, split).
// A wavefront covers 64/LPT tokens per pass; a token's code row is split over LPT lanes.
template <int D, int G, int LPT>
__global__ __launch_bounds__(256) void decode_int4_kernel(DecodeParams p) {
  constexpr int TPW = 64 / LPT;        // tokens per wave pass
  constexpr int CPL = D / LPT;         // codes per lane
  constexpr int WPL = CPL / 8;         // dwords per lane
  // (the partition index is rotated by kv head and sequence, so that no XCD serves a fixed set of partitions)
  const int split = (blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int L = min(p.seq_lens[b] + p.len_bias, p.bound);
  const int t_begin = split * p.chunk_tokens;
  const int t_end = min(L, t_begin + p.chunk_tokens);
  if (t_begin >= t_end) return;

  __shared__ float qs[G * D];
  __shared__ float qsum[G];
  __shared__ float red[4][G][D + 4];

  // ---- q~ = (q H_blk) * sm_scale * log2 e ----
  for (int i = tid; i < G * D; i += 256) {
    const float v = load_elem(p.q, p.q_dtype, ((int64_t)b * p.n_q_heads + kvh * G) * D + i);
    qs[i] = (p.rot_k && p.has_signs) ? apply_sign(p.signs, i % D, v) : v;       // q diag(sigma), then H_blk
  }
  __syncthreads();
  float qmul = p.q_scale;
  if (p.rot_k) {
    lds_fwht<D>(qs, G, p.had_block, tid, 256);
    qmul *= had_norm(p.had_block);
  }
  for (int i = tid; i < G * D; i += 256) qs[i] *= qmul;
  __syncthreads();
  if (tid < G) {
    float s = 0.f;
    for (int c = 0; c < D; ++c) s += qs[tid * D + c];
    qsum[tid] = s;
  }
  __syncthreads();

  const int part = lane % LPT;
  float m[G], lsum[G], zsum[G], acc[G][CPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; lsum[g] = 0.f; zsum[g] = 0.f;
#pragma unroll
    for (int j = 0; j < CPL; ++j) acc[g][j] = 0.f;
  }

  const int64_t pt_row = (int64_t)b * p.max_pages;
  for (int t0 = t_begin + wave * TPW; t0 < t_end; t0 += 4 * TPW) {
    const int t = t0 + lane / LPT;
    const bool valid = t < t_end;
    const int tt = valid ? t : t_end - 1;
    int32_t page = p.page_table[pt_row + (tt >> 4)];
    page = (page < 0 || page >= p.num_pages) ? 0 : page;
    const int64_t vec = ((int64_t)page * p.n_kv_heads + kvh) * 16 + (tt & 15);
    uint32_t kw[WPL], vw[WPL];
    {
      const uint32_t* kp = (const uint32_t*)(p.k_codes + vec * (D / 2)) + part * WPL;
      const uint32_t* vp = (const uint32_t*)(p.v_codes + vec * (D / 2)) + part * WPL;
#pragma unroll
      for (int i = 0; i < WPL; ++i) { kw[i] = kp[i]; vw[i] = vp[i]; }
    }
    const float2 ksz = *(const float2*)(p.k_meta + vec * 2);
    const float2 vsz = *(const float2*)(p.v_meta + vec * 2);

    float dot[G];
#pragma unroll
    for (int g = 0; g < G; ++g) dot[g] = 0.f;
#pragma unroll
    for (int i = 0; i < WPL; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float c = (float)((kw[i] >> (4 * j)) & 15u);
#pragma unroll
        for (int g = 0; g < G; ++g) dot[g] = fmaf(qs[g * D + part * CPL + i * 8 + j], c, dot[g]);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int mk = 1; mk < LPT; mk <<= 1) dot[g] += __shfl_xor(dot[g], mk, SAW_WAVE);
    }
    float w[G];
    bool grow = false;
    float mnew[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float logit = valid ? ksz.x * (dot[g] - ksz.y * qsum[g]) : -INFINITY;
      float mt = logit;
#pragma unroll
      for (int mk = LPT; mk < 64; mk <<= 1) mt = fmaxf(mt, __shfl_xor(mt, mk, SAW_WAVE));
      mnew[g] = fmaxf(m[g], mt);
      grow |= mnew[g] > m[g];
      w[g] = logit;
    }
    if (grow) {  // wave-uniform: m and mt are identical in every lane
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float a = fast_exp2(m[g] - mnew[g]);   // exp2(-inf) = 0 on the first pass
        lsum[g] *= a; zsum[g] *= a;
#pragma unroll
        for (int j = 0; j < CPL; ++j) acc[g][j] *= a;
        m[g] = mnew[g];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float pr = valid ? fast_exp2(w[g] - m[g]) : 0.f;
      lsum[g] += pr;
      w[g] = pr * vsz.x;
      zsum[g] = fmaf(w[g], vsz.y, zsum[g]);
    }
#pragma unroll
    for (int i = 0; i < WPL; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float c = (float)((vw[i] >> (4 * j)) & 15u);
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g][i * 8 + j] = fmaf(w[g], c, acc[g][i * 8 + j]);
      }
    }
  }

  // ---- reduce over the token lanes of the wave ----
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int mk = LPT; mk < 64; mk <<= 1) {
      lsum[g] += __shfl_xor(lsum[g], mk, SAW_WAVE);
      zsum[g] += __shfl_xor(zsum[g], mk, SAW_WAVE);
#pragma unroll
      for (int j = 0; j < CPL; ++j) acc[g][j] += __shfl_xor(acc[g][j], mk, SAW_WAVE);
    }
  }
  if (lane < LPT) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int j = 0; j < CPL; ++j) red[wave][g][part * CPL + j] = acc[g][j] - zsum[g];
      if (part == 0) { red[wave][g][D] = m[g]; red[wave][g][D + 1] = lsum[g]; }
    }
  }
  __syncthreads();
  // ---- merge the four waves, write the split's partial ----
  for (int idx = tid; idx < G * (D + 2); idx += 256) {
    const int g = idx / (D + 2), c = idx % (D + 2);
    float mm = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) mm = fmaxf(mm, red[wv][g][D]);
    float v;
    if (c == 0) {
      v = mm;
    } else {
      const int src = (c == 1) ? D + 1 : c - 2;
      v = 0.f;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) v += fast_exp2(red[wv][g][D] - mm) * red[wv][g][src];
    }
    p.ws[(((int64_t)b * p.n_q_heads + kvh * G + g) * p.num_splits + split) * (D + 2) + c] = v;
  }
}

// ---------------------------------------------------------------------------------------
// 16-bit KV decode (comparison path).  Same decomposition; a token row of D 16-bit values is
// split over LPT lanes.
template <int D, int G, int LPT, int DT>
__global__ __launch_bounds__(256) void decode_kv16_kernel(DecodeParams p) {
  constexpr int TPW = 64 / LPT;
  constexpr int CPL = D / LPT;         // elements per lane
  constexpr int WPL = CPL / 2;         // dwords per lane
  // (the partition index is rotated by kv head and sequence, so that no XCD serves a fixed set of partitions)
  const int split = (blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int L = min(p.seq_lens[b] + p.len_bias, p.bound);
  const int t_begin = split * p.chunk_tokens;
  const int t_end = min(L, t_begin + p.chunk_tokens);
  if (t_begin >= t_end) return;

  __shared__ float qs[G * D];
  __shared__ float red[4][G][D + 4];
  for (int i = tid; i < G * D; i += 256)
    qs[i] = p.q_scale * load_elem(p.q, p.q_dtype, ((int64_t)b * p.n_q_heads + kvh * G) * D + i);
  __syncthreads();

  const int part = lane % LPT;
  float m[G], lsum[G], acc[G][CPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; lsum[g] = 0.f;
#pragma unroll
    for (int j = 0; j < CPL; ++j) acc[g][j] = 0.f;
  }
  const uint16_t* kpages = (const uint16_t*)p.k_codes;
  const uint16_t* vpages = (const uint16_t*)p.v_codes;
  const int64_t pt_row = (int64_t)b * p.max_pages;
  for (int t0 = t_begin + wave * TPW; t0 < t_end; t0 += 4 * TPW) {
    const int t = t0 + lane / LPT;
    const bool valid = t < t_end;
    const int tt = valid ? t : t_end - 1;
    int32_t page = p.page_table[pt_row + (tt >> 4)];
    page = (page < 0 || page >= p.num_pages) ? 0 : page;
    const int64_t vec = ((int64_t)page * p.n_kv_heads + kvh) * 16 + (tt & 15);
    const uint4* kp = (const uint4*)(kpages + vec * D + part * CPL);
    const uint4* vp = (const uint4*)(vpages + vec * D + part * CPL);
    float dot[G];
#pragma unroll
    for (int g = 0; g < G; ++g) dot[g] = 0.f;
#pragma unroll
    for (int i = 0; i < WPL / 4; ++i) {
      const uint4 w4 = kp[i];
      const uint32_t ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float lo, hi;
        widen2<DT>(ww[j], lo, hi);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          dot[g] = fmaf(qs[g * D + part * CPL + i * 8 + 2 * j], lo, dot[g]);
          dot[g] = fmaf(qs[g * D + part * CPL + i * 8 + 2 * j + 1], hi, dot[g]);
        }
      }
    }
    float w[G], mnew[G];
    bool grow = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int mk = 1; mk < LPT; mk <<= 1) dot[g] += __shfl_xor(dot[g], mk, SAW_WAVE);
      const float logit = valid ? dot[g] : -INFINITY;
      float mt = logit;
#pragma unroll
      for (int mk = LPT; mk < 64; mk <<= 1) mt = fmaxf(mt, __shfl_xor(mt, mk, SAW_WAVE));
      mnew[g] = fmaxf(m[g], mt);
      grow |= mnew[g] > m[g];
      w[g] = logit;
    }
    if (grow) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float a = fast_exp2(m[g] - mnew[g]);
        lsum[g] *= a;
#pragma unroll
        for (int j = 0; j < CPL; ++j) acc[g][j] *= a;
        m[g] = mnew[g];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      w[g] = valid ? fast_exp2(w[g] - m[g]) : 0.f;
      lsum[g] += w[g];
    }
#pragma unroll
    for (int i = 0; i < WPL / 4; ++i) {
      const uint4 w4 = vp[i];
      const uint32_t ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float lo, hi;
        widen2<DT>(ww[j], lo, hi);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          acc[g][i * 8 + 2 * j] = fmaf(w[g], lo, acc[g][i * 8 + 2 * j]);
          acc[g][i * 8 + 2 * j + 1] = fmaf(w[g], hi, acc[g][i * 8 + 2 * j + 1]);
        }
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int mk = LPT; mk < 64; mk <<= 1) {
      lsum[g] += __shfl_xor(lsum[g], mk, SAW_WAVE);
#pragma unroll
      for (int j = 0; j < CPL; ++j) acc[g][j] += __shfl_xor(acc[g][j], mk, SAW_WAVE);
    }
  }
  if (lane < LPT) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int j = 0; j < CPL; ++j) red[wave][g][part * CPL + j] = acc[g][j];
      if (part == 0) { red[wave][g][D] = m[g]; red[wave][g][D + 1] = lsum[g]; }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * (D + 2); idx += 256) {
    const int g = idx / (D + 2), c = idx % (D + 2);
    float mm = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) mm = fmaxf(mm, red[wv][g][D]);
    float v;
    if (c == 0) {
      v = mm;
    } else {
      const int src = (c == 1) ? D + 1 : c - 2;
      v = 0.f;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) v += fast_exp2(red[wv][g][D] - mm) * red[wv][g][src];
    }
    p.ws[(((int64_t)b * p.n_q_heads + kvh * G + g) * p.num_splits + split) * (D + 2) + c] = v;
  }
}

// ---------------------------------------------------------------------------------------
// Merge the splits of one (sequence, query head), rotate the output back, write it.
template <int D, int NT>
__global__ __launch_bounds__(NT) void decode_merge_kernel(DecodeParams p) {
  constexpr int NG = NT / D;                  // channel groups working on different splits
  constexpr int NW = NT / 64;
  const int j = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = tid % D, g = tid / D;
  const int L = min(p.seq_lens[b] + p.len_bias, p.bound);
  const int64_t o_idx = ((int64_t)b * p.n_q_heads + j) * D + c;
  // partitions that ran: those that start inside the cached tokens, and with a fused append the
  // first one in any case (it carries the step's own token)
  const int ns = max((max(L, 0) + p.chunk_tokens - 1) / p.chunk_tokens, p.append ? 1 : 0);
  if (ns == 0) {
    if (g == 0) store_elem(p.out, p.out_dtype, o_idx, 0.f);
    return;
  }
  __shared__ float wgt[1024];
  __shared__ __attribute__((aligned(16))) float red[NG][D];
  __shared__ float wred[2][NW];
  const float* base = p.ws + ((int64_t)b * p.n_q_heads + j) * p.num_splits * (D + 2);
  // Every split's (max, sum) pair is read once, by thread s (the launch gives the block at least as
  // many threads as there are splits): reference maximum, then weights and the denominator.
  float2 ml = make_float2(-INFINITY, 0.f);
  if (tid < ns) ml = *(const float2*)(base + (int64_t)tid * (D + 2));
  float mm = max_xor32(max_xor16(row_allmax(ml.x)));
  if (lane == 0) wred[0][wave] = mm;
  __syncthreads();
  mm = wred[0][0];
#pragma unroll
  for (int k = 1; k < NW; ++k) mm = fmaxf(mm, wred[0][k]);
  const float a_mine = (tid < ns) ? fast_exp2(ml.x - mm) : 0.f;
  if (tid < ns) wgt[tid] = a_mine;
  float den = add_xor32(add_xor16(row_allsum(a_mine * ml.y)));
  if (lane == 0) wred[1][wave] = den;
  __syncthreads();
  den = wred[1][0];
#pragma unroll
  for (int k = 1; k < NW; ++k) den += wred[1][k];
  // numerator: group g takes splits g, g + NG, ...
  float num = 0.f;
#pragma unroll 4
  for (int s = g; s < ns; s += NG) num = fmaf(wgt[s], base[s * (D + 2) + 2 + c], num);
  red[g][c] = num;
  __syncthreads();
  float o = 0.f;
  if (g == 0) {
#pragma unroll
    for (int k = 1; k < NG; ++k) num += red[k][c];
    o = num / den;
  }
  if (D == 128 && p.dense_v) {        // block-uniform: the learned rotation's transpose first (App. A.3)
    float* x = red[0];
    __syncthreads();                  // every read of red[][] above is done
    if (g == 0) x[c] = o;
    __syncthreads();
    if (wave == 0) wave_lds_matvec128<1>(x, p.dense + kDenseD * kDenseD, lane);
    __syncthreads();
    o = x[c];
  }
  if (p.rot_v) {                      // block-uniform
    float* x = red[0];
    __syncthreads();                  // every read of red[][] above is done
    if (g == 0) x[c] = o;
    __syncthreads();
    if (D == 128) {                   // one wavefront, three register passes, no block barriers in between
      if (wave == 0) wave_lds_fwht128<1>(x, p.had_block, lane);
      __syncthreads();
    } else {
      for (int st = 1; st < p.had_block; st <<= 1) {
        if (tid < D / 2) {            // each butterfly pair is owned by one thread
          const int i = ((tid & ~(st - 1)) << 1) | (tid & (st - 1));
          const float a = x[i], bb = x[i + st];
          x[i] = a + bb;
          x[i + st] = a - bb;
        }
        __syncthreads();
      }
    }
    o = x[c] * had_norm(p.had_block);
    if (p.has_signs) o = apply_sign(p.signs, c, o);             // (o~ H_blk) diag(sigma) = o~ R^T
  }
  if (g != 0) return;
  store_elem(p.out, p.out_dtype, o_idx, o);
}

// ---------------------------------------------------------------------------------------
template <int D, int G>
static void launch_int4(const DecodeParams& p, dim3 grid, hipStream_t st) {
  constexpr int LPT = (G >= 8) ? 8 : 4;
  decode_int4_kernel<D, G, LPT><<<grid, dim3(256), 0, st>>>(p);
}
template <int D, int G, int DT>
static void launch_kv16(const DecodeParams& p, dim3 grid, hipStream_t st) {
  constexpr int LPT = (G >= 8 || D == 128) ? 8 : 4;
  constexpr int LPT2 = (G >= 8 && D == 128) ? 16 : LPT;
  decode_kv16_kernel<D, G, LPT2, DT><<<grid, dim3(256), 0, st>>>(p);
}

int launch_decode(const DecodeParams& p, int B, int D, int G, bool kv16, int kv_dtype, hipStream_t st) {
  dim3 grid(p.num_splits, p.n_kv_heads, B);
  const bool head_pairs = !kv16 && decode_head_pairs(D, p.n_kv_heads, G);
  if (!kv16 && (D == 128 || head_pairs)) {
    const dim3 mgrid(grid.x, head_pairs ? grid.y / 2 : grid.y, grid.z);
    if (launch_decode_int4_mfma(p, G, B, p.waves_per_item, head_pairs, mgrid, st) != SAW_OK) return SAW_EINVAL;
    if (hipGetLastError() != hipSuccess) return SAW_ELAUNCH;
    if (p.num_splits == 1) return SAW_OK;       // the kernel wrote the output itself
  } else if (kv16 && D == 128 && launch_decode_kv16_mfma(p, G, kv_dtype, grid, st)) {
    if (hipGetLastError() != hipSuccess) return SAW_ELAUNCH;
    if (p.num_splits == 1) return SAW_OK;       // the kernel wrote the output itself
  } else {
#define SAW_DISPATCH_G(DD)                                                          \
  switch (G) {                                                                      \
    case 1: if (kv16) { if (kv_dtype == SAW_BF16) launch_kv16<DD, 1, SAW_BF16>(p, grid, st); else launch_kv16<DD, 1, SAW_F16>(p, grid, st); } else launch_int4<DD, 1>(p, grid, st); break; \
    case 2: if (kv16) { if (kv_dtype == SAW_BF16) launch_kv16<DD, 2, SAW_BF16>(p, grid, st); else launch_kv16<DD, 2, SAW_F16>(p, grid, st); } else launch_int4<DD, 2>(p, grid, st); break; \
    case 4: if (kv16) { if (kv_dtype == SAW_BF16) launch_kv16<DD, 4, SAW_BF16>(p, grid, st); else launch_kv16<DD, 4, SAW_F16>(p, grid, st); } else launch_int4<DD, 4>(p, grid, st); break; \
    case 8: if (kv16) { if (kv_dtype == SAW_BF16) launch_kv16<DD, 8, SAW_BF16>(p, grid, st); else launch_kv16<DD, 8, SAW_F16>(p, grid, st); } else launch_int4<DD, 8>(p, grid, st); break; \
    default: return SAW_EINVAL;                                                     \
  }
  if (D == 128) { SAW_DISPATCH_G(128) } else { SAW_DISPATCH_G(64) }
#undef SAW_DISPATCH_G
  }
  if (hipGetLastError() != hipSuccess) return SAW_ELAUNCH;
  dim3 mgrid(p.n_q_heads, B);
  if (p.num_splits > 16) {
    if (D == 128) decode_merge_kernel<128, 1024><<<mgrid, dim3(1024), 0, st>>>(p);
    else decode_merge_kernel<64, 1024><<<mgrid, dim3(1024), 0, st>>>(p);
  } else {
    if (D == 128) decode_merge_kernel<128, 256><<<mgrid, dim3(256), 0, st>>>(p);
    else decode_merge_kernel<64, 256><<<mgrid, dim3(256), 0, st>>>(p);
  }
  return hipGetLastError() == hipSuccess ? SAW_OK : SAW_ELAUNCH;
}

int run_decode(const saw_cache_t* c, bool kv16, const void* k_pages, const void* v_pages, int kv_dtype,
               const void* q, int q_dtype, int B, int Hq, const int32_t* pt, int max_pages,
               const int32_t* seq_lens, float sm_scale, void* out, int out_dtype, void* ws,
               const SplitPlan& plan, const void* k_new, const void* v_new, int kv_new_dtype, int len_bias,
               const int32_t* order, hipStream_t st) {
  DecodeParams p;
  p.order = kv16 ? nullptr : order;
  p.k_codes = (const uint8_t*)k_pages;
  p.v_codes = (const uint8_t*)v_pages;
  p.k_meta = c->k_meta;
  p.v_meta = c->v_meta;
  p.q = q;
  p.page_table = pt;
  p.seq_lens = seq_lens;
  p.ws = (float*)ws;
  p.out = out;
  const float scale = (sm_scale > 0.f) ? sm_scale : 1.0f / sqrtf((float)c->head_dim);
  p.q_scale = scale * 1.4426950408889634f;
  p.q_dtype = q_dtype;
  p.out_dtype = out_dtype;
  p.n_q_heads = Hq;
  p.n_kv_heads = c->n_kv_heads;
  p.max_pages = max_pages;
  p.num_pages = c->num_pages;
  p.had_block = c->had_block;
  p.rot_k = !kv16 && c->had_block > 1 && (c->rotate_mask & SAW_ROT_K);
  p.rot_v = !kv16 && c->had_block > 1 && (c->rotate_mask & SAW_ROT_V);
  for (int i = 0; i < 4; ++i) p.signs.w[i] = kv16 ? 0u : c->sign_bits[i];
  p.has_signs = (p.signs.w[0] | p.signs.w[1] | p.signs.w[2] | p.signs.w[3]) != 0;
  p.dense = kv16 ? nullptr : (const float*)c->dense_rot;
  p.dense_k = p.dense && (c->rotate_mask & SAW_ROT_K);
  p.dense_v = p.dense && (c->rotate_mask & SAW_ROT_V);
  p.num_splits = plan.num_splits;
  p.chunk_tokens = plan.chunk_tokens;
  p.bound = plan.bound;
  p.waves_per_item = plan.waves_per_item;
  // Pair mode: one partition per sequence, enough (sequence, kv head) items that every compute
  // unit gets several, and at most 16 lengths per lane for the in-kernel ranking.
  p.k_new = k_new;
  p.v_new = v_new;
  p.kv_new_dtype = kv_new_dtype;
  p.append = k_new != nullptr;
  p.len_bias = len_bias;
  p.batch = B;
  // How the matrix-core INT4 kernel hands out work when one partition covers each sequence and the
  // batch provides more (sequence, kv head) items than compute units (and at most 16 lengths per
  // lane for the in-kernel ranking).  A compute unit holds 8 wavefronts of this kernel, 2048 on
  // the chip:
  //   * up to 2048 items everything is resident at once and nothing rebalances later, so the
  //     work is evened out up front: pair mode, blocks over (long, short) pairs of sequences, of
  //     four wavefronts while that still fits the 2048 slots and of two beyond.  Four-wavefront
  //     blocks pay off on ragged batches from 576 items on (256 sequences x 4 heads: 82 -> 70 us,
  //     90 x 8: 70 -> 61 us, 72 x 8: 63 -> 57 us against 2 or 4 wavefronts interleaving each
  //     item's batches; equal lengths lose 2-8 us to the ranking and the records; at 528 items
  //     four interleaving wavefronts per item are ahead: 51 against 64 us).  Between 1025 and 1151
  //     items two interleaving wavefronts per item still fit the slots well enough (136 x 8: 79
  //     against 94 us in pair mode); from 1152 on they spill into a second round.  Up to 1536
  //     items blocks of four wavefronts over THREE sequences then fill the chip where blocks of two
  //     over pairs leave a quarter to a half of the slots empty (144 x 8: 93 -> 83 us, 160 x 8:
  //     93 -> 85 us, 176 x 8: 94 -> 89 us, level at 192 x 8), beyond that blocks of two;
  //   * beyond that blocks queue for slots in index order, which is list scheduling: one
  //     wavefront per item, sequences taken longest first, so the launch ends on the shortest.
  //     (Measured at 288..512 sequences x 8 heads: 173-270 us against 224-332 us in pair mode,
  //     whose equal blocks make the last round as long as the others; 2 or 4 wavefronts per item
  //     were never better.)
  p.pair = 0;
  p.pair_seqs = 2;
  p.sorted = 0;
  const int G = Hq / c->n_kv_heads;
  const int items = decode_items_per_seq(c->head_dim, c->n_kv_heads);   // head_dim 64: pairs of kv heads
  if (!kv16 && (c->head_dim == 128 || decode_head_pairs(c->head_dim, c->n_kv_heads, G)) &&
      plan.num_splits == 1 && B <= 1024) {
    const int64_t blocks = (int64_t)((B + 1) / 2) * items;
    const int64_t blocks3 = (int64_t)((B + 2) / 3) * items;
    if ((int64_t)B * items >= 576 && blocks <= 512) p.pair = 4;
    else if ((int64_t)B * items >= 1152 && blocks3 <= 512 && !(c->head_dim == 64 && G == 4)) {
      // four wavefronts over three sequences (not for head pairs with eight query rows: two such
      // blocks with their two spare records do not fit a compute unit's LDS)
      p.pair = 4;
      p.pair_seqs = 3;
    }
    else if ((int64_t)B * items >= 1152 && blocks <= 1024) p.pair = 2;   // (whatever the plan's wavefronts per item)
    else if (plan.waves_per_item == 1 && (int64_t)B * items > 256) {
      if (blocks <= 1024) p.pair = 2;
      else if ((int64_t)B * items <= 2304 && blocks3 <= 1024 && !(c->head_dim == 64 && G == 4)) {
        // just above 2048 items: blocks of two wavefronts over THREE sequences keep everything resident
        // (equal lengths, where the longest-first order has nothing to reorder and the last 32 items ran
        // alone: 260 x 8 sequences of 2304 tokens 165 -> 135 us; ragged batches 137-148 us either way up
        // to 288 x 8; from 320 x 8 on the longest-first order is ahead: 155 against 166 us)
        p.pair = 2;
        p.pair_seqs = 3;
      }
      else p.sorted = 1;
    }
  }
  // the 16-bit matrix-core kernel has the two-wavefront pair mode as well (same conditions), so that
  // the comparison on a ragged batch is between formats and not between schedules
  if (kv16 && c->head_dim == 128 && G <= 4 && plan.num_splits == 1 && B <= 1024 &&
      (int64_t)B * c->n_kv_heads > 256 && (int64_t)((B + 1) / 2) * c->n_kv_heads <= 1024)
    p.pair = 2;
  return launch_decode(p, B, c->head_dim, G, kv16, kv_dtype, st);
}

}  // namespace saw
