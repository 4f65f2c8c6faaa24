// In-kernel longest-first ranking of a batch's sequences, shared by the decode kernels.
#pragma once

#include "saw_decode.h"
#include "saw_wave_util.h"

namespace saw {

// Longest-first order of the batch's sequences, derived by every block from the same seq_lens:
// rank by (64 length classes, sequence index).  `build` reads the lengths once (all loads issued
// together: one memory latency), leaves them clamped in LDS and their classes in registers, makes
// the class histogram (LDS atomics) and its prefix sums across lanes (lane c owns class c, class
// 0 = longest); `seq_of_rank` finds the sequence at a rank with two ballots per 64 sequences.
// The classes are scaled to the longest sequence the batch actually holds (a wavefront-wide
// maximum of the clamped lengths), not to the caller's bound, so that a loose bound - the usual
// serving call, which avoids a host read of the lengths - costs no balance; and class 63 holds the
// sequences without cached tokens and nothing else, so an empty sequence never ranks ahead of a
// non-empty one (the pair-mode share logic relies on that: see rank_class()).
// LDS scratch: 64 + B ints, B <= kMaxRanked.
constexpr int kMaxRanked = 1024;
struct LenClasses {
  int cnt, start, incl;      // this lane's class: members, ranks [start, incl)
  int V;                     // ceil(B / 64)
  const int* lens;           // LDS: the clamped lengths
  int cls[kMaxRanked / 64];  // class of sequence 64 v + lane (-1 past the batch)
};
template <int CTRL, int ROWMASK>
__device__ __forceinline__ int dpp_i0(int v) {               // lanes without a source (or outside ROWMASK) read 0
  return __builtin_amdgcn_update_dpp(0, v, CTRL, ROWMASK, 0xf, false);
}
__device__ __forceinline__ LenClasses build_len_classes(const DecodeParams& p, int B, int lane, int* scratch) {
  LenClasses lc;
  lc.V = (B + 63) >> 6;
  int* const hist = scratch;
  int* const lens = scratch + 64;
  lc.lens = lens;
  int mine[kMaxRanked / 64];
  // (the `v < lc.V` tests are wavefront-uniform: the groups of 64 past the batch cost a branch each)
#pragma unroll
  for (int v = 0; v < kMaxRanked / 64; ++v) {
    const int idx = 64 * v + lane;
    mine[v] = 0;
    if (v < lc.V) mine[v] = (idx < B) ? p.seq_lens[idx] : 0;
  }
  hist[lane] = 0;
  // clamp, and the batch's longest sequence in 64-token units (a max over the lanes)
  int nbmax = 0;
#pragma unroll
  for (int v = 0; v < kMaxRanked / 64; ++v) {
    if (v < lc.V) {
      mine[v] = (64 * v + lane < B) ? max(min(mine[v] + p.len_bias, p.bound), 0) : 0;
      nbmax = max(nbmax, (mine[v] + 63) >> 6);
    }
  }
  nbmax = max(nbmax, dpp_i0<0x121, 0xf>(nbmax));         // row_ror:1, 2, 4, 8: every lane of a row has the row's max
  nbmax = max(nbmax, dpp_i0<0x122, 0xf>(nbmax));
  nbmax = max(nbmax, dpp_i0<0x124, 0xf>(nbmax));
  nbmax = max(nbmax, dpp_i0<0x128, 0xf>(nbmax));
  nbmax = max(max(__builtin_amdgcn_readlane(nbmax, 0), __builtin_amdgcn_readlane(nbmax, 16)),
              max(__builtin_amdgcn_readlane(nbmax, 32), __builtin_amdgcn_readlane(nbmax, 48)));
  const float kscale = rank_scale(nbmax);
  wave_sync();
#pragma unroll
  for (int v = 0; v < kMaxRanked / 64; ++v) {
    const int idx = 64 * v + lane;
    lc.cls[v] = -1;
    if (v < lc.V && idx < B) {
      lens[idx] = mine[v];
      lc.cls[v] = rank_class(mine[v], kscale);
      atomicAdd(&hist[lc.cls[v]], 1);
    }
  }
  wave_sync();
  lc.cnt = hist[lane];
  // inclusive prefix sum over the 64 lanes in registers: four shifted adds inside each row of 16
  // lanes, then each row's last lane is broadcast into the rows after it
  int incl = lc.cnt;
  incl += dpp_i0<0x111, 0xf>(incl);      // row_shr:1
  incl += dpp_i0<0x112, 0xf>(incl);      // row_shr:2
  incl += dpp_i0<0x114, 0xf>(incl);      // row_shr:4
  incl += dpp_i0<0x118, 0xf>(incl);      // row_shr:8
  incl += dpp_i0<0x142, 0xa>(incl);      // row_bcast:15 into rows 1 and 3
  incl += dpp_i0<0x143, 0xc>(incl);      // row_bcast:31 into rows 2 and 3
  lc.incl = incl;
  lc.start = incl - lc.cnt;
  return lc;
}
__device__ __forceinline__ int seq_of_rank(int lane, const LenClasses& lc, int srank) {
  const unsigned long long hit = __ballot(srank >= lc.start && srank < lc.incl);   // exactly one class
  const int cls = __ffsll((long long)hit) - 1;
  int o = srank - __builtin_amdgcn_readlane(lc.start, cls);                        // index inside the class
  int found = 0;
  bool done = false;
#pragma unroll
  for (int v = 0; v < kMaxRanked / 64; ++v) {
    if (v < lc.V && !done) {                                                       // wavefront-uniform
      const bool in = lc.cls[v] == cls;
      const unsigned long long mask = __ballot(in);
      const int c = __popcll(mask);
      if (o < c) {
        const int myrank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
        const unsigned long long me = __ballot(in && myrank == o);
        found = 64 * v + __ffsll((long long)me) - 1;
        done = true;
      }
      o -= c;
    }
  }
  return __builtin_amdgcn_readfirstlane(found);
}

}  // namespace saw
