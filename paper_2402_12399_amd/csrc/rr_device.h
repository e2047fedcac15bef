// Device helpers shared by the routing kernels.
#pragma once

#include "rr_internal.h"

namespace rr {

constexpr int kMaxRank = kMaxK + 1;

// Ranking key of a (score, expert) pair: the order-preserving image of the score in the high word,
// the complement of the expert index in the low one.  A greater key is a better rank - a higher
// score, or an equal score at a lower expert index (Eq. 1 argtopk, ties -> lower expert index) - so
// the order is ONE unsigned comparison, and the keys of different experts never tie.  0 lies below
// every real key (the image of a score is never 0) and decodes to expert -1.
__device__ inline unsigned long long rank_key(float v, int e) {
  return ((unsigned long long)score_key(v) << 32) | (u32)~e;
}
__device__ inline int rank_key_expert(unsigned long long key) { return (int)~(u32)key; }
__device__ inline u32 rank_key_score(unsigned long long key) { return (u32)(key >> 32); }

// b[0] > b[1] > ... > b[N-1] are the N greatest keys seen so far: one compare-exchange per position.
template <int N>
__device__ inline void insert_key(unsigned long long (&b)[N], unsigned long long a) {
#pragma unroll
  for (int q = 0; q < N; ++q) {
    const bool c = a > b[q];
    const unsigned long long hi = c ? a : b[q];
    a = c ? b[q] : a;
    b[q] = hi;
  }
}

// Eq. 1 argtopk over experts [e0, e1) of one row of scores held in LDS: the N best keys, best first
// (positions past the number of experts stay 0).
template <int N>
__device__ inline void top_keys_of_range(const float *row, int e0, int e1, unsigned long long (&b)[N]) {
#pragma unroll
  for (int q = 0; q < N; ++q) b[q] = 0ull;
  for (int e = e0; e < e1; ++e) insert_key(b, rank_key(row[e], e));
}

// Sec. 4.1: best expert among those of one group, ties -> lower expert index.
__device__ inline void best_in_group(const float *row, int e0, int e1, float &best, int &arg) {
  best = row[e0];
  arg = e0;
  for (int e = e0 + 1; e < e1; ++e) {
    float v = row[e];
    if (v > best) { best = v; arg = e; }
  }
}

__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }

// Workgroup -> token block for kernels whose neighbouring token blocks write neighbouring words of
// the same per-expert arrays.  Workgroups are dealt to the 8 XCDs round-robin and each XCD has its
// own L2: with block = workgroup, one cache line would be completed piecewise from 8 L2s.  Here XCD
// x walks its own contiguous eighth of the blocks, so the pieces of a line meet in one L2.
__device__ inline int xcd_block(int g, int NB) {
  const int per = NB >> 3, main = per << 3;
  return g < main ? (g & 7) * per + (g >> 3) : g;
}


}  // namespace rr
