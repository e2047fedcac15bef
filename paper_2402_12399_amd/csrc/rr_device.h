// Device helpers shared by the routing kernels.
#pragma once

#include "rr_internal.h"

namespace rr {

constexpr int kMaxRank = kMaxK + 1;

// Eq. 1 argtopk over one row of scores held in LDS: the n best experts by descending score,
// ties -> lower expert index (a later expert must be strictly greater to displace an earlier one).
__device__ inline void top_n_of_row(const float *row, int E, int n, float (&bs)[kMaxRank], int (&be)[kMaxRank]) {
#pragma unroll
  for (int q = 0; q < kMaxRank; ++q) { bs[q] = -INFINITY; be[q] = -1; }
  for (int e = 0; e < E; ++e) {
    float cv = row[e];
    int ce = e;
    bool ins = false;
#pragma unroll
    for (int q = 0; q < kMaxRank; ++q) {
      bool s = (q < n) && (ins || cv > bs[q]);
      if (s) {
        float tv = bs[q]; int te = be[q];
        bs[q] = cv; be[q] = ce;
        cv = tv; ce = te;
        ins = true;
      }
    }
  }
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
