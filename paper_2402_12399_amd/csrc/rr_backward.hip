// Backward pass of the combine weights: gradient of a loss with respect to the router scores
// (App. A, Eq. 5 and Eq. 6).
//
// Eq. 2 / Eq. 3 are linear in the weights, o_i = sum_p c_ip y_p over the token's processed
// assignments p (kept top-k ranks, a placed fill-in, the Intra-GPU expert), y_p the dispatched row
// of that assignment in the expert outputs, so dL/dc_ip = <dL/do_i, y_p>.  With
// D_i = sum_p c_ip dL/dc_ip, g_il the softmax over all experts and m_il the weight mass of expert l
// (the sum of c_ip over the assignments that go to expert l),
//   straight-through (Eq. 6, normaliser of the weights held constant):
//       dL/da_il = sum_{p: e_p = l} c_ip dL/dc_ip - g_il D_i
//   plain derivative of the normalised weights:
//       dL/da_il = sum_{p: e_p = l} c_ip dL/dc_ip - m_il D_i
// (both follow from c_ip = n_p g_{i,e_p} / S_i: the drop count n_p and S_i cancel out of the closed
// forms, so the weights the forward pass stored are all that is needed).
//
// One wave per token: the lanes stride over the 16-byte vectors of the rows (dL/do_i is read once,
// each y_p once), reduce the dot products across the wave, then lane l owns expert l.
#include "rr_device.h"

namespace rr {

namespace {

constexpr int RB_THREADS = 256;
constexpr int RB_TOKENS = RB_THREADS / kWave;
constexpr int RB_NP = kMaxRank + 1;  // ranks 0..k (the last one is the fill-in), then the Intra-GPU expert

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

__device__ inline float dot_vec(const uint4 a, const uint4 b, bool bf16) {
  const u32 pa[4] = {a.x, a.y, a.z, a.w}, pb[4] = {b.x, b.y, b.z, b.w};
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (bf16) {
      s = fmaf(__builtin_bit_cast(float, pa[j] << 16), __builtin_bit_cast(float, pb[j] << 16), s);
      s = fmaf(__builtin_bit_cast(float, pa[j] & 0xffff0000u), __builtin_bit_cast(float, pb[j] & 0xffff0000u), s);
    } else {
      s = fmaf(__builtin_bit_cast(float, pa[j]), __builtin_bit_cast(float, pb[j]), s);
    }
  }
  return s;
}

template <bool BF16>
__global__ __launch_bounds__(RB_THREADS) void router_backward_kernel(
    const uint4 *__restrict__ y, const uint4 *__restrict__ dout, int vec_per_row, int T, int E, int k, int NR,
    const int32_t *__restrict__ rank_expert, const int32_t *__restrict__ slot, const int32_t *__restrict__ ir_expert,
    const int32_t *__restrict__ ir_row, const int32_t *__restrict__ fill_total, const int32_t *__restrict__ row_base,
    const int32_t *__restrict__ grp_off, int Cq, int Gq, const float *__restrict__ combine_w,
    const float *__restrict__ logits, int straight_through, float *__restrict__ dcombine_w,
    float *__restrict__ dlogits) {
  const int i = blockIdx.x * RB_TOKENS + (threadIdx.x >> 6);  // wave-uniform
  if (i >= T) return;
  const int lane = lane_id();

  // lane p < NR: rank p; lane kMaxRank: the Intra-GPU expert
  int my_row = -1, my_e = -1;
  float my_c = 0.0f;
  if (lane < NR) {
    const int s = slot[(size_t)i * (k + 1) + lane];
    if (s >= 0) {
      const int g = s / Cq;
      my_e = rank_expert[(size_t)i * (k + 1) + lane];
      my_row = row_base[my_e] + grp_off[my_e * Gq + g] + (s - g * Cq);
      my_c = combine_w[(size_t)i * (k + 2) + lane];
    }
  } else if (lane == kMaxRank) {
    const int h = ir_expert[i];
    if (h >= 0) {
      my_e = h;
      my_row = row_base[h] + fill_total[h] + ir_row[i];
      my_c = combine_w[(size_t)i * (k + 2) + k + 1];
    }
  }
  int row[RB_NP], ex[RB_NP];
  float c[RB_NP], dc[RB_NP];
#pragma unroll
  for (int p = 0; p < RB_NP; ++p) {
    row[p] = __shfl(my_row, p, kWave);
    ex[p] = __shfl(my_e, p, kWave);
    c[p] = __shfl(my_c, p, kWave);
    dc[p] = 0.0f;
  }

  const uint4 *go = dout + (size_t)i * vec_per_row;
  for (int v = lane; v < vec_per_row; v += kWave) {
    const uint4 gv = go[v];
#pragma unroll
    for (int p = 0; p < RB_NP; ++p)
      if (row[p] >= 0) dc[p] += dot_vec(gv, y[(size_t)row[p] * vec_per_row + v], BF16);
  }
  float D = 0.0f;
#pragma unroll
  for (int p = 0; p < RB_NP; ++p) {
    dc[p] = row[p] >= 0 ? wave_sum(dc[p]) : 0.0f;  // row[p] is wave-uniform
    D = fmaf(c[p], dc[p], D);
  }
  if (dcombine_w && lane < k + 2) {
    // column r < NR: rank r; column k + 1: Intra-GPU; a column without an assignment gets 0
    float val = 0.0f;
#pragma unroll
    for (int p = 0; p < RB_NP; ++p) {
      const int col = p == kMaxRank ? k + 1 : p;
      if (lane == col && (p == kMaxRank || p < NR)) val = dc[p];
    }
    dcombine_w[(size_t)i * (k + 2) + lane] = val;
  }

  // lane l owns expert l (E <= 64)
  const float a = lane < E ? logits[(size_t)i * E + lane] : -INFINITY;
  const float amax = wave_max(a);
  const float z = lane < E ? expf(a - amax) : 0.0f;
  const float Z = wave_sum(z);
  float direct = 0.0f, mass = 0.0f;
#pragma unroll
  for (int p = 0; p < RB_NP; ++p)
    if (row[p] >= 0 && ex[p] == lane) {
      direct = fmaf(c[p], dc[p], direct);
      mass += c[p];
    }
  const float pull = straight_through ? z / Z : mass;
  if (lane < E) dlogits[(size_t)i * E + lane] = direct - pull * D;
}

}  // namespace

hipError_t launch_router_backward(const Dims &D, const void *dout, const float *logits, const rr_tables &tb,
                                  const Work &W, bool straight_through, float *dcombine_w, float *dlogits,
                                  hipStream_t s) {
  const int es = D.dtype == RR_BF16 ? 2 : 4;
  const int vec_per_row = D.d * es / 16;
  const int grid = (D.T + RB_TOKENS - 1) / RB_TOKENS;
  prof_begin(K_ROUTER_BWD, s);
  if (D.dtype == RR_BF16)
    router_backward_kernel<true><<<grid, RB_THREADS, 0, s>>>(
        static_cast<const uint4 *>(W.y), static_cast<const uint4 *>(dout), vec_per_row, D.T, D.E, D.k, D.NR,
        tb.rank_expert, tb.slot, tb.ir_expert, tb.ir_row, tb.fill_total, W.row_base, W.grp_off, D.Cq, D.Gq,
        tb.combine_w, logits, straight_through ? 1 : 0, dcombine_w, dlogits);
  else
    router_backward_kernel<false><<<grid, RB_THREADS, 0, s>>>(
        static_cast<const uint4 *>(W.y), static_cast<const uint4 *>(dout), vec_per_row, D.T, D.E, D.k, D.NR,
        tb.rank_expert, tb.slot, tb.ir_expert, tb.ir_row, tb.fill_total, W.row_base, W.grp_off, D.Cq, D.Gq,
        tb.combine_w, logits, straight_through ? 1 : 0, dcombine_w, dlogits);
  prof_end(K_ROUTER_BWD, s);
  return hipGetLastError();
}

}  // namespace rr
