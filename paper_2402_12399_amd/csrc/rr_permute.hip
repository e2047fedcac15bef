// Dispatch gather and weighted combine: on one GPU the expert-parallel all-to-all of Sec. 3 is a
// row permutation in device memory.
//
// Dispatched-row layout (built with the routing tables): expert e owns rows [row_base[e], row_base[e+1]): its
// occupied capacity slots in slot order, then its Intra-GPU list.  Padding slots get no row:
// FFN(0) = 0 contributes nothing (Sec. 3, zero padding).  Slot s of capacity block g = s / Cq is
// row row_base[e] + grp_off[e, g] + s % Cq, where grp_off counts the occupied slots of the expert's
// earlier blocks (one block and grp_off = 0 unless capacity is per group); row
// row_base[e] + fill_total[e] + q holds the q-th token of the expert's Intra-GPU list.
#include "rr_device.h"

namespace rr {

namespace {

constexpr int PG_THREADS = 256;
constexpr int PG_ROWS = PG_THREADS / kWave;  // one wave per row

// x_disp[row] = x[token(row)]; rows are 16-byte vectors of `vec_per_row` elements
__global__ __launch_bounds__(PG_THREADS) void gather_kernel(const uint4 *__restrict__ x, uint4 *__restrict__ x_disp,
                                                            int vec_per_row, int E, int C,
                                                            const int32_t *__restrict__ slot_token,
                                                            const int32_t *__restrict__ fill_total,
                                                            const int32_t *__restrict__ ir_offset,
                                                            const int32_t *__restrict__ ir_token,
                                                            const int32_t *__restrict__ ir_expert,
                                                            const int32_t *__restrict__ row_base) {
  const int q = blockIdx.x * PG_ROWS + (threadIdx.x >> 6);
  const int lane = lane_id();
  int tok, dst;
  if (q < E * C) {
    int e = q / C, s = q - e * C;
    if (s >= fill_total[e]) return;
    tok = slot_token[q];
    dst = row_base[e] + s;
  } else {
    int p = q - E * C;
    if (p >= ir_offset[E]) return;
    tok = ir_token[p];
    int e = ir_expert[tok];
    dst = row_base[e] + fill_total[e] + (p - ir_offset[e]);
  }
  const uint4 *src = x + (size_t)tok * vec_per_row;
  uint4 *out = x_disp + (size_t)dst * vec_per_row;
  for (int v = lane; v < vec_per_row; v += kWave) out[v] = src[v];
}

// Per-group quotas: x_disp[row] = x[row_token[row]] for the rows that exist (row_base[E] of them).
__global__ __launch_bounds__(PG_THREADS) void gather_rows_kernel(const uint4 *__restrict__ x, uint4 *__restrict__ x_disp,
                                                                 int vec_per_row, int E,
                                                                 const int32_t *__restrict__ row_token,
                                                                 const int32_t *__restrict__ row_base) {
  const int q = blockIdx.x * PG_ROWS + (threadIdx.x >> 6);
  if (q >= row_base[E]) return;
  const int lane = lane_id();
  const uint4 *src = x + (size_t)row_token[q] * vec_per_row;
  uint4 *out = x_disp + (size_t)q * vec_per_row;
  for (int v = lane; v < vec_per_row; v += kWave) out[v] = src[v];
}

__device__ inline void fma_row(float (&acc)[8], float w, const uint4 v, bool bf16) {
  if (bf16) {
    u32 p[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[2 * j] = fmaf(w, __builtin_bit_cast(float, p[j] << 16), acc[2 * j]);
      acc[2 * j + 1] = fmaf(w, __builtin_bit_cast(float, p[j] & 0xffff0000u), acc[2 * j + 1]);
    }
  } else {
    acc[0] = fmaf(w, __builtin_bit_cast(float, v.x), acc[0]);
    acc[1] = fmaf(w, __builtin_bit_cast(float, v.y), acc[1]);
    acc[2] = fmaf(w, __builtin_bit_cast(float, v.z), acc[2]);
    acc[3] = fmaf(w, __builtin_bit_cast(float, v.w), acc[3]);
  }
}

__device__ inline u32 f32_to_bf16_rne(float f) {
  u32 u = __builtin_bit_cast(u32, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// Eq. 2 / Eq. 3: out[i] = sum_r cw[i,r] * y[row(i,r)] + cw[i,k+1] * y[ir row(i)], fp32 accumulate,
// rounded once.  Token-major (a gather per token), so the result does not depend on any order of
// atomics.  A token without any processed assignment gets a row of zeros.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4 *__restrict__ y, uint4 *__restrict__ out,
                                                      int vec_per_row, int k, int NR,
                                                      const int32_t *__restrict__ rank_expert,
                                                      const int32_t *__restrict__ slot,
                                                      const int32_t *__restrict__ ir_expert,
                                                      const int32_t *__restrict__ ir_row,
                                                      const int32_t *__restrict__ fill_total,
                                                      const int32_t *__restrict__ row_base,
                                                      const int32_t *__restrict__ grp_off, int Cq, int Gq,
                                                      const float *__restrict__ combine_w, int skip_single) {
  const int i = blockIdx.x;
  __shared__ int s_row[kMaxRank + 1];
  __shared__ float s_w[kMaxRank + 1];
  if (threadIdx.x <= kMaxRank) {
    int r = threadIdx.x, row = -1;
    float w = 0.0f;
    if (r < NR) {
      int s = slot[(size_t)i * (k + 1) + r];
      if (s >= 0) {
        const int e = rank_expert[(size_t)i * (k + 1) + r], g = s / Cq;
        row = row_base[e] + grp_off[e * Gq + g] + (s - g * Cq);
        w = combine_w[(size_t)i * (k + 2) + r];
      }
    } else if (r == kMaxRank) {
      int h = ir_expert[i];
      if (h >= 0) {
        row = row_base[h] + fill_total[h] + ir_row[i];
        w = combine_w[(size_t)i * (k + 2) + k + 1];
      }
    }
    s_row[r] = row;
    s_w[r] = w;
  }
  __syncthreads();
  if (skip_single) {  // a token with exactly one row: the down projection has stored its output row
    int nrows = 0;
#pragma unroll
    for (int r = 0; r <= kMaxRank; ++r) nrows += s_row[r] >= 0;
    if (nrows == 1) return;
  }
  for (int v = threadIdx.x; v < vec_per_row; v += 256) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r <= kMaxRank; ++r) {
      int row = s_row[r];
      if (row >= 0) fma_row(acc, s_w[r], y[(size_t)row * vec_per_row + v], BF16);
    }
    uint4 o;
    if (BF16) {
      o.x = f32_to_bf16_rne(acc[0]) | (f32_to_bf16_rne(acc[1]) << 16);
      o.y = f32_to_bf16_rne(acc[2]) | (f32_to_bf16_rne(acc[3]) << 16);
      o.z = f32_to_bf16_rne(acc[4]) | (f32_to_bf16_rne(acc[5]) << 16);
      o.w = f32_to_bf16_rne(acc[6]) | (f32_to_bf16_rne(acc[7]) << 16);
    } else {
      o.x = __builtin_bit_cast(u32, acc[0]);
      o.y = __builtin_bit_cast(u32, acc[1]);
      o.z = __builtin_bit_cast(u32, acc[2]);
      o.w = __builtin_bit_cast(u32, acc[3]);
    }
    out[(size_t)i * vec_per_row + v] = o;
  }
}

// The same sum with one wave per token and no LDS: lane p fetches the row and weight of assignment p,
// the wave broadcasts them, every lane then strides over the 16-byte vectors of the rows.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_wave_kernel(const uint4 *__restrict__ y, uint4 *__restrict__ out,
                                                           int vec_per_row, int T, int k, int NR,
                                                           const int32_t *__restrict__ rank_expert,
                                                           const int32_t *__restrict__ slot,
                                                           const int32_t *__restrict__ ir_expert,
                                                           const int32_t *__restrict__ ir_row,
                                                           const int32_t *__restrict__ fill_total,
                                                           const int32_t *__restrict__ row_base,
                                                           const int32_t *__restrict__ grp_off, int Cq, int Gq,
                                                           const float *__restrict__ combine_w, int skip_single) {
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= T) return;
  const int lane = lane_id();
  int my_row = -1;
  float my_w = 0.0f;
  if (lane < NR) {
    const int s = slot[(size_t)i * (k + 1) + lane];
    if (s >= 0) {
      const int e = rank_expert[(size_t)i * (k + 1) + lane], g = s / Cq;
      my_row = row_base[e] + grp_off[e * Gq + g] + (s - g * Cq);
      my_w = combine_w[(size_t)i * (k + 2) + lane];
    }
  } else if (lane == kMaxRank) {
    const int h = ir_expert[i];
    if (h >= 0) {
      my_row = row_base[h] + fill_total[h] + ir_row[i];
      my_w = combine_w[(size_t)i * (k + 2) + k + 1];
    }
  }
  // a token with exactly one row: the down projection has stored its output row
  if (skip_single && __popcll(__ballot(my_row >= 0)) == 1) return;
  int row[kMaxRank + 1];
  float wgt[kMaxRank + 1];
#pragma unroll
  for (int p = 0; p <= kMaxRank; ++p) {
    row[p] = __shfl(my_row, p, kWave);
    wgt[p] = __shfl(my_w, p, kWave);
  }
  for (int v = lane; v < vec_per_row; v += kWave) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p <= kMaxRank; ++p)
      if (row[p] >= 0) fma_row(acc, wgt[p], y[(size_t)row[p] * vec_per_row + v], BF16);
    uint4 o;
    if (BF16) {
      o.x = f32_to_bf16_rne(acc[0]) | (f32_to_bf16_rne(acc[1]) << 16);
      o.y = f32_to_bf16_rne(acc[2]) | (f32_to_bf16_rne(acc[3]) << 16);
      o.z = f32_to_bf16_rne(acc[4]) | (f32_to_bf16_rne(acc[5]) << 16);
      o.w = f32_to_bf16_rne(acc[6]) | (f32_to_bf16_rne(acc[7]) << 16);
    } else {
      o.x = __builtin_bit_cast(u32, acc[0]);
      o.y = __builtin_bit_cast(u32, acc[1]);
      o.z = __builtin_bit_cast(u32, acc[2]);
      o.w = __builtin_bit_cast(u32, acc[3]);
    }
    out[(size_t)i * vec_per_row + v] = o;
  }
}

}  // namespace

hipError_t launch_gather(const Dims &D, const void *x, const rr_tables &tb, const Work &W, hipStream_t s) {
  const int es = D.dtype == RR_BF16 ? 2 : 4;
  const int vec_per_row = D.d * es / 16;
  const long long cand = (long long)D.E * D.C + (D.ir ? D.T : 0);
  const int grid = (int)((cand + PG_ROWS - 1) / PG_ROWS);
  prof_begin(K_GATHER, s);
  if (D.quota)
    gather_rows_kernel<<<(D.Rmax + PG_ROWS - 1) / PG_ROWS, PG_THREADS, 0, s>>>(
        static_cast<const uint4 *>(x), static_cast<uint4 *>(W.x_disp), vec_per_row, D.E, W.row_token, W.row_base);
  else
    gather_kernel<<<grid, PG_THREADS, 0, s>>>(static_cast<const uint4 *>(x), static_cast<uint4 *>(W.x_disp), vec_per_row,
                                              D.E, D.C, tb.slot_token, tb.fill_total, tb.ir_offset, tb.ir_token,
                                              tb.ir_expert, W.row_base);
  prof_end(K_GATHER, s);
  return hipGetLastError();
}

hipError_t launch_combine(const Dims &D, const rr_tables &tb, const Work &W, void *out, hipStream_t s) {
  const int es = D.dtype == RR_BF16 ? 2 : 4;
  const int vec_per_row = D.d * es / 16;
  const int skip = ffn_writes_single_rows(D) ? 1 : 0;
  prof_begin(K_COMBINE, s);
  // rows of up to 4 KB: one wave per token (no LDS, no barrier); longer rows: one workgroup per token
  if (vec_per_row <= 256) {
    if (D.dtype == RR_BF16)
      combine_wave_kernel<true><<<(D.T + 3) / 4, 256, 0, s>>>(static_cast<const uint4 *>(W.y), static_cast<uint4 *>(out),
                                                              vec_per_row, D.T, D.k, D.NR, tb.rank_expert, tb.slot,
                                                              tb.ir_expert, tb.ir_row, tb.fill_total, W.row_base, W.grp_off,
                                                              D.Cq, D.Gq, tb.combine_w, skip);
    else
      combine_wave_kernel<false><<<(D.T + 3) / 4, 256, 0, s>>>(static_cast<const uint4 *>(W.y), static_cast<uint4 *>(out),
                                                               vec_per_row, D.T, D.k, D.NR, tb.rank_expert, tb.slot,
                                                               tb.ir_expert, tb.ir_row, tb.fill_total, W.row_base,
                                                               W.grp_off, D.Cq, D.Gq, tb.combine_w, skip);
  } else {
    if (D.dtype == RR_BF16)
      combine_kernel<true><<<D.T, 256, 0, s>>>(static_cast<const uint4 *>(W.y), static_cast<uint4 *>(out), vec_per_row,
                                               D.k, D.NR, tb.rank_expert, tb.slot, tb.ir_expert, tb.ir_row,
                                               tb.fill_total, W.row_base, W.grp_off, D.Cq, D.Gq, tb.combine_w, skip);
    else
      combine_kernel<false><<<D.T, 256, 0, s>>>(static_cast<const uint4 *>(W.y), static_cast<uint4 *>(out), vec_per_row,
                                                D.k, D.NR, tb.rank_expert, tb.slot, tb.ir_expert, tb.ir_row,
                                                tb.fill_total, W.row_base, W.grp_off, D.Cq, D.Gq, tb.combine_w, skip);
  }
  prof_end(K_COMBINE, s);
  return hipGetLastError();
}

}  // namespace rr
