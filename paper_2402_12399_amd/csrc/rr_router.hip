// Router scores (Eq. 1), softmax over all experts (App. A, Eq. 5) and argtopk.
//
// logits[T,E] = x[T,d] . w_router[E,d]^T (+ bias), fp32 accumulate.  One workgroup owns
// kTokBlock tokens and all E <= 64 experts, streams x once from HBM in K-chunks through LDS and
// keeps the [tokens x experts] accumulators in registers.  The finished tile is parked in LDS so
// that logits / probs leave as coalesced rows and each token's ranking is done by one lane.
#include "rr_device.h"

namespace rr {

namespace {

constexpr int RT_THREADS = 256;
constexpr int RT_BK = 32;                    // K-chunk
constexpr int RT_XS = kTokBlock + 2;         // LDS row stride of the transposed x chunk (words)
constexpr int RT_WS = kMaxE + 2;             // LDS row stride of the transposed w chunk
constexpr int RT_TS = kMaxE + 1;             // LDS row stride of the finished [token][expert] tile
constexpr int RT_LDS_WORDS =
    (RT_BK * RT_XS + RT_BK * RT_WS) > (kTokBlock * RT_TS) ? (RT_BK * RT_XS + RT_BK * RT_WS) : (kTokBlock * RT_TS);

__device__ inline float bf16_to_f32(uint16_t b) { return __builtin_bit_cast(float, (u32)b << 16); }

template <bool BF16>
__global__ __launch_bounds__(RT_THREADS) void router_kernel(const void *__restrict__ xv, const float *__restrict__ wr,
                                                            const float *__restrict__ bias, float *__restrict__ logits,
                                                            float *__restrict__ probs, int32_t *__restrict__ rank_expert,
                                                            int T, int d, int E, int k) {
  __shared__ float lds[RT_LDS_WORDS];
  __shared__ float row_max[kTokBlock], row_inv[kTokBlock];
  float *xs = lds;                      // [RT_BK][RT_XS]  xs[kk][token]
  float *ws = lds + RT_BK * RT_XS;      // [RT_BK][RT_WS]  ws[kk][expert]
  const int tid = threadIdx.x;
  const int t0 = blockIdx.x * kTokBlock;
  const int ty = tid >> 3, tx = tid & 7;  // tokens ty*4..+3, experts tx + 8q
  const int nq = (E + 7) >> 3;

  float acc[4][8];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[a][q] = 0.0f;

  for (int k0 = 0; k0 < d; k0 += RT_BK) {
    // ---- stage x chunk [kTokBlock][RT_BK] transposed into xs
    if (BF16) {
      const uint16_t *x = static_cast<const uint16_t *>(xv);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        int idx = tid + i * RT_THREADS;       // 512 loads of 8 bf16
        int row = idx >> 2, c8 = idx & 3;
        int tok = t0 + row, kk = k0 + c8 * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (tok < T && kk < d) v = *reinterpret_cast<const uint4 *>(x + (size_t)tok * d + kk);
        u32 w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          xs[(c8 * 8 + 2 * j) * RT_XS + row] = __builtin_bit_cast(float, w4[j] << 16);
          xs[(c8 * 8 + 2 * j + 1) * RT_XS + row] = __builtin_bit_cast(float, w4[j] & 0xffff0000u);
        }
      }
    } else {
      const float *x = static_cast<const float *>(xv);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int idx = tid + i * RT_THREADS;       // 1024 loads of 4 floats
        int row = idx >> 3, c4 = idx & 7;
        int tok = t0 + row, kk = k0 + c4 * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (tok < T && kk < d) v = *reinterpret_cast<const float4 *>(x + (size_t)tok * d + kk);
        xs[(c4 * 4 + 0) * RT_XS + row] = v.x;
        xs[(c4 * 4 + 1) * RT_XS + row] = v.y;
        xs[(c4 * 4 + 2) * RT_XS + row] = v.z;
        xs[(c4 * 4 + 3) * RT_XS + row] = v.w;
      }
    }
    // ---- stage w chunk [E][RT_BK] transposed into ws
    for (int idx = tid; idx < E * (RT_BK / 4); idx += RT_THREADS) {
      int e = idx >> 3, c4 = idx & 7;
      int kk = k0 + c4 * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (kk < d) v = *reinterpret_cast<const float4 *>(wr + (size_t)e * d + kk);
      ws[(c4 * 4 + 0) * RT_WS + e] = v.x;
      ws[(c4 * 4 + 1) * RT_WS + e] = v.y;
      ws[(c4 * 4 + 2) * RT_WS + e] = v.z;
      ws[(c4 * 4 + 3) * RT_WS + e] = v.w;
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < RT_BK; ++kk) {
      float xa[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) xa[a] = xs[kk * RT_XS + ty * 4 + a];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        if (q < nq) {
          float wv = ws[kk * RT_WS + tx + 8 * q];
#pragma unroll
          for (int a = 0; a < 4; ++a) acc[a][q] = fmaf(xa[a], wv, acc[a][q]);
        }
      }
    }
    __syncthreads();
  }

  // ---- park the finished tile in LDS (bias added), tile[token][expert]
  float *tile = lds;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    int e = tx + 8 * q;
    if (e < E) {
      float b = bias ? bias[e] : 0.0f;
#pragma unroll
      for (int a = 0; a < 4; ++a) tile[(ty * 4 + a) * RT_TS + e] = acc[a][q] + b;
    }
  }
  __syncthreads();

  const int ntok = min(kTokBlock, T - t0);
  // logits rows of this tile are contiguous in memory
  for (int idx = tid; idx < ntok * E; idx += RT_THREADS) {
    int row = idx / E, e = idx - row * E;
    logits[(size_t)t0 * E + idx] = tile[row * RT_TS + e];
  }
  if (tid < ntok) {
    const float *row = tile + tid * RT_TS;
    if (probs) {
      float m = row[0];
      for (int e = 1; e < E; ++e) m = fmaxf(m, row[e]);
      float s = 0.0f;
      for (int e = 0; e < E; ++e) s += expf(row[e] - m);
      row_max[tid] = m;
      row_inv[tid] = 1.0f / s;
    }
    if (rank_expert) {
      float bs[kMaxRank];
      int be[kMaxRank];
      int n = min(k + 1, E);
      top_n_of_row(row, E, n, bs, be);
#pragma unroll
      for (int q = 0; q < kMaxRank; ++q)
        if (q <= k) rank_expert[(size_t)(t0 + tid) * (k + 1) + q] = (q < n) ? be[q] : -1;
    }
  }
  if (probs) {
    __syncthreads();
    for (int idx = tid; idx < ntok * E; idx += RT_THREADS) {
      int row = idx / E, e = idx - row * E;
      probs[(size_t)t0 * E + idx] = expf(tile[row * RT_TS + e] - row_max[row]) * row_inv[row];
    }
  }
}

}  // namespace

hipError_t launch_router(const Dims &D, const void *x, const float *w_router, const float *bias, float *logits,
                         float *probs, int32_t *rank_expert, hipStream_t s) {
  dim3 grid(D.NB), block(RT_THREADS);
  prof_begin(K_ROUTER, s);
  if (D.dtype == RR_BF16)
    router_kernel<true><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k);
  else
    router_kernel<false><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k);
  prof_end(K_ROUTER, s);
  return hipGetLastError();
}

}  // namespace rr
