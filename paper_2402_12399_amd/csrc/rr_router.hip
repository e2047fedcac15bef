// Router scores (Eq. 1), softmax over all experts (App. A, Eq. 5) and argtopk.
//
// logits[T,E] = x[T,d] . w_router[E,d]^T (+ bias) with fp32 accuracy on the bf16 matrix cores:
// every fp32 operand is split exactly into three bf16 parts (8 + 8 + 8 mantissa bits, by
// truncation, so hi + lo + lo2 == value) and the products that matter are accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16:
//   bf16 x : x.w_hi + x.w_lo + x.w_lo2                                        (3 MFMAs, exact operands)
//   fp32 x : x_hi.w_hi + x_hi.w_lo + x_lo.w_hi + x_lo.w_lo + x_hi.w_lo2 + x_lo2.w_hi   (6 MFMAs; the
//            dropped products are below 2^-24 of the leading one)
// This keeps the kernel bound by the one pass over x in HBM instead of by fp32 FMA throughput.
//
// A workgroup of 4 waves owns TM*32 tokens; the waves split K four ways and each streams its K slice
// straight from global memory into MFMA operand registers (no LDS in the main loop, no barriers):
// lane (row r = lane%32, half h = lane/32) loads 64 contiguous bytes of row r per macro-step, the
// two halves taking adjacent segments, so every row is read in whole 128-byte lines.  The order in
// which K is fed to the MFMAs is permuted by that, identically for x and w, which a dot product does
// not see.  The four partial tiles are summed through LDS in a fixed order (deterministic), then the
// finished [token][expert] tile leaves as coalesced logits / probs rows and one lane per token ranks.
#include "rr_device.h"

namespace rr {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int RT_THREADS = 256;
constexpr int RT_NW = RT_THREADS / kWave;
constexpr int RT_TS = kMaxE + 1;  // LDS row stride of a [token][expert] tile

union Frag {
  u32 w[4];
  bf16x8 v;
};

// two fp32 values -> their three bf16 parts, packed pairwise (element 0 in the low half)
__device__ inline void split_pair(float f0, float f1, u32 &hi, u32 &lo, u32 &lo2) {
  const u32 b0 = __builtin_bit_cast(u32, f0), b1 = __builtin_bit_cast(u32, f1);
  const float r0 = f0 - __builtin_bit_cast(float, b0 & 0xffff0000u);
  const float r1 = f1 - __builtin_bit_cast(float, b1 & 0xffff0000u);
  const u32 c0 = __builtin_bit_cast(u32, r0), c1 = __builtin_bit_cast(u32, r1);
  const float s0 = r0 - __builtin_bit_cast(float, c0 & 0xffff0000u);
  const float s1 = r1 - __builtin_bit_cast(float, c1 & 0xffff0000u);
  hi = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
  lo = __builtin_amdgcn_perm(c1, c0, 0x07060302u);
  lo2 = __builtin_amdgcn_perm(__builtin_bit_cast(u32, s1), __builtin_bit_cast(u32, s0), 0x07060302u);
}

__device__ inline void split8(const uint4 a, const uint4 b, Frag &hi, Frag &lo, Frag &lo2) {
  const u32 raw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
  for (int p = 0; p < 4; ++p)
    split_pair(__builtin_bit_cast(float, raw[2 * p]), __builtin_bit_cast(float, raw[2 * p + 1]), hi.w[p], lo.w[p],
               lo2.w[p]);
}

template <bool BF16, int TM, int NJ>
__global__ __launch_bounds__(RT_THREADS) void router_kernel(const void *__restrict__ xv, const float *__restrict__ wr,
                                                            const float *__restrict__ bias, float *__restrict__ logits,
                                                            float *__restrict__ probs, int32_t *__restrict__ rank_expert,
                                                            int T, int d, int E, int k) {
  constexpr int TB = TM * 32;                 // tokens per workgroup
  constexpr int S = BF16 ? 32 : 16;           // elements in a lane's 64-byte segment
  constexpr int KM = 2 * S;                   // K advance per macro-step
  constexpr int MS = S / 8;                   // MFMA k-steps per macro-step
  constexpr int ES = BF16 ? 2 : 4;
  __shared__ float red[RT_NW][TB * RT_TS];
  __shared__ float row_max[TB], row_inv[TB];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int fr = lane & 31, fh = lane >> 5;
  const int t0 = blockIdx.x * TB;

  // this wave's K slice, in whole macro-steps
  const int steps_total = (d + KM - 1) / KM;
  const int steps_per_wave = (steps_total + RT_NW - 1) / RT_NW;
  const int kbeg = min(w * steps_per_wave, steps_total) * KM;
  const int kend = min(min((w + 1) * steps_per_wave, steps_total) * KM, d);

  const char *xrow[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i)
    xrow[i] = static_cast<const char *>(xv) + (size_t)min(t0 + i * 32 + fr, T - 1) * d * ES;
  const float *wrow[NJ];
  bool wok[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    wok[j] = j * 32 + fr < E;
    wrow[j] = wr + (size_t)min(j * 32 + fr, E - 1) * d;
  }

  f32x16 acc[TM][NJ];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  uint4 xr[TM][4], xn[TM][4];
  auto load_x = [&](int kb, uint4 (&dst)[TM][4]) {
    const int k0 = kb + fh * S;  // first element of this lane's segment
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int kq = k0 + q * (16 / ES);
        dst[i][q] = kq < kend ? *reinterpret_cast<const uint4 *>(xrow[i] + (size_t)kq * ES) : make_uint4(0, 0, 0, 0);
      }
  };

  if (kbeg < kend) load_x(kbeg, xr);
  for (int kb = kbeg; kb < kend; kb += KM) {
    if (kb + KM < kend) load_x(kb + KM, xn);
#pragma unroll
    for (int m = 0; m < MS; ++m) {
      // w fragments of this k-step: 8 consecutive fp32 of row (expert) fr, split into three parts
      const int kw = kb + fh * S + m * 8;
      Frag wh[NJ], wl[NJ], wl2[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        uint4 a = make_uint4(0, 0, 0, 0), b = a;
        if (wok[j] && kw < kend) {
          a = *reinterpret_cast<const uint4 *>(wrow[j] + kw);
          b = *reinterpret_cast<const uint4 *>(wrow[j] + kw + 4);
        }
        split8(a, b, wh[j], wl[j], wl2[j]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if (BF16) {
          Frag xf;
          xf.w[0] = xr[i][m].x; xf.w[1] = xr[i][m].y; xf.w[2] = xr[i][m].z; xf.w[3] = xr[i][m].w;
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.v, wl2[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.v, wl[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.v, wh[j].v, acc[i][j], 0, 0, 0);
          }
        } else {
          Frag xh, xl, xl2;
          split8(xr[i][2 * m], xr[i][2 * m + 1], xh, xl, xl2);
#pragma unroll
          for (int j = 0; j < NJ; ++j) {  // smallest products first
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl2.v, wh[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wl2[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, wl[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, wh[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wl[j].v, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wh[j].v, acc[i][j], 0, 0, 0);
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) xr[i][q] = xn[i][q];
  }

  // ---- partial tiles to LDS: accumulator element v is token 8*(v/4) + 4*(lane/32) + v%4, expert lane%32
  float *mine = red[w];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        mine[(i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3)) * RT_TS + j * 32 + fr] = acc[i][j][v];
  __syncthreads();
  // ---- fixed-order sum of the four K slices, plus bias
  float *tile = red[0];
  for (int idx = tid; idx < TB * E; idx += RT_THREADS) {
    const int row = idx / E, e = idx - row * E;
    const int o = row * RT_TS + e;
    tile[o] = ((red[0][o] + red[1][o]) + (red[2][o] + red[3][o])) + (bias ? bias[e] : 0.0f);
  }
  __syncthreads();

  const int ntok = min(TB, T - t0);
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

template <bool BF16, int TM>
void launch_one(const Dims &D, const void *x, const float *w_router, const float *bias, float *logits, float *probs,
                int32_t *rank_expert, hipStream_t s) {
  dim3 grid((D.T + TM * 32 - 1) / (TM * 32)), block(RT_THREADS);
  if (D.E <= 32)
    router_kernel<BF16, TM, 1><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k);
  else
    router_kernel<BF16, TM, 2><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k);
}

}  // namespace

hipError_t launch_router(const Dims &D, const void *x, const float *w_router, const float *bias, float *logits,
                         float *probs, int32_t *rank_expert, hipStream_t s) {
  // 32-token tiles while the batch is small enough that larger ones would leave CUs idle
  const bool small = D.T <= 64 * 1024;
  prof_begin(K_ROUTER, s);
  if (D.dtype == RR_BF16) {
    if (small) launch_one<true, 1>(D, x, w_router, bias, logits, probs, rank_expert, s);
    else launch_one<true, 2>(D, x, w_router, bias, logits, probs, rank_expert, s);
  } else {
    if (small) launch_one<false, 1>(D, x, w_router, bias, logits, probs, rank_expert, s);
    else launch_one<false, 2>(D, x, w_router, bias, logits, probs, rank_expert, s);
  }
  prof_end(K_ROUTER, s);
  return hipGetLastError();
}

}  // namespace rr
