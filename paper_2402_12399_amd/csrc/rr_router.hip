// Router scores (Eq. 1), softmax over all experts (App. A, Eq. 5) and argtopk.
//
// logits[T,E] = x[T,d] . w_router[E,d]^T (+ bias) with fp32 accuracy on the bf16 matrix cores:
// fp32 operands are split into bf16 parts, each the nearest bf16 (v_cvt_pk_bf16_f32) of what the
// previous parts left over, so k parts carry 9k mantissa bits; the products that matter are
// accumulated in fp32 by v_mfma_f32_32x32x16_bf16:
//   w      : three parts (27 bits)
//   bf16 x : x.w_hi + x.w_lo + x.w_lo2                                          (3 MFMAs, x exact)
//   fp32 x : two parts (18 bits: |x - x_hi - x_lo| <= 2^-18 |x|, i.e. <= 4e-6 relative per element,
//            ~1e-6 of a logit after the random-sign sum); x_hi.(w_hi + w_lo + w_lo2) + x_lo.(w_hi + w_lo)
//            (5 MFMAs; a third x part would double the splitting arithmetic, which is what bounds
//            the fp32 kernel, for accuracy below the fp32 rounding of the accumulation itself)
// The streaming kernel for large batches keeps two parts of w (18 bits, the precision it keeps of
// fp32 x anyway): x.w_hi + x.w_lo for bf16 x, x_hi.w_hi + x_hi.w_lo + x_lo.w_hi for fp32 x.
// This keeps the kernel near the one pass over x in HBM instead of bound by fp32 FMA throughput.
//
// A workgroup of 4 waves owns TM*32 tokens; the waves split K four ways and each streams its K slice
// straight from global memory into MFMA operand registers (no LDS in the main loop, no barriers):
// lane (row r = lane%32, half h = lane/32) loads 64 contiguous bytes of row r per macro-step, the
// two halves taking adjacent segments, so every row is read in whole 128-byte lines.  The order in
// which K is fed to the MFMAs is permuted by that, identically for x and w, which a dot product does
// not see.  The four partial tiles are summed through LDS in a fixed order (deterministic), then the
// finished [token][expert] tile leaves as coalesced logits / probs rows and one lane per token ranks.
#include <type_traits>

#include "rr_device.h"

namespace rr {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int RT_THREADS = 256;
constexpr int RT_NW = RT_THREADS / kWave;

union Frag {
  u32 w[4];
  bf16x8 v;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32), element 0 in the low half
__device__ inline u32 pack_bf16(float a, float b) {
  const f32x2_t f = {a, b};
  return __builtin_bit_cast(u32, __builtin_convertvector(f, bf16x2_t));
}
__device__ inline float lo_half(u32 p) { return __builtin_bit_cast(float, p << 16); }
__device__ inline float hi_half(u32 p) { return __builtin_bit_cast(float, p & 0xffff0000u); }

// value = hi + lo + lo2 up to 2^-27 of the value: each part is the nearest bf16 of what is left
// (the subtractions are exact), so three parts carry 27 bits
__device__ inline void split3_pair(float f0, float f1, u32 &hi, u32 &lo, u32 &lo2) {
  hi = pack_bf16(f0, f1);
  const float r0 = f0 - lo_half(hi), r1 = f1 - hi_half(hi);
  lo = pack_bf16(r0, r1);
  lo2 = pack_bf16(r0 - lo_half(lo), r1 - hi_half(lo));
}
// value = hi + lo up to 2^-18 of the value
__device__ inline void split2_pair(float f0, float f1, u32 &hi, u32 &lo) {
  hi = pack_bf16(f0, f1);
  lo = pack_bf16(f0 - lo_half(hi), f1 - hi_half(hi));
}

__device__ inline void split3x8(const uint4 a, const uint4 b, Frag &hi, Frag &lo, Frag &lo2) {
  const u32 raw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
  for (int p = 0; p < 4; ++p)
    split3_pair(__builtin_bit_cast(float, raw[2 * p]), __builtin_bit_cast(float, raw[2 * p + 1]), hi.w[p], lo.w[p],
                lo2.w[p]);
}
__device__ inline void split2x8(const uint4 a, const uint4 b, Frag &hi, Frag &lo) {
  const u32 raw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
  for (int p = 0; p < 4; ++p)
    split2_pair(__builtin_bit_cast(float, raw[2 * p]), __builtin_bit_cast(float, raw[2 * p + 1]), hi.w[p], lo.w[p]);
}

// acc += x . w for fp32 x in two parts and w in three: the five products above 2^-27 of the leading
// one, smallest first
__device__ inline f32x16 mfma5(const Frag &xh, const Frag &xl, const Frag &wh, const Frag &wl, const Frag &wl2, f32x16 acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wl2.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, wl.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, wh.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wl.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wh.v, acc, 0, 0, 0);
  return acc;
}

struct RankOut {
  int32_t *rank_expert, *slot;  // [T,k+1]
  u32 *key;                     // [T,NR]
  float *ir_score;              // [T]
  int32_t *ir_cand;             // [T]
  int32_t *blk_cnt;             // [NCAT, NBc]
  int k, NR, fr, Eg, Tg, NCAT, NBc;
};

// Two lanes rank one token from its finished row of logits (LDS): lanes l and l + 32 of a wave
// (half = 0, 1) each find the best experts of one half of the row, exchange them and merge, so the
// serial scan is half as long; both lanes of a token must call this together.  Lane half 0 then
// writes the top-(k+1) experts and, with FUSE, what the routing tables start from - score keys, the
// candidate counts of the token's count block (LDS atomics on cnt[round * E + expert]) - and lane
// half 1 the best expert of the token's own group (Sec. 4.1), so that the logits are not read back
// from HBM.
template <bool FUSE>
__device__ inline void rank_row(const float *row, int tok, int half, int E, int k, int32_t *rank_expert,
                                const RankOut &R, int *cnt) {
  const int n = min(k + 1, E);
  const int h = (E + 1) >> 1;
  int32_t *ranks = FUSE ? R.rank_expert : rank_expert;
  auto rank = [&](auto tag) {
    constexpr int N = decltype(tag)::value;  // list length: at least n
    unsigned long long b[N], o[N];
    top_keys_of_range<N>(row, half ? h : 0, half ? E : h, b);
#pragma unroll
    for (int q = 0; q < N; ++q) {  // the other half's list (fetched whole before this lane's own list changes)
      const u32 lo = __shfl_xor((u32)b[q], 32), hi = __shfl_xor((u32)(b[q] >> 32), 32);
      o[q] = ((unsigned long long)hi << 32) | lo;
    }
#pragma unroll
    for (int q = 0; q < N; ++q) insert_key(b, o[q]);
    if (half == 0) {
#pragma unroll
      for (int q = 0; q < kMaxRank; ++q) {
        const unsigned long long key = q < N ? b[q < N ? q : 0] : 0ull;
        const int e = rank_key_expert(key);  // -1 past the number of experts
        if (q <= k) ranks[(size_t)tok * (k + 1) + q] = (q < n) ? e : -1;
        if (FUSE && q < R.NR) {
          R.key[(size_t)tok * R.NR + q] = rank_key_score(key);
          atomicAdd(&cnt[q * E + e], 1);
        }
      }
      if (FUSE && !R.fr) R.slot[(size_t)tok * (k + 1) + k] = -1;
    }
  };
  if (n <= 3) rank(std::integral_constant<int, 3>{});
  else rank(std::integral_constant<int, kMaxRank>{});
  if (FUSE && half == 1) {
    const int g = tok / R.Tg;
    float best;
    int arg;
    best_in_group(row, g * R.Eg, (g + 1) * R.Eg, best, arg);
    R.ir_score[tok] = best;
    R.ir_cand[tok] = arg;
  }
}

// The same per-token results as rank_row from a [tokens][experts] tile in LDS, with every thread
// of the workgroup at work: the thread of (token, expert e) counts the experts that beat e - a
// greater score, or an equal one at a lower index (Eq. 1 argtopk, ties -> lower expert index) - and
// that count is e's rank; the same count inside the token's own group finds the best local expert
// (Sec. 4.1).  E^2 comparisons per token instead of E insertion steps, but no serial chain: the
// small-batch kernel's epilogue is latency, not arithmetic.
template <bool FUSE>
__device__ inline void rank_tile(const float *tile, int TS, int ntok, int t0, int E, int k, int32_t *rank_expert,
                                 const RankOut &R, int *cnt) {
  const int n = min(k + 1, E);
  int32_t *ranks = FUSE ? R.rank_expert : rank_expert;
  for (int idx = threadIdx.x; idx < ntok * E; idx += RT_THREADS) {
    const int row = idx / E, e = idx - row * E, tok = t0 + row;
    const float *a = tile + row * TS;
    const float v = a[e];
    int rank = 0;
    for (int o = 0; o < E; ++o) {
      const float x = a[o];
      rank += (x > v) || (x == v && o < e);
    }
    if (rank < n) {
      ranks[(size_t)tok * (k + 1) + rank] = e;
      if (FUSE && rank < R.NR) {
        R.key[(size_t)tok * R.NR + rank] = score_key(v);
        atomicAdd(&cnt[rank * E + e], 1);
      }
    }
    if (e == 0) {
      for (int q = n; q <= k; ++q) ranks[(size_t)tok * (k + 1) + q] = -1;
      if (FUSE && !R.fr) R.slot[(size_t)tok * (k + 1) + k] = -1;
    }
    if (FUSE) {
      const int g = tok / R.Tg, e0 = g * R.Eg;
      if (e >= e0 && e < e0 + R.Eg) {
        int before = 0;
        for (int o = e0; o < e0 + R.Eg; ++o) {
          const float x = a[o];
          before += (x > v) || (x == v && o < e);
        }
        if (before == 0) {
          R.ir_score[tok] = v;
          R.ir_cand[tok] = e;
        }
      }
    }
  }
}

template <bool BF16, int TM, int NJ, bool FUSE>
__global__ __launch_bounds__(RT_THREADS) void router_kernel(const void *__restrict__ xv, const float *__restrict__ wr,
                                                            const float *__restrict__ bias, float *__restrict__ logits,
                                                            float *__restrict__ probs, int32_t *__restrict__ rank_expert,
                                                            int T, int d, int E, int k, RankOut R) {
  constexpr int TB = TM * 32;                 // tokens per workgroup = one candidate-count block (FUSE)
  constexpr int S = BF16 ? 32 : 16;           // elements in a lane's 64-byte segment
  constexpr int KM = 2 * S;                   // K advance per macro-step
  constexpr int MS = S / 8;                   // MFMA k-steps per macro-step
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int TS = NJ * 32 + 1;             // LDS row stride of a [token][expert] tile
  __shared__ float red[RT_NW][TB * TS];
  __shared__ float row_max[TB], row_inv[TB];
  __shared__ int cnt[kMaxRounds * kMaxE];
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

  // w of a macro-step: per k-step 8 consecutive fp32 of row (expert) fr.  Fetched one macro-step
  // ahead like x (the weights sit in L2, but an L2 round trip per macro-step is most of a small
  // batch's run time when it is not hidden).
  uint4 wc[MS][NJ][2], wnx[MS][NJ][2];
  auto load_wm = [&](int kb, uint4 (&dst)[MS][NJ][2]) {
#pragma unroll
    for (int m = 0; m < MS; ++m) {
      const int kw = kb + fh * S + m * 8;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        dst[m][j][0] = dst[m][j][1] = make_uint4(0, 0, 0, 0);
        if (wok[j] && kw < kend) {
          dst[m][j][0] = *reinterpret_cast<const uint4 *>(wrow[j] + kw);
          dst[m][j][1] = *reinterpret_cast<const uint4 *>(wrow[j] + kw + 4);
        }
      }
    }
  };
  if (kbeg < kend) {
    load_x(kbeg, xr);
    load_wm(kbeg, wc);
  }
  for (int kb = kbeg; kb < kend; kb += KM) {
    if (kb + KM < kend) {
      load_x(kb + KM, xn);
      load_wm(kb + KM, wnx);
    }
#pragma unroll
    for (int m = 0; m < MS; ++m) {
      Frag wh[NJ], wl[NJ], wl2[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) split3x8(wc[m][j][0], wc[m][j][1], wh[j], wl[j], wl2[j]);
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
          Frag xh, xl;
          split2x8(xr[i][2 * m], xr[i][2 * m + 1], xh, xl);
#pragma unroll
          for (int j = 0; j < NJ; ++j) acc[i][j] = mfma5(xh, xl, wh[j], wl[j], wl2[j], acc[i][j]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) xr[i][q] = xn[i][q];
#pragma unroll
    for (int m = 0; m < MS; ++m)
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        wc[m][j][0] = wnx[m][j][0];
        wc[m][j][1] = wnx[m][j][1];
      }
  }

  // ---- partial tiles to LDS: accumulator element v is token 8*(v/4) + 4*(lane/32) + v%4, expert lane%32
  float *mine = red[w];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        mine[(i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3)) * TS + j * 32 + fr] = acc[i][j][v];
  __syncthreads();
  // ---- fixed-order sum of the four K slices, plus bias
  float *tile = red[0];
  for (int idx = tid; idx < TB * E; idx += RT_THREADS) {
    const int row = idx / E, e = idx - row * E;
    const int o = row * TS + e;
    tile[o] = ((red[0][o] + red[1][o]) + (red[2][o] + red[3][o])) + (bias ? bias[e] : 0.0f);
  }
  if (FUSE)
    for (int c = tid; c < R.NCAT; c += RT_THREADS) cnt[c] = 0;
  __syncthreads();

  const int ntok = min(TB, T - t0);
  // logits rows of this tile are contiguous in memory
  for (int idx = tid; idx < ntok * E; idx += RT_THREADS) {
    int row = idx / E, e = idx - row * E;
    logits[(size_t)t0 * E + idx] = tile[row * TS + e];
  }
  if (tid < ntok && probs) {
    const float *row = tile + tid * TS;
    float m = row[0];
    for (int e = 1; e < E; ++e) m = fmaxf(m, row[e]);
    float s = 0.0f;
    for (int e = 0; e < E; ++e) s += expf(row[e] - m);
    row_max[tid] = m;
    row_inv[tid] = 1.0f / s;
  }
  // more than 16 experts: two lanes per token, each scanning half the row (the E^2 comparisons of
  // rank_tile then cost more than the serial insertion saves); lanes l and l + 32 of wave 0 share token l
  static_assert(TB <= 32, "the two lanes of a token sit in one wave");
  if ((rank_expert || FUSE) && E > 16 && tid < 64 && (tid & 31) < ntok)
    rank_row<FUSE>(tile + (tid & 31) * TS, t0 + (tid & 31), tid >> 5, E, k, rank_expert, R, cnt);
  if ((rank_expert || FUSE) && E <= 16) rank_tile<FUSE>(tile, TS, ntok, t0, E, k, rank_expert, R, cnt);
  if (probs || FUSE) __syncthreads();
  if (probs) {
    for (int idx = tid; idx < ntok * E; idx += RT_THREADS) {
      int row = idx / E, e = idx - row * E;
      probs[(size_t)t0 * E + idx] = expf(tile[row * TS + e] - row_max[row]) * row_inv[row];
    }
  }
  if (FUSE)
    for (int c = tid; c < R.NCAT; c += RT_THREADS) R.blk_cnt[(size_t)c * R.NBc + blockIdx.x] = cnt[c];
}

// ------------------------------------------------------------------ large batches
// Streaming kernel (no K split, no reduction): a workgroup of 4 waves owns 128 tokens - one block of
// the routing kernels - and wave w the 32 tokens [32 w, 32 w + 32) over the whole K.
//   * x takes the route of the grouped GEMM's operands: buffer_load ... lds, 16 bytes per lane
//     straight into LDS, where a wave instruction covers 8 rows x 128 contiguous bytes (8 whole cache
//     lines); the MFMA fragments are then read from LDS (ds_read_b128; rows of 128 bytes, piece c of
//     row r at position c ^ ((r >> 1) & 7)).  Reading x with one row per lane, straight into the
//     fragment registers, makes every wave instruction touch 64 different lines for 16 bytes each,
//     and the rate at which the load unit looks lines up - not HBM - then bounds the kernel
//     (measured: 4.1 TB/s of algorithmic bytes at 1M x 1024 fp32 tokens, against 4.9 here).  No
//     registers hold x in flight, so the ring is as deep as LDS allows;
//   * a wave's part of the ring is its own, filled and read by nobody else: x needs no barrier,
//     the wave waits (counted, vmcnt) for its own loads.  Ring of XS stages of one K chunk (128
//     bytes of every row); a chunk's fragments are read into registers first thing and chunk c + XS
//     is requested into the stage that this frees, so XS chunks are in flight.  Rows past
//     the batch and pieces past d_model lie outside the buffer range and read as zero; requests
//     past the last chunk re-read the last chunk, so every chunk issues the same x loads and the
//     counted wait holds for any shape;
//   * the router weights go through LDS as well: every K chunk of w is split into its two bf16
//     parts ONCE per workgroup and stored as MFMA operand rows (swizzled like x); the weights of
//     chunk c + 2 are fetched (global -> registers) during chunk c and written to LDS at the end
//     of chunk c + 1; two stages, one barrier per chunk;
//   * two workgroups per CU (each at most 80 KB of LDS): one's epilogue overlaps the other's stream;
//   * the epilogue goes through a per-wave LDS tile; with a RankOut it also does the per-token work
//     that the routing tables start from (see rank_row), so the logits are not read back from HBM.
// What the compiler must not see: it makes every LDS load or store that follows an LDS-DMA load
// wait for that load - the ring's youngest request - because it cannot tell the stages apart.
// The fragment reads of x and the stores of the weight parts are therefore spelled out in assembly.
constexpr int RX_TB = kTokBlock;  // tokens per workgroup
static_assert(RX_TB == RT_NW * 32, "one 32-token fragment per wave");

template <bool BF16, int NJ>
struct RxLayout {
  static constexpr int KC = BF16 ? 64 : 32;          // K chunk: 128 bytes of a row of x
  static constexpr int ROWS = NJ * 32;               // expert rows staged
  static constexpr int ROWB = KC * 2;                // bytes of a staged bf16 weight row
  static constexpr int PART = ROWS * ROWB;           // one bf16 part of a weight chunk
  static constexpr int WSTAGE = 2 * PART;            // two bf16 parts of w
  static constexpr int XSTAGE = RX_TB * 128;         // one chunk of x for the workgroup: 16 KB
  static constexpr int XS = 4;                       // ring depth: two pairs of chunks
  static constexpr int TSTR = ROWS + 1;
  static constexpr int TILE_BYTES = RT_NW * 32 * TSTR * 4;  // epilogue tiles reuse the ring
  static constexpr int X_BYTES = XS * XSTAGE > TILE_BYTES ? XS * XSTAGE : TILE_BYTES;
  static constexpr int EPI_BYTES = (kMaxRounds * kMaxE + 2 * RT_NW * 32) * 4;  // epilogue counters and row statistics reuse the weight stages
  static constexpr int SMEM = X_BYTES + (2 * WSTAGE > EPI_BYTES ? 2 * WSTAGE : EPI_BYTES);
};

template <bool BF16, int NJ, bool FUSE>
__global__ __launch_bounds__(RT_THREADS, 2) void router_lds_kernel(const void *__restrict__ xv,
                                                                   const float *__restrict__ wr,
                                                                   const float *__restrict__ bias,
                                                                   float *__restrict__ logits, float *__restrict__ probs,
                                                                   int32_t *__restrict__ rank_expert, int T, int d, int E,
                                                                   int k, RankOut R) {
#if defined(__HIP_DEVICE_COMPILE__)  // buffer-resource and LDS-DMA builtins exist in the device pass only
  using L = RxLayout<BF16, NJ>;
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int KC = L::KC, ROWS = L::ROWS, ROWB = L::ROWB, PART = L::PART, WSTAGE = L::WSTAGE, XSTAGE = L::XSTAGE;
  constexpr int XS = L::XS, TSTR = L::TSTR;
  constexpr int NCH = ROWB / 16;                     // 16-byte pieces per weight row: 8 (bf16 x) or 4 (fp32 x)
  constexpr int WLD = ROWS * (KC / 4) / RT_THREADS;  // float4 loads of w per thread per chunk
  constexpr int NX = 32 * 128 / 1024;                // LDS-DMA instructions per wave per chunk (4)
  constexpr int KS = KC / 16;                        // MFMA k-steps per chunk
  extern __shared__ __attribute__((aligned(16))) char lds[];
  char *const wst = lds + L::X_BYTES;
  // only used after the K loop, in place of the weight stages (no static LDS: two workgroups fill a CU's 160 KB)
  int *const cnt = reinterpret_cast<int *>(wst);
  float(*const row_max)[32] = reinterpret_cast<float(*)[32]>(wst + kMaxRounds * kMaxE * 4);
  float(*const row_inv)[32] = row_max + RT_NW;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
  auto wswz = [](int r) { return NCH == 8 ? ((r >> 1) & 7) : ((r >> 2) & 3); };
  const int fsw_w = wswz(fr), fsw_x = (fr >> 1) & 7;
  // token block of this workgroup: XCD-aware, because neighbouring blocks write neighbouring words of
  // the per-list candidate counts (and neighbouring rows of every other output)
  const int blk = xcd_block(blockIdx.x, gridDim.x);
  const int t0 = blk * RX_TB, tw0 = t0 + w * 32;
  const int nchunk = (d + KC - 1) / KC;
  // Workgroup b walks the K chunks from chunk 11 b mod nchunk on, wrapping around (the same order for x
  // and w; a dot product does not care, only the rounding order of the sum changes with the block).
  // Workgroups that run side by side would otherwise all ask for the same 128-byte column of their
  // 4 KB rows at the same time, and those addresses fall on few memory channels (+6 % at 1M x 1024).
  const int rot = (int)((blockIdx.x * 11u) % (unsigned)nchunk);
  auto rc = [&](int c) { int q = c + rot; return q >= nchunk ? q - nchunk : q; };

  // ---- x: this wave's 32 rows as a buffer (rows past the batch are outside its range)
  const int rows_valid = max(0, min(32, T - tw0));
  const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char *>(static_cast<const char *>(xv)) + (size_t)min(tw0, T - 1) * d * ES, 0,
      __builtin_amdgcn_readfirstlane(rows_valid * d * ES), 0x00020000);
  // instruction i fills LDS rows [8 i, 8 i + 8) of the wave's stage: lane l -> row 8 i + l / 8, position
  // l % 8, i.e. it fetches piece (l % 8) ^ swizzle(row) of that row's chunk
  int xoff[NX], xpiece[NX];
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const int row = 8 * i + (lane >> 3);
    xpiece[i] = (lane & 7) ^ ((row >> 1) & 7);
    xoff[i] = row * d * ES + xpiece[i] * 16;
  }
  // requests chunk ca into stage sa and chunk cb into stage sb, alternating between the two instruction by instruction
  auto issue_x = [&](int ca, int sa, int cb, int sb) {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int c = h ? cb : ca, stage = h ? sb : sa;
        auto lp = (__attribute__((address_space(3))) void *)(lds + stage * XSTAGE + w * (32 * 128) + i * 1024);
        // pieces past d_model (the last chunk of a d_model that is not a multiple of KC) lie outside the range
        const int cr = rc(c);
        const bool past = (cr + 1) * KC > d && cr * KC + xpiece[i] * (16 / ES) >= d;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsx, lp, 16, past ? 0x7ffffff0 : xoff[i], cr * 128, 0, 0);
      }
    }
  };

  // ---- w staging: thread owns float4 (4 consecutive k) number tid + 256 q of the [ROWS][KC] chunk.
  // Out-of-range elements are fetched from a clamped address and zeroed when they are written to LDS
  // (not where they are loaded: a use right behind the load would wait for every load in flight), so
  // every chunk issues exactly WLD loads.
  float4 wbuf0[WLD], wbuf1[WLD];
  auto load_w = [&](int kc, float4 (&wreg)[WLD]) {
#pragma unroll
    for (int q = 0; q < WLD; ++q) {
      const int idx = tid + q * RT_THREADS, e = idx / (KC / 4), kk = kc + (idx % (KC / 4)) * 4;
      wreg[q] = *reinterpret_cast<const float4 *>(wr + (size_t)min(e, E - 1) * d + min(kk, d - 4));
    }
  };
  auto store_w = [&](int stage, int kc, const float4 (&wreg)[WLD]) {
    char *st = wst + stage * WSTAGE;
#pragma unroll
    for (int q = 0; q < WLD; ++q) {
      const int idx = tid + q * RT_THREADS, e = idx / (KC / 4), f4 = idx % (KC / 4);
      const float keep = (e < E && kc + f4 * 4 < d) ? 1.0f : 0.0f;  // d_model % 8 == 0: four elements are in or out together
      u32 h0, l0, h1, l1;
      split2_pair(wreg[q].x * keep, wreg[q].y * keep, h0, l0);
      split2_pair(wreg[q].z * keep, wreg[q].w * keep, h1, l1);
      const int off = e * ROWB + (((f4 >> 1) ^ wswz(e)) << 4) + (f4 & 1) * 8;
      // ds_write_b64 spelled out: the compiler makes an LDS store wait for every LDS-DMA load in flight
      // (it cannot tell the weight stages from the ring), which would drain the ring once per chunk
      typedef u32 u32x2 __attribute__((ext_vector_type(2)));
      const u32 a = (u32)(size_t)(__attribute__((address_space(3))) char *)(st + off);
      const u32x2 ph = {h0, h1}, pl = {l0, l1};
      asm volatile("ds_write_b64 %0, %1" ::"v"(a), "v"(ph) : "memory");
      asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(a), "v"(pl), "n"(PART) : "memory");
    }
  };

  f32x16 acc[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

  // x fragments of one chunk: four 16-byte pieces per lane.  Read with ds_read_b128 spelled out (see above).
  typedef u32 u32x4 __attribute__((ext_vector_type(4)));
  struct XFrag { u32x4 q0, q1, q2, q3; };
  auto read_x = [&](int c, XFrag &f) {
    const u32 sx = (u32)(size_t)(__attribute__((address_space(3))) char *)(lds + (c % XS) * XSTAGE + w * (32 * 128) + fr * 128);
    asm volatile("ds_read_b128 %0, %1" : "=v"(f.q0) : "v"(sx + (((4 * fh + 0) ^ fsw_x) << 4)) : "memory");
    asm volatile("ds_read_b128 %0, %1" : "=v"(f.q1) : "v"(sx + (((4 * fh + 1) ^ fsw_x) << 4)) : "memory");
    asm volatile("ds_read_b128 %0, %1" : "=v"(f.q2) : "v"(sx + (((4 * fh + 2) ^ fsw_x) << 4)) : "memory");
    asm volatile("ds_read_b128 %0, %1" : "=v"(f.q3) : "v"(sx + (((4 * fh + 3) ^ fsw_x) << 4)) : "memory");
  };
  // the arithmetic of one chunk: x fragments in registers, weights in LDS stage c & 1
  auto multiply = [&](int c, const XFrag &f) {
    const uint4 xq[4] = {make_uint4(f.q0.x, f.q0.y, f.q0.z, f.q0.w), make_uint4(f.q1.x, f.q1.y, f.q1.z, f.q1.w),
                         make_uint4(f.q2.x, f.q2.y, f.q2.z, f.q2.w), make_uint4(f.q3.x, f.q3.y, f.q3.z, f.q3.w)};
    const char *sw = wst + (c & 1) * WSTAGE;
#pragma unroll
    for (int m = 0; m < KS; ++m) {
      const int posw = ((KS * fh + m) ^ fsw_w) << 4;
      Frag wh[NJ], wl[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const char *rowp = sw + (j * 32 + fr) * ROWB + posw;
        wh[j].v = *reinterpret_cast<const bf16x8 *>(rowp);
        wl[j].v = *reinterpret_cast<const bf16x8 *>(rowp + PART);
      }
      if (BF16) {
        // lane (row fr, half fh) takes elements [32 fh + 8 m, +8): piece 4 fh + m
        Frag xf;
        xf.w[0] = xq[m].x; xf.w[1] = xq[m].y; xf.w[2] = xq[m].z; xf.w[3] = xq[m].w;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.v, wl[j].v, acc[j], 0, 0, 0);
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.v, wh[j].v, acc[j], 0, 0, 0);
        }
      } else {
        // elements [16 fh + 8 m, +8) of the chunk: pieces 4 fh + 2 m and the next
        Frag xh, xl;
        split2x8(xq[2 * m], xq[2 * m + 1], xh, xl);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {  // the three products above 2^-18 of the leading one, smallest first
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, wh[j].v, acc[j], 0, 0, 0);
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wl[j].v, acc[j], 0, 0, 0);
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, wh[j].v, acc[j], 0, 0, 0);
        }
      }
    }
  };
  // Two K chunks per trip.  x is requested in PAIRS of chunks, instruction by instruction, so that the
  // two adjacent 128-byte lines of a row reach the memory together (one open DRAM page serves both).
  // At the top of a trip the pair (c, c + 1) has landed: both chunks' fragments go into registers,
  // which frees their stages for the pair (c + XS, c + XS + 1); two pairs are always in flight.
  // The weights keep their own rhythm: chunk c's are in LDS stage c & 1 after the barrier, chunk
  // c + 1's in registers (wbuf1), chunk c + 2's are fetched into wbuf0 meanwhile.
  load_w(rc(0) * KC, wbuf0);
  load_w(rc(min(1, nchunk - 1)) * KC, wbuf1);
#pragma unroll
  for (int q = 0; q < XS; q += 2) {
    issue_x(min(q, nchunk - 1), q, min(q + 1, nchunk - 1), q + 1);
  }
  store_w(0, rc(0) * KC, wbuf0);
  for (int c = 0; c < nchunk; c += 2) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    load_w(rc(min(c + 2, nchunk - 1)) * KC, wbuf0);
    __builtin_amdgcn_sched_barrier(0);
    // The pair (c, c + 1) was requested XS chunks ago and one pair (2 NX x requests) has been issued since:
    // when no more loads than that are outstanding, it has landed (loads complete in order).  The weight
    // loads are left out of the count on purpose - the compiler may move them across this wait in either
    // direction, and counting a load that is not there would let the wait pass early; not counting one
    // that is there only makes it wait for part of the next pair as well.
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((XS - 2) * NX) : "memory");
    XFrag f0, f1;
    read_x(c, f0);
    read_x(c + 1, f1);
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f0.q0), "+v"(f0.q1), "+v"(f0.q2), "+v"(f0.q3), "+v"(f1.q0), "+v"(f1.q1), "+v"(f1.q2), "+v"(f1.q3)::"memory");
    issue_x(min(c + XS, nchunk - 1), c % XS, min(c + XS + 1, nchunk - 1), (c + 1) % XS);
    __builtin_amdgcn_sched_barrier(0);
    multiply(c, f0);
    __builtin_amdgcn_sched_barrier(0);
    store_w((c + 1) & 1, rc(min(c + 1, nchunk - 1)) * KC, wbuf1);
    if (c + 1 < nchunk) {
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      load_w(rc(min(c + 3, nchunk - 1)) * KC, wbuf1);
      __builtin_amdgcn_sched_barrier(0);
      multiply(c + 1, f1);
      __builtin_amdgcn_sched_barrier(0);
      store_w(c & 1, rc(min(c + 2, nchunk - 1)) * KC, wbuf0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // requests past the last chunk have landed: the ring becomes the tiles
  __syncthreads();

  // ---- epilogue through this wave's LDS tile
  float *tile = reinterpret_cast<float *>(lds) + w * 32 * TSTR;
  if (FUSE) {
    for (int c = tid; c < kMaxRounds * kMaxE; c += RT_THREADS) cnt[c] = 0;
    __syncthreads();
  }
  {
    const int tf0 = tw0;
    const int ntok = min(32, T - tf0);  // may be <= 0 for the last workgroup
    // accumulator element v is token 8*(v/4) + 4*(lane/32) + v%4, expert lane%32
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int e = j * 32 + fr;
      const float b = (bias && e < E) ? bias[e] : 0.0f;
#pragma unroll
      for (int v = 0; v < 16; ++v) tile[(8 * (v >> 2) + 4 * fh + (v & 3)) * TSTR + e] = acc[j][v] + b;
    }
    __builtin_amdgcn_wave_barrier();
    if (E == ROWS) {
      // a lane stores four consecutive experts of a token, a wave 1 KB per instruction
      constexpr int LPR = ROWS / 4;  // lanes per row
      const int r0 = lane / LPR, e0 = (lane % LPR) * 4;
#pragma unroll
      for (int it = 0; it < 32 / (kWave / LPR); ++it) {
        const int row = it * (kWave / LPR) + r0;
        const float *src = tile + row * TSTR + e0;
        if (row < ntok)
          *reinterpret_cast<float4 *>(logits + (size_t)(tf0 + row) * ROWS + e0) = make_float4(src[0], src[1], src[2], src[3]);
      }
    } else {
      for (int idx = lane; idx < ntok * E; idx += kWave) {
        const int row = idx / E, e = idx - row * E;
        logits[(size_t)tf0 * E + idx] = tile[row * TSTR + e];
      }
    }
    if (lane < ntok && probs) {
      const float *row = tile + lane * TSTR;
      float mx = row[0];
      for (int e = 1; e < E; ++e) mx = fmaxf(mx, row[e]);
      float sum = 0.0f;
      for (int e = 0; e < E; ++e) sum += expf(row[e] - mx);
      row_max[w][lane] = mx;
      row_inv[w][lane] = 1.0f / sum;
    }
    // lanes l and l + 32 rank token l of the wave's 32 together
    if ((rank_expert || FUSE) && fr < ntok) rank_row<FUSE>(tile + fr * TSTR, tf0 + fr, fh, E, k, rank_expert, R, cnt);
    if (probs) {
      __builtin_amdgcn_wave_barrier();
      for (int idx = lane; idx < ntok * E; idx += kWave) {
        const int row = idx / E, e = idx - row * E;
        probs[(size_t)tf0 * E + idx] = expf(tile[row * TSTR + e] - row_max[w][row]) * row_inv[w][row];
      }
    }
  }
  if (FUSE) {
    __syncthreads();
    for (int c = tid; c < R.NCAT; c += RT_THREADS) R.blk_cnt[(size_t)c * R.NBc + blk] = cnt[c];
  }
#endif
}

template <bool BF16, int TM>
void launch_one(const Dims &D, const void *x, const float *w_router, const float *bias, float *logits, float *probs,
                int32_t *rank_expert, const RankOut *R, hipStream_t s) {
  dim3 grid((D.T + TM * 32 - 1) / (TM * 32)), block(RT_THREADS);
  RankOut none{};
  if (D.E <= 32) {
    if (R) router_kernel<BF16, TM, 1, true><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k, *R);
    else router_kernel<BF16, TM, 1, false><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k, none);
  } else if constexpr (TM == 1) {  // two column fragments: the partial tiles of two token fragments would not fit LDS
    if (R) router_kernel<BF16, TM, 2, true><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k, *R);
    else router_kernel<BF16, TM, 2, false><<<grid, block, 0, s>>>(x, w_router, bias, logits, probs, rank_expert, D.T, D.d, D.E, D.k, none);
  }
}

template <bool BF16>
void launch_stream(const Dims &D, const void *x, const float *w_router, const float *bias, float *logits, float *probs,
                   int32_t *rank_expert, const RankOut *R, hipStream_t s) {
  dim3 grid((D.T + RX_TB - 1) / RX_TB), block(RT_THREADS);
  RankOut none{};
#define RR_LAUNCH_STREAM(NJ)                                                                                            \
  do {                                                                                                                  \
    constexpr int smem = RxLayout<BF16, NJ>::SMEM;                                                                      \
    if (R) router_lds_kernel<BF16, NJ, true><<<grid, block, smem, s>>>(x, w_router, bias, logits, probs, rank_expert,    \
                                                                       D.T, D.d, D.E, D.k, *R);                         \
    else router_lds_kernel<BF16, NJ, false><<<grid, block, smem, s>>>(x, w_router, bias, logits, probs, rank_expert,     \
                                                                      D.T, D.d, D.E, D.k, none);                        \
  } while (0)
  if (D.E <= 32) RR_LAUNCH_STREAM(1);
  else RR_LAUNCH_STREAM(2);
#undef RR_LAUNCH_STREAM
}

}  // namespace

// The streaming kernel's dynamic LDS exceeds the default limit: raised once per device by the caller.
hipError_t router_kernel_attributes() {
  hipError_t e = hipSuccess;
  auto set = [&e](auto kern, int bytes) {
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  };
  set(router_lds_kernel<true, 1, true>, RxLayout<true, 1>::SMEM);
  set(router_lds_kernel<true, 1, false>, RxLayout<true, 1>::SMEM);
  set(router_lds_kernel<true, 2, true>, RxLayout<true, 2>::SMEM);
  set(router_lds_kernel<true, 2, false>, RxLayout<true, 2>::SMEM);
  set(router_lds_kernel<false, 1, true>, RxLayout<false, 1>::SMEM);
  set(router_lds_kernel<false, 1, false>, RxLayout<false, 1>::SMEM);
  set(router_lds_kernel<false, 2, true>, RxLayout<false, 2>::SMEM);
  set(router_lds_kernel<false, 2, false>, RxLayout<false, 2>::SMEM);
  return e;
}

// Up to 16 K tokens the K-split kernel (32 tokens per workgroup: 512 workgroups at 16 K tokens), above
// the streaming kernel (128 tokens per workgroup; at 32 K tokens x 4096 bf16 it takes 76 us, the
// K-split kernel 115 us; at 16 K tokens the K-split kernel is still ahead, 47 against 55 us).
static bool router_small(const Dims &D) { return D.T <= 16 * 1024; }
int router_count_blocks(const Dims &D) { return router_small(D) ? kTokBlock / 32 : 1; }

hipError_t launch_router(const Dims &D, const void *x, const float *w_router, const float *bias, float *logits,
                         float *probs, int32_t *rank_expert, const rr_tables *tb, const Work *W, hipStream_t s) {
  // small batches: 32-token tiles with K split across the waves, so that the launch still fills the
  // chip; large ones: the streaming kernel
  const bool small = router_small(D);
  prof_begin(K_ROUTER, s);
  RankOut R{};
  if (tb && W)  // D.NBc is then the count-block grid of this router (see router_count_blocks)
    R = RankOut{tb->rank_expert, tb->slot, W->key, W->ir_score, W->ir_cand, W->blk_cnt,
                D.k, D.NR, D.fr, D.Eg, D.Tg, D.NCAT, D.NBc};
  if (small) {
    const RankOut *Rp = tb && W ? &R : nullptr;
    if (D.dtype == RR_BF16) launch_one<true, 1>(D, x, w_router, bias, logits, probs, rank_expert, Rp, s);
    else launch_one<false, 1>(D, x, w_router, bias, logits, probs, rank_expert, Rp, s);
  } else {
    if (D.dtype == RR_BF16) launch_stream<true>(D, x, w_router, bias, logits, probs, rank_expert, tb && W ? &R : nullptr, s);
    else launch_stream<false>(D, x, w_router, bias, logits, probs, rank_expert, tb && W ? &R : nullptr, s);
  }
  prof_end(K_ROUTER, s);
  return hipGetLastError();
}

}  // namespace rr
