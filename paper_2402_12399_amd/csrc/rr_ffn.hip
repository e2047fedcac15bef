// Expert FFN as a grouped GEMM over the dispatched rows (Sec. 5.1: every expert is a LLaMA FFN):
//   up   : h[row, f] = silu(x_disp[row] . W1_e[f]) * (x_disp[row] . W3_e[f])      (SwiGLU)
//          h[row, f] = gelu(x_disp[row] . W1_e[f])                                 (GELU)
//   down : y[row, c] = h[row] . W2_e[c]
// Both are "A[rows,K] times B[N,K]^T" with K contiguous in both operands; rows of expert e are
// row_base[e] .. row_base[e+1]-1 and are cut into row tiles by row_plan (tile_expert, tile_row0).
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulate.  A workgroup of 4 waves owns a BM x BN
// output tile; K advances in chunks of 64 through double-buffered LDS (global -> registers -> LDS
// overlapped with the MFMAs of the previous chunk).  LDS rows are 128 B; the 16-byte chunk c of
// row r lives at chunk position c ^ (r & 7), which makes both the row-wise stores and the
// fragment loads (32 rows x one chunk) conflict-free.
// fp32 path (tiny fp32 workload): plain FMA tiles, fp32 throughout.
#include <type_traits>

#include "rr_device.h"

namespace rr {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ inline u32 f32_to_bf16_bits(float f) {
  u32 u = __builtin_bit_cast(u32, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ inline float silu(float g) { return g / (1.0f + __expf(-g)); }
__device__ inline float gelu_erf(float g) { return 0.5f * g * (1.0f + erff(g * 0.70710678118654752f)); }

constexpr int GB_THREADS = 256;
constexpr int GB_BK = 64;             // bf16 elements per K chunk = 128 B per LDS row
constexpr int GB_ROW_BYTES = 128;

struct GemmArgs {
  const void *A;        // [rows, K]
  const void *B0;       // [E, N, K]
  const void *B1;       // [E, N, K] gated only
  void *Cout;           // [rows, N]
  int K, N;
  int NT;               // column tiles
  int map_mode;         // workgroup id -> tile mapping (see map_tile)
  const int32_t *row_base, *tile_expert, *tile_row0, *n_tiles;
};

// WAVES_M x WAVES_N waves, each owning WM x WN fragments of 32x32.
// GATED: the staged B rows are [BN gate rows | BN up rows] with BN = BROWS / 2, and a wave's
// fragments j < WN/2 are gate columns, j >= WN/2 the matching up columns.
// Epilogue shared by the bf16 kernels: activation, round to bf16, store (masked on edge tiles).
// Accumulator element v of a 32x32 fragment is row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
template <int WAVES_N, int WM, int WN, bool GATED, int ACT>
__device__ inline void store_tile(f32x16 (&acc)[WM][WN], uint16_t *Cb, int rbase, int rows_e, int m0, int n0, int N,
                                  int wm, int wn, int lane) {
  constexpr int NJ = GATED ? WN / 2 : WN;           // output column fragments per wave
  constexpr int BM = 0;                             // (unused; tile extents come from the wave layout)
  (void)BM;
  const int fr = lane & 31, fh = lane >> 5;
  const int wrow0 = m0 + wm * WM * 32, wcol0 = n0 + wn * NJ * 32;
  const bool interior = wrow0 + WM * 32 <= rows_e && wcol0 + NJ * 32 <= N;
  uint16_t *base = Cb + (size_t)(rbase + wrow0 + 4 * fh) * N + wcol0 + fr;
#pragma unroll
  for (int i = 0; i < WM; ++i) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      uint16_t *p = base + (size_t)(i * 32) * N + j * 32;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float c = acc[i][j][v];
        if (GATED) c = silu(c) * acc[i][j + NJ][v];
        if (ACT == RR_ACT_GELU) c = gelu_erf(c);
        const int dr = 8 * (v >> 2) + (v & 3);
        if (interior || (wrow0 + i * 32 + 4 * fh + dr < rows_e && wcol0 + j * 32 + fr < N))
          p[(size_t)dr * N] = (uint16_t)f32_to_bf16_bits(c);
      }
    }
  }
}

// Workgroup id -> (row tile, column tile).  Consecutive workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2, so XCD x runs ids x, x+8, ...  The tile grid is cut into panels of
// GEMM_GM row tiles x GEMM_GN column tiles = 32 tiles, about what one XCD holds at a time; panel p
// goes to XCD p % 8 and the 32 consecutive ids of that XCD walk it.  Workgroups resident on an XCD
// then share their operand tiles through its L2, neighbouring panels (same row tiles, next column
// tiles) run on the other XCDs at the same time and share the A rows through the memory-side cache,
// and every XCD gets the same mix of full and ragged tiles.
constexpr int GEMM_GM = 4, GEMM_GN = 8;
__host__ __device__ inline int gemm_grid(int m_tiles, int NT) {
  const int panels = ((m_tiles + GEMM_GM - 1) / GEMM_GM) * ((NT + GEMM_GN - 1) / GEMM_GN);
  return ((panels + 7) / 8) * 8 * (GEMM_GM * GEMM_GN);
}
// mode 0: plain order, column tile fastest (used when the column tiles do not fill whole panels: a
// half-empty panel would leave its XCD short of work); mode 2: panels.
__device__ inline bool map_tile(int bid, int n_tiles, int NT, int &mt, int &nt, int mode) {
  if (mode == 0) {
    mt = bid / NT;
    nt = bid - mt * NT;
    return mt < n_tiles;
  }
  const int xcd = bid & 7, j = bid >> 3;
  const int p = (j / (GEMM_GM * GEMM_GN)) * 8 + xcd, within = j % (GEMM_GM * GEMM_GN);
  const int npn = (NT + GEMM_GN - 1) / GEMM_GN;
  const int mg = p / npn, np = p - mg * npn;
  mt = mg * GEMM_GM + within % GEMM_GM;
  nt = np * GEMM_GN + within / GEMM_GM;
  return mt < n_tiles && nt < NT;
}

template <int SWZ>
__device__ inline int swz(int r) { return SWZ == 0 ? (r & 7) : ((r >> 1) & 7); }

template <int WAVES_M, int WAVES_N, int WM, int WN, bool GATED, int ACT, int SWZ>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_bf16_kernel(GemmArgs P) {
  constexpr int NTHR = WAVES_M * WAVES_N * 64;
  constexpr int RPP = NTHR / 8;       // rows covered by one pass of 16-byte loads
  constexpr int BM = WAVES_M * WM * 32;
  constexpr int BROWS = WAVES_N * WN * 32;
  constexpr int BN = GATED ? BROWS / 2 : BROWS;
  constexpr int A_LD = BM / RPP;      // 16-byte loads per thread per chunk
  constexpr int B_LD = BROWS / RPP;
  constexpr int STAGE_BYTES = (BM + BROWS) * GB_ROW_BYTES;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  int mt, nt;
  if (!map_tile(blockIdx.x, *P.n_tiles, P.NT, mt, nt, P.map_mode)) return;
  const int e = P.tile_expert[mt];
  const int m0 = P.tile_row0[mt];
  const int rbase = P.row_base[e];
  const int rows_e = P.row_base[e + 1] - rbase;
  const int n0 = nt * BN;
  const int K = P.K, N = P.N;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w / WAVES_N, wn = w % WAVES_N;

  const char *Ab = static_cast<const char *>(P.A);
  const char *B0b = static_cast<const char *>(P.B0) + (size_t)e * N * K * 2;
  const char *B1b = GATED ? static_cast<const char *>(P.B1) + (size_t)e * N * K * 2 : nullptr;

  // per-thread global sources: chunk id q = tid + 256 i -> row q / 8, chunk q % 8
  const int lc = tid & 7;
  const char *a_src[A_LD];
  const char *b_src[B_LD];
  int lds_off_a[A_LD], lds_off_b[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    int r = (tid >> 3) + RPP * i;
    int gr = min(m0 + r, rows_e - 1);
    a_src[i] = Ab + ((size_t)(rbase + gr) * K + lc * 8) * 2;
    lds_off_a[i] = r * GB_ROW_BYTES + ((lc ^ swz<SWZ>(r)) << 4);
  }
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    int r = (tid >> 3) + RPP * i;
    const char *bb = B0b;
    int nr = r;
    if (GATED && r >= BN) { bb = B1b; nr = r - BN; }
    int gn = min(n0 + nr, N - 1);
    b_src[i] = bb + ((size_t)gn * K + lc * 8) * 2;
    lds_off_b[i] = BM * GB_ROW_BYTES + r * GB_ROW_BYTES + ((lc ^ swz<SWZ>(r)) << 4);
  }

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  uint4 ra[A_LD], rb[B_LD];
  const int KT = (K + GB_BK - 1) / GB_BK;
  auto load_global = [&](int kt) {
    const int kbyte = kt * GB_BK * 2;
    const bool in = (kt * GB_BK + lc * 8) < K;
#pragma unroll
    for (int i = 0; i < A_LD; ++i) ra[i] = in ? *reinterpret_cast<const uint4 *>(a_src[i] + kbyte) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < B_LD; ++i) rb[i] = in ? *reinterpret_cast<const uint4 *>(b_src[i] + kbyte) : make_uint4(0, 0, 0, 0);
  };
  auto store_lds = [&](int buf) {
    char *st = smem + buf * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < A_LD; ++i) *reinterpret_cast<uint4 *>(st + lds_off_a[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) *reinterpret_cast<uint4 *>(st + lds_off_b[i]) = rb[i];
  };

  // fragment addressing: lane reads row (lane & 31), chunk 2*ks + (lane >> 5)
  const int fr = lane & 31, fh = lane >> 5;
  int a_row_off[WM], b_row_off[WN], a_sw[WM], b_sw[WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    int r = (wm * WM + i) * 32 + fr;
    a_row_off[i] = r * GB_ROW_BYTES;
    a_sw[i] = swz<SWZ>(r);
  }
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    int r;
    if (GATED) {
      constexpr int H = WN / 2;
      r = (j < H) ? (wn * H + j) * 32 + fr : BN + (wn * H + (j - H)) * 32 + fr;
    } else {
      r = (wn * WN + j) * 32 + fr;
    }
    b_row_off[j] = BM * GB_ROW_BYTES + r * GB_ROW_BYTES;
    b_sw[j] = swz<SWZ>(r);
  }

  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    if (kt + 1 < KT) load_global(kt + 1);
    const char *st = smem + (kt & 1) * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < GB_BK / 16; ++ks) {
      bf16x8 af[WM], bfr[WN];
      const int c = 2 * ks + fh;
#pragma unroll
      for (int i = 0; i < WM; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(st + a_row_off[i] + ((c ^ a_sw[i]) << 4));
#pragma unroll
      for (int j = 0; j < WN; ++j) bfr[j] = *reinterpret_cast<const bf16x8 *>(st + b_row_off[j] + ((c ^ b_sw[j]) << 4));
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  store_tile<WAVES_N, WM, WN, GATED, ACT>(acc, static_cast<uint16_t *>(P.Cout), rbase, rows_e, m0, n0, N, wm, wn, lane);
}

// Direct-to-LDS variant (K % 64 == 0): global_load_lds_dwordx4 moves 16 bytes per lane straight
// into LDS, a wave instruction filling 1 KB = 8 consecutive LDS rows (lane l -> row l/8, chunk
// position l%8), so the swizzle is applied on the global side: the lane fetches the chunk that
// belongs at its position.  Two 64 KB stages; the loads of chunk kt+1 are in flight during all
// MFMAs of chunk kt, and fragments are double-buffered in registers across the four 16-wide
// k-steps of a chunk.
template <int WAVES_M, int WAVES_N, int WM, int WN, bool GATED, int ACT, int SWZ>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_bf16_dl_kernel(GemmArgs P) {
#if defined(__HIP_DEVICE_COMPILE__)  // buffer-resource and LDS-DMA builtins exist in the device pass only
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int BM = WAVES_M * WM * 32;
  constexpr int BROWS = WAVES_N * WN * 32;
  constexpr int BN = GATED ? BROWS / 2 : BROWS;
  constexpr int STAGE_BYTES = (BM + BROWS) * GB_ROW_BYTES;
  constexpr int NI = (BM + BROWS) / 8 / NW;  // load instructions per wave per chunk
  constexpr int NIA = BM / 8 / NW, NIB0 = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "operand boundaries must fall between load instructions");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  int mt, nt;
  if (!map_tile(blockIdx.x, *P.n_tiles, P.NT, mt, nt, P.map_mode)) return;
  const int e = P.tile_expert[mt];
  const int m0 = P.tile_row0[mt];
  const int rbase = P.row_base[e];
  const int rows_e = P.row_base[e + 1] - rbase;
  const int n0 = nt * BN;
  const int K = P.K, N = P.N;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps LDS-DMA addressing scalar
  const int wm = w / WAVES_N, wn = w % WAVES_N;

  const char *Ab = static_cast<const char *>(P.A);
  const char *B0b = static_cast<const char *>(P.B0) + (size_t)e * N * K * 2;
  const char *B1b = GATED ? static_cast<const char *>(P.B1) + (size_t)e * N * K * 2 : nullptr;

  // instruction i of wave w fills stage rows [8 q, 8 q + 8), q = i * NW + w.  Buffer loads: one
  // descriptor per operand, rows past the end of the operand read as zero.
  const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char *>(Ab + (size_t)rbase * K * 2), 0, (int)min((size_t)rows_e * K * 2, (size_t)0x7fffffff), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsB0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(B0b), 0, N * K * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsB1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(GATED ? B1b : B0b), 0, N * K * 2, 0x00020000);
  int voff[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int r = (i * NW + w) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz<SWZ>(r);
    int row;
    if (r < BM) {
      row = m0 + r;
    } else {
      int nr = r - BM;
      if (GATED && nr >= BN) nr -= BN;
      row = n0 + nr;
    }
    voff[i] = row * K * 2 + c * 16;
  }
  auto issue_loads = [&](int kt, int buf) {
    char *st = smem + buf * STAGE_BYTES + w * 1024;
    const int koff = kt * (GB_BK * 2);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      // which operand instruction i reads is known at compile time: 8 NW | BM and 8 NW | BN
      auto lp = (__attribute__((address_space(3))) void *)(st + i * NW * 1024);
      if (i < NIA)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, lp, 16, voff[i], koff, 0, 0);
      else if (!GATED || i < NIA + NIB0)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB0, lp, 16, voff[i], koff, 0, 0);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB1, lp, 16, voff[i], koff, 0, 0);
    }
  };

  const int fr = lane & 31, fh = lane >> 5;
  int a_off[WM], b_off[WN], a_sw[WM], b_sw[WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    int r = (wm * WM + i) * 32 + fr;
    a_off[i] = r * GB_ROW_BYTES;
    a_sw[i] = swz<SWZ>(r);
  }
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    int r;
    if (GATED) {
      constexpr int H = WN / 2;
      r = (j < H) ? (wn * H + j) * 32 + fr : BN + (wn * H + (j - H)) * 32 + fr;
    } else {
      r = (wn * WN + j) * 32 + fr;
    }
    b_off[j] = (BM + r) * GB_ROW_BYTES;
    b_sw[j] = swz<SWZ>(BM + r);
  }

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int KT = K / GB_BK;
  // Ragged row tiles: the last tile of an expert is mostly padding.  A wave skips the fragment
  // loads and MFMAs of its 32-row fragments that lie wholly past the expert's last row (a
  // wave-uniform test), so a padded tile costs MFMA time in proportion to its real rows.  Full
  // tiles take a branch-free copy of the loop (FULL), which keeps its counted waits exact.
  const int live = min(WM, max(0, (rows_e - m0 - wm * WM * 32 + 31) >> 5));
  auto k_loop = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    bf16x8 af[2][WM], bfr[2][WN];
    auto load_frags = [&](const char *st, int ks, int slot) {
      const int c = 2 * ks + fh;
#pragma unroll
      for (int i = 0; i < WM; ++i)
        if (FULL || i < live) af[slot][i] = *reinterpret_cast<const bf16x8 *>(st + a_off[i] + ((c ^ a_sw[i]) << 4));
      if (FULL || live > 0) {
#pragma unroll
        for (int j = 0; j < WN; ++j) bfr[slot][j] = *reinterpret_cast<const bf16x8 *>(st + b_off[j] + ((c ^ b_sw[j]) << 4));
      }
    };
    auto mfma_step = [&](int slot) {
#pragma unroll
      for (int i = 0; i < WM; ++i)
        if (FULL || i < live) {
#pragma unroll
          for (int j = 0; j < WN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
        }
    };
    // Software pipeline.  sched_barrier(0) pins the order "fragment loads of the NEXT k-step, then
    // the MFMAs of the current one", so every LDS read has a whole MFMA block to complete in.  The
    // last k-step of a chunk runs after the barrier, overlapping the first fragment loads of the
    // next chunk and the issue of the global loads two chunks ahead.  The loop is rotated so that
    // its body starts at the barrier.
    auto step = [&](const char *st, int ks_next, int slot_next, int slot_now) {
      load_frags(st, ks_next, slot_next);
      __builtin_amdgcn_sched_barrier(0);
      mfma_step(slot_now);
      __builtin_amdgcn_sched_barrier(0);
    };
    issue_loads(0, 0);
    __syncthreads();  // waits for this wave's loads (vmcnt 0), then for everybody's
    if (KT > 1) issue_loads(1, 1);
    load_frags(smem, 0, 0);
    step(smem, 1, 1, 0);
    step(smem, 2, 0, 1);
    step(smem, 3, 1, 0);
    for (int kt = 1; kt < KT; ++kt) {
      // chunk kt has landed (mine: vmcnt 0; everybody's: barrier) and nobody reads the other stage any more
      __syncthreads();
      const char *st = smem + (kt & 1) * STAGE_BYTES;
      load_frags(st, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      mfma_step(1);  // last k-step of chunk kt-1; the global loads of chunk kt+1 are issued in its shadow
      if (kt + 1 < KT) issue_loads(kt + 1, (kt + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      step(st, 1, 1, 0);
      step(st, 2, 0, 1);
      step(st, 3, 1, 0);
    }
    mfma_step(1);
  };
  if (live == WM)
    k_loop(std::true_type{});
  else
    k_loop(std::false_type{});
  store_tile<WAVES_N, WM, WN, GATED, ACT>(acc, static_cast<uint16_t *>(P.Cout), rbase, rows_e, m0, n0, N, wm, wn, lane);
#endif
}

// Four-stage variant (K % 32 == 0): 32-element K chunks (64-byte LDS rows), a ring of four 32 KB
// stages, three chunks of global loads in flight.  With one chunk in flight the waves spend about
// half their time waiting for the slowest load of the chunk (an L2 miss takes longer than the MFMAs
// of one chunk); three chunks in flight cover it.  The waits are hand-counted: a wave issues NI
// buffer loads per chunk and they complete in order, so "all but the newest 2*NI loads are done"
// means that its part of the chunk about to be used has landed; the barrier extends that to every
// wave.  Past the last chunk the ring is fed with reloads of the last chunk so that the count stays
// uniform.  LDS rows are 64 B: chunk c of row r sits at position c ^ ((r >> 2) & 3), conflict-free
// for 16 consecutive rows on 64 banks.
template <int WAVES_M, int WAVES_N, int WM, int WN, bool GATED, int ACT>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_bf16_dl4_kernel(GemmArgs P) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int BM = WAVES_M * WM * 32;
  constexpr int BROWS = WAVES_N * WN * 32;
  constexpr int BN = GATED ? BROWS / 2 : BROWS;
  constexpr int BK = 32, ROWB = 64, NS = 4;
  constexpr int STAGE_BYTES = (BM + BROWS) * ROWB;
  constexpr int NI = (BM + BROWS) / 16 / NW;  // 1 KB load instructions per wave per chunk
  constexpr int NIA = BM / 16 / NW, NIB0 = BN / 16 / NW;
  static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "operand boundaries must fall between load instructions");
  static_assert(NI == 4, "the wait counts below assume four loads per wave per chunk");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  int mt, nt;
  if (!map_tile(blockIdx.x, *P.n_tiles, P.NT, mt, nt, P.map_mode)) return;
  const int e = P.tile_expert[mt];
  const int m0 = P.tile_row0[mt];
  const int rbase = P.row_base[e];
  const int rows_e = P.row_base[e + 1] - rbase;
  const int n0 = nt * BN;
  const int K = P.K, N = P.N;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w / WAVES_N, wn = w % WAVES_N;

  const char *Ab = static_cast<const char *>(P.A);
  const char *B0b = static_cast<const char *>(P.B0) + (size_t)e * N * K * 2;
  const char *B1b = GATED ? static_cast<const char *>(P.B1) + (size_t)e * N * K * 2 : B0b;
  const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char *>(Ab + (size_t)rbase * K * 2), 0, (int)min((size_t)rows_e * K * 2, (size_t)0x7fffffff), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsB0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(B0b), 0, N * K * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsB1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(B1b), 0, N * K * 2, 0x00020000);
  // instruction i of wave w fills stage rows [16 q, 16 q + 16), q = i * NW + w; lane -> row lane/4, position lane%4
  int voff[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int r = (i * NW + w) * 16 + (lane >> 2);
    const int c = (lane & 3) ^ ((r >> 2) & 3);
    int row;
    if (r < BM) {
      row = m0 + r;
    } else {
      int nr = r - BM;
      if (GATED && nr >= BN) nr -= BN;
      row = n0 + nr;
    }
    voff[i] = row * K * 2 + c * 16;
  }
  auto issue_loads = [&](int kt, int buf) {
    char *st = smem + buf * STAGE_BYTES + w * 1024;
    const int koff = kt * (BK * 2);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      auto lp = (__attribute__((address_space(3))) void *)(st + i * NW * 1024);
      if (i < NIA)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, lp, 16, voff[i], koff, 0, 0);
      else if (!GATED || i < NIA + NIB0)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB0, lp, 16, voff[i], koff, 0, 0);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB1, lp, 16, voff[i], koff, 0, 0);
    }
  };

  const int fr = lane & 31, fh = lane >> 5;
  const int sw = (fr >> 2) & 3;  // the same for every fragment: fragment rows start at multiples of 32
  int a_off[WM], b_off[WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) a_off[i] = ((wm * WM + i) * 32 + fr) * ROWB;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    int r;
    if (GATED) {
      constexpr int H = WN / 2;
      r = (j < H) ? (wn * H + j) * 32 + fr : BN + (wn * H + (j - H)) * 32 + fr;
    } else {
      r = (wn * WN + j) * 32 + fr;
    }
    b_off[j] = (BM + r) * ROWB;
  }

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int KT = K / BK;
  bf16x8 af[2][WM], bfr[2][WN];
  auto load_frags = [&](const char *st, int ks, int slot) {
    const int pos = ((2 * ks + fh) ^ sw) << 4;
#pragma unroll
    for (int i = 0; i < WM; ++i) af[slot][i] = *reinterpret_cast<const bf16x8 *>(st + a_off[i] + pos);
#pragma unroll
    for (int j = 0; j < WN; ++j) bfr[slot][j] = *reinterpret_cast<const bf16x8 *>(st + b_off[j] + pos);
  };
  auto mfma_step = [&](int slot) {
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
  };
  auto step = [&](const char *st, int ks_next, int slot_next, int slot_now) {
    load_frags(st, ks_next, slot_next);
    __builtin_amdgcn_sched_barrier(0);
    mfma_step(slot_now);
    __builtin_amdgcn_sched_barrier(0);
  };
  // chunk t lives in stage t % 4; chunks t+1, t+2 are in flight while chunk t is consumed
  issue_loads(0, 0);
  issue_loads(min(1, KT - 1), 1);
  issue_loads(min(2, KT - 1), 2);
  asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
  issue_loads(min(3, KT - 1), 3);
  load_frags(smem, 0, 0);
  step(smem, 1, 1, 0);
  for (int t = 1; t < KT; ++t) {
    // mine: all but the newest 8 loads done -> chunk t landed; all waves: barrier.  Stage (t-1) % 4
    // is free again once every wave is past this barrier (its fragment reads were waited for here).
    asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    issue_loads(min(t + 3, KT - 1), (t + 3) & 3);
    const char *st = smem + (t & 3) * STAGE_BYTES;
    step(st, 0, 0, 1);  // MFMAs: second k-step of chunk t-1
    step(st, 1, 1, 0);
  }
  // the ring's trailing reloads must have landed before this workgroup's LDS can be handed on
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  mfma_step(1);
  store_tile<WAVES_N, WM, WN, GATED, ACT>(acc, static_cast<uint16_t *>(P.Cout), rbase, rows_e, m0, n0, N, wm, wn, lane);
#endif
}

// ------------------------------------------------------------------ fp32 path
constexpr int GF_BM = 64, GF_BN = 64, GF_BK = 16, GF_LD = GF_BM + 4;

// ACT: -1 none, RR_ACT_GELU, RR_ACT_SWIGLU (gated: B0 = gate, B1 = up)
template <int ACT>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs P) {
  constexpr bool GATED = ACT == RR_ACT_SWIGLU;
  __shared__ float As[GF_BK][GF_LD], Bs0[GF_BK][GF_LD], Bs1[GATED ? GF_BK : 1][GF_LD];
  const int mt = blockIdx.x / P.NT;
  if (mt >= *P.n_tiles) return;
  const int e = P.tile_expert[mt];
  const int m0 = P.tile_row0[mt];
  const int rbase = P.row_base[e];
  const int rows_e = P.row_base[e + 1] - rbase;
  const int n0 = (blockIdx.x - mt * P.NT) * GF_BN;
  const int K = P.K, N = P.N;
  const float *A = static_cast<const float *>(P.A);
  const float *B0 = static_cast<const float *>(P.B0) + (size_t)e * N * K;
  const float *B1 = GATED ? static_cast<const float *>(P.B1) + (size_t)e * N * K : nullptr;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int lr = tid >> 2, lc = tid & 3;
  const float *a_src = A + (size_t)(rbase + min(m0 + lr, rows_e - 1)) * K + lc * 4;
  const size_t b_off = (size_t)min(n0 + lr, N - 1) * K + lc * 4;

  float g[4][4], u[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) { g[a][b] = 0.0f; u[a][b] = 0.0f; }

  for (int k0 = 0; k0 < K; k0 += GF_BK) {
    const bool in = k0 + lc * 4 < K;
    float4 va = in ? *reinterpret_cast<const float4 *>(a_src + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 vb = in ? *reinterpret_cast<const float4 *>(B0 + b_off + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
    As[lc * 4 + 0][lr] = va.x; As[lc * 4 + 1][lr] = va.y; As[lc * 4 + 2][lr] = va.z; As[lc * 4 + 3][lr] = va.w;
    Bs0[lc * 4 + 0][lr] = vb.x; Bs0[lc * 4 + 1][lr] = vb.y; Bs0[lc * 4 + 2][lr] = vb.z; Bs0[lc * 4 + 3][lr] = vb.w;
    if (GATED) {
      float4 vc = in ? *reinterpret_cast<const float4 *>(B1 + b_off + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
      Bs1[lc * 4 + 0][lr] = vc.x; Bs1[lc * 4 + 1][lr] = vc.y; Bs1[lc * 4 + 2][lr] = vc.z; Bs1[lc * 4 + 3][lr] = vc.w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GF_BK; ++kk) {
      float av[4], bv[4], cv[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) av[a] = As[kk][ty * 4 + a];
#pragma unroll
      for (int b = 0; b < 4; ++b) { bv[b] = Bs0[kk][tx * 4 + b]; cv[b] = GATED ? Bs1[kk][tx * 4 + b] : 0.0f; }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          g[a][b] = fmaf(av[a], bv[b], g[a][b]);
          if (GATED) u[a][b] = fmaf(av[a], cv[b], u[a][b]);
        }
    }
    __syncthreads();
  }
  float *Cf = static_cast<float *>(P.Cout);
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int row = m0 + ty * 4 + a;
    if (row >= rows_e) continue;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int col = n0 + tx * 4 + b;
      if (col >= N) continue;
      float c = g[a][b];
      if (ACT == RR_ACT_SWIGLU) c = c / (1.0f + expf(-c)) * u[a][b];
      if (ACT == RR_ACT_GELU) c = gelu_erf(c);
      Cf[(size_t)(rbase + row) * N + col] = c;
    }
  }
}

template <typename Kern>
hipError_t set_lds(Kern kern, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace

// Tile configuration: 2 x 4 waves, each 4 x 2 fragments of 32x32 -> 256 x 256 staged rows, two waves
// per SIMD so that one wave's LDS reads overlap the other's MFMAs.
#ifndef RR_GEMM_CFG
#define RR_GEMM_CFG 2, 4, 4, 2
#define RR_GEMM_THREADS 512
#define RR_GEMM_SWZ 1
#endif
#ifndef RR_GEMM_STAGES
#define RR_GEMM_STAGES 2
#endif

// which: bit 0 = up projection (+ activation), bit 1 = down projection
hipError_t launch_ffn_part(const Dims &D, const void *w1, const void *w3, const void *w2, const Work &W,
                           hipStream_t s, int which) {
  GemmArgs up{W.x_disp, w1, w3, W.h, D.d, D.F, 0, 0, W.row_base, W.tile_expert, W.tile_row0, W.n_tiles};
  GemmArgs down{W.h, w2, nullptr, W.y, D.F, D.d, 0, 0, W.row_base, W.tile_expert, W.tile_row0, W.n_tiles};
  hipError_t err = hipSuccess;
  if (D.dtype == RR_BF16) {
    // 256 x 256 staged rows; BM must equal Dims::BM (row tiles are cut by row_plan)
    constexpr int LDS = 2 * (256 + 256) * GB_ROW_BYTES;
    // direct-to-LDS kernels need whole 64-element K chunks; other sizes take the register-staged kernels
    const bool dl_up = D.d % GB_BK == 0, dl_dn = D.F % GB_BK == 0;
#if RR_GEMM_STAGES == 4
    auto k_up_gated = dl_up ? gemm_bf16_dl4_kernel<RR_GEMM_CFG, true, -1>
                            : gemm_bf16_kernel<RR_GEMM_CFG, true, -1, RR_GEMM_SWZ>;
    auto k_up_gelu = dl_up ? gemm_bf16_dl4_kernel<RR_GEMM_CFG, false, RR_ACT_GELU>
                           : gemm_bf16_kernel<RR_GEMM_CFG, false, RR_ACT_GELU, RR_GEMM_SWZ>;
    auto k_down = dl_dn ? gemm_bf16_dl4_kernel<RR_GEMM_CFG, false, -1>
                        : gemm_bf16_kernel<RR_GEMM_CFG, false, -1, RR_GEMM_SWZ>;
#else
    auto k_up_gated = dl_up ? gemm_bf16_dl_kernel<RR_GEMM_CFG, true, -1, RR_GEMM_SWZ>
                            : gemm_bf16_kernel<RR_GEMM_CFG, true, -1, RR_GEMM_SWZ>;
    auto k_up_gelu = dl_up ? gemm_bf16_dl_kernel<RR_GEMM_CFG, false, RR_ACT_GELU, RR_GEMM_SWZ>
                           : gemm_bf16_kernel<RR_GEMM_CFG, false, RR_ACT_GELU, RR_GEMM_SWZ>;
    auto k_down = dl_dn ? gemm_bf16_dl_kernel<RR_GEMM_CFG, false, -1, RR_GEMM_SWZ>
                        : gemm_bf16_kernel<RR_GEMM_CFG, false, -1, RR_GEMM_SWZ>;
#endif
    static bool attr_done = false;
    if (!attr_done) {
      if ((err = set_lds(gemm_bf16_dl4_kernel<RR_GEMM_CFG, true, -1>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_dl4_kernel<RR_GEMM_CFG, false, RR_ACT_GELU>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_dl4_kernel<RR_GEMM_CFG, false, -1>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_dl_kernel<RR_GEMM_CFG, true, -1, RR_GEMM_SWZ>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_dl_kernel<RR_GEMM_CFG, false, RR_ACT_GELU, RR_GEMM_SWZ>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_dl_kernel<RR_GEMM_CFG, false, -1, RR_GEMM_SWZ>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_kernel<RR_GEMM_CFG, true, -1, RR_GEMM_SWZ>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_kernel<RR_GEMM_CFG, false, RR_ACT_GELU, RR_GEMM_SWZ>, LDS)) != hipSuccess) return err;
      if ((err = set_lds(gemm_bf16_kernel<RR_GEMM_CFG, false, -1, RR_GEMM_SWZ>, LDS)) != hipSuccess) return err;
      attr_done = true;
    }
    up.NT = D.act == RR_ACT_SWIGLU ? (D.F + 127) / 128 : (D.F + 255) / 256;
    down.NT = (D.d + 255) / 256;
    up.map_mode = up.NT % GEMM_GN == 0 ? 2 : 0;
    down.map_mode = down.NT % GEMM_GN == 0 ? 2 : 0;
    const int g_up = up.map_mode == 2 ? gemm_grid(D.max_mtiles, up.NT) : D.max_mtiles * up.NT;
    const int g_dn = down.map_mode == 2 ? gemm_grid(D.max_mtiles, down.NT) : D.max_mtiles * down.NT;
    if (which & 1) {
      prof_begin(K_FFN_UP, s);
      if (D.act == RR_ACT_SWIGLU)
        k_up_gated<<<g_up, RR_GEMM_THREADS, LDS, s>>>(up);
      else
        k_up_gelu<<<g_up, RR_GEMM_THREADS, LDS, s>>>(up);
      prof_end(K_FFN_UP, s);
    }
    if (which & 2) {
      prof_begin(K_FFN_DOWN, s);
      k_down<<<g_dn, RR_GEMM_THREADS, LDS, s>>>(down);
      prof_end(K_FFN_DOWN, s);
    }
  } else {
    up.NT = (D.F + GF_BN - 1) / GF_BN;
    down.NT = (D.d + GF_BN - 1) / GF_BN;
    if (which & 1) {
      prof_begin(K_FFN_UP, s);
      if (D.act == RR_ACT_SWIGLU)
        gemm_f32_kernel<RR_ACT_SWIGLU><<<up.NT * D.max_mtiles, 256, 0, s>>>(up);
      else
        gemm_f32_kernel<RR_ACT_GELU><<<up.NT * D.max_mtiles, 256, 0, s>>>(up);
      prof_end(K_FFN_UP, s);
    }
    if (which & 2) {
      prof_begin(K_FFN_DOWN, s);
      gemm_f32_kernel<-1><<<down.NT * D.max_mtiles, 256, 0, s>>>(down);
      prof_end(K_FFN_DOWN, s);
    }
  }
  return hipGetLastError();
}

hipError_t launch_ffn(const Dims &D, const void *w1, const void *w3, const void *w2, const Work &W, hipStream_t s) {
  return launch_ffn_part(D, w1, w3, w2, W, s, 3);
}

}  // namespace rr
