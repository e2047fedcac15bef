// Expert FFN as a grouped GEMM over the dispatched rows (Sec. 5.1: every expert is a LLaMA FFN):
//   up   : h[row, f] = silu(x[row] . W1_e[f]) * (x[row] . W3_e[f])      (SwiGLU)
//          h[row, f] = gelu(x[row] . W1_e[f])                            (GELU)
//   down : y[row, c] = h[row] . W2_e[c]
// Both are "A[rows,K] times B[N,K]^T" with K contiguous in both operands.  Rows of expert e are
// row_base[e] .. row_base[e+1]-1 and are cut into row tiles when the routing tables are built (TileInfo).
//
// bf16 main path (K % 64 == 0, K >= 192): persistent kernel, one workgroup of 8 waves per CU, tiles of
// 256 x 256 staged rows dealt in an XCD-aware panel order (see "Tile order" in the kernel).
//   * v_mfma_f32_32x32x16_bf16, fp32 accumulate; 2 x 4 waves, wave tile 128 x 64; two waves per SIMD
//     so that one wave's LDS reads overlap the other's MFMAs.
//   * K advances in chunks of 64 through LDS rings - two 32 KB stages of A, three of B, 160 KB in all
//     - filled by buffer_load ... lds (16 bytes per lane straight into LDS, no staging registers);
//     the chunks of a workgroup's successive tiles form one stream.  A wave instruction fills 1 KB = 8
//     consecutive LDS rows (lane l -> row l/8, chunk position l%8), so the swizzle is applied on the
//     global side: the lane fetches the chunk that belongs at its position.  Rows past the end of
//     an operand read as zero (buffer range check): ragged tiles need no masks on the load side.
//   * LDS rows are 128 B; chunk c of row r sits at position c ^ ((r >> 1) & 7): conflict-free for
//     the 16 lanes x 16 B that the 64-bank LDS serves per cycle, for the DMA writes as well.
//   * The K loop is software-pipelined by hand (see k_loop): the compiler's own schedule waits for
//     every LDS read right before its first use.
//   * The up projection can read its A rows straight from x through the dispatch tables (GATHER):
//     the dispatch gather is then a per-lane row offset of the LDS DMA and costs no pass over HBM.
//   * While a tile's epilogue stores drain, the first K chunk of the workgroup's next tile is
//     already in flight (its tile id and table entries were fetched during the K loop).
// Other bf16 shapes take a register-staged kernel; fp32 workloads a plain fp32 FMA tile kernel
// (the fp32 accuracy bar forbids bf16 products).
#include <type_traits>

#include "rr_device.h"

namespace rr {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Scheduling groups for the instruction scheduler (masks of sched_group_barrier: 0x008 MFMA,
// 0x100 LDS read, 0x020 global or buffer load).  They order the instructions of the surrounding
// scheduling region only; what the instructions compute is untouched.
// N times "one MFMA, then one LDS read":
template <int N>
__device__ __forceinline__ void sched_mfma_lds_read() {
  if constexpr (N > 0) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    sched_mfma_lds_read<N - 1>();
  }
}
// N times "one MFMA, then up to PER global loads":
template <int N, int PER>
__device__ __forceinline__ void sched_mfma_global_load() {
  if constexpr (N > 0) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x020, PER, 0);
    sched_mfma_global_load<N - 1, PER>();
  }
}

__device__ inline u32 f32_to_bf16_bits(float f) {
  u32 u = __builtin_bit_cast(u32, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ inline float silu(float g) { return g / (1.0f + __expf(-g)); }
// for results that are rounded to bf16 right away: hardware reciprocal (1 ulp) instead of a division
__device__ inline float silu_fast(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32), first value in the low half
__device__ inline u32 pack_bf16(float a, float b) {
  const f32x2_t f = {a, b};
  return __builtin_bit_cast(u32, __builtin_convertvector(f, bf16x2_t));
}
__device__ inline float gelu_erf(float g) { return 0.5f * g * (1.0f + erff(g * 0.70710678118654752f)); }

constexpr int GB_BK = 64;             // bf16 elements per K chunk = 128 B per LDS row
constexpr int GB_ROW_BYTES = 128;
[[maybe_unused]] constexpr u32 BUF_FLAGS = 0x00020000; // raw buffer descriptor word 3 (32-bit data format)

struct GemmArgs {
  const void *A;        // [rows, K] dispatched rows; with GATHER: x [T, K]
  const void *B0;       // [E, N, K]
  const void *B1;       // [E, N, K] gated only
  void *Cout;           // [rows, N]
  int K, N;
  int NT;               // column tiles
  const TileInfo *tiles;
  const int32_t *ctl;   // [0] number of row tiles
  // GATHER only
  const int32_t *slot_token, *ir_token;
  const int32_t *row_token;  // token of every dispatched row (per-group quotas), or NULL: rows are slots, then the Intra-GPU list
  int C;
  long long a_bytes;    // size of the A operand in bytes (buffer range of the gather)
  // DIRECT only (down projection): row_dest[row] = the token whose only processed row this is, else -1;
  // such a row is also stored as row row_dest[row] of Out, the layer's output (Eq. 2 with a single term)
  const int32_t *row_dest;
  void *Out;
};

// Epilogue shared by the bf16 kernels: activation, round to bf16, store (masked on edge tiles).
// Accumulator element v of a 32x32 fragment is row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
// GATED: fragments j < WN/2 are gate columns, j >= WN/2 the matching up columns.
template <int WM, int WN, bool GATED, int ACT>
__device__ inline void store_tile(f32x16 (&acc)[WM][WN], uint16_t *Cb, int rbase, int rows_e, int m0, int n0, int N,
                                  int wm, int wn, int lane) {
  constexpr int NJ = GATED ? WN / 2 : WN;  // output column fragments per wave
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

// Epilogue of the persistent kernel, which multiplies with the operands swapped (B fragment first):
// the 32x32 accumulator then holds the transposed tile, i.e. a lane owns ONE output row (lane % 32
// of the A fragment) and, per fragment, four groups of four consecutive columns
// (8 * (v / 4) + 4 * (lane / 32) + v % 4): four 8-byte stores per fragment instead of sixteen
// 2-byte ones.
// dest (DIRECT): per fragment row of this lane, the row of Ob that the same values are also stored to, or -1.
template <int WM, int WN, bool GATED, int ACT, bool DIRECT = false>
__device__ inline void store_tile_t(f32x16 (&acc)[WM][WN], uint16_t *Cb, int rbase, int rows_e, int m0, int n0, int N,
                                    int wm, int wn, int lane, const int *dest = nullptr, uint16_t *Ob = nullptr) {
  constexpr int NJ = GATED ? WN / 2 : WN;  // output column fragments per wave
  const int fr = lane & 31, fh = lane >> 5;
  const int wrow0 = m0 + wm * WM * 32, wcol0 = n0 + wn * NJ * 32;
  const bool cols_in = wcol0 + NJ * 32 <= N;  // N % 8 == 0: a group of four columns is inside or outside as a whole
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    const int row = wrow0 + i * 32 + fr;
    if (row >= rows_e) continue;
    uint16_t *prow = Cb + (size_t)(rbase + row) * N + wcol0 + 4 * fh;
    uint16_t *orow = nullptr;
    if (DIRECT && dest[i] >= 0) orow = Ob + (size_t)dest[i] * N + wcol0 + 4 * fh;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          c[u] = acc[i][j][4 * g + u];
          if (GATED) c[u] = silu_fast(c[u]) * acc[i][j + NJ][4 * g + u];
          if (ACT == RR_ACT_GELU) c[u] = gelu_erf(c[u]);
        }
        if (cols_in || wcol0 + j * 32 + 8 * g + 4 * fh < N) {
          const uint2 val = make_uint2(pack_bf16(c[0], c[1]), pack_bf16(c[2], c[3]));
          *reinterpret_cast<uint2 *>(prow + j * 32 + 8 * g) = val;
          if (DIRECT && orow) *reinterpret_cast<uint2 *>(orow + j * 32 + 8 * g) = val;
        }
      }
    }
  }
}

__device__ inline int swz(int r) { return (r >> 1) & 7; }

// Barrier that publishes LDS-DMA data.  Before it signals, a wave's own buffer_load ... lds must
// have written LDS - all of them but the youngest YOUNGER, which belong to a later chunk (memory
// instructions complete in order) - and its own fragment reads of the stage that is about to be
// refilled must have returned (lgkmcnt 0).  Spelled out in assembly: the compiler's barrier waits
// for what its memory model takes for LDS traffic only, and when it does drain vmcnt it drains all.
template <int YOUNGER>
__device__ inline void dma_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(YOUNGER) : "memory");
}

// ------------------------------------------------------------------ bf16, persistent, LDS DMA
constexpr int PK_WAVES_M = 2, PK_WAVES_N = 4, PK_WM = 4, PK_WN = 2;
constexpr int PK_NW = PK_WAVES_M * PK_WAVES_N;
constexpr int PK_THREADS = PK_NW * 64;
constexpr int PK_BM = PK_WAVES_M * PK_WM * 32;     // 256
constexpr int PK_BROWS = PK_WAVES_N * PK_WN * 32;  // 256 staged B rows
constexpr int PK_STAGE = (PK_BM + PK_BROWS) * GB_ROW_BYTES;  // one K chunk of A and B (the register-staged kernel)
constexpr int PK_LDS = 2 * PK_STAGE;
constexpr int PK_A_STAGE = PK_BM * GB_ROW_BYTES, PK_B_STAGE = PK_BROWS * GB_ROW_BYTES;
constexpr int PK_A_STAGES = 2, PK_B_STAGES = 3;
constexpr int PK_B_BASE = PK_A_STAGES * PK_A_STAGE;
constexpr int PK_SMEM = PK_B_BASE + PK_B_STAGES * PK_B_STAGE;  // 160 KB: all of a CU's LDS
[[maybe_unused]] constexpr int PK_NI = (PK_BM + PK_BROWS) / 8 / PK_NW;  // 1 KB load instructions per wave per chunk
[[maybe_unused]] constexpr int PK_NIA = PK_BM / 8 / PK_NW;

template <bool GATED, int ACT, bool GATHER, bool DIRECT = false>
__global__ __launch_bounds__(PK_THREADS) void gemm_bf16_persistent_kernel(GemmArgs P) {
#if defined(__HIP_DEVICE_COMPILE__)  // buffer-resource and LDS-DMA builtins exist in the device pass only
  constexpr int WM = PK_WM, WN = PK_WN, NW = PK_NW, BM = PK_BM, NI = PK_NI, NIA = PK_NIA;
  constexpr int BN = GATED ? PK_BROWS / 2 : PK_BROWS;
  constexpr int NIB0 = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "operand boundaries must fall between load instructions");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int K = P.K, N = P.N, NT = P.NT, KT = K / GB_BK;
  // Tile order.  Workgroups are dealt to the 8 XCDs round-robin (workgroup g runs on XCD g % 8) and
  // each XCD has its own L2.  The tiles are numbered panel by panel - panels of pm x pn neighbouring
  // tiles (4 row tiles x 8 column tiles for 32 workgroups per XCD), column panels first, ragged at the
  // right and bottom edges of the tile grid - and each run of pm * pn consecutive numbers goes to the
  // workgroups of one XCD: a chunk of an A row tile is then fetched into that L2 once for pn tiles
  // and a chunk of a B column tile once for pm, instead of once per tile, and consecutive rounds of
  // an XCD stay on the same rows of the same expert.
  const int MT = P.ctl[0], total = MT * NT;
  const int G = gridDim.x;
  const int nX = (G & 7) == 0 ? 8 : 1, S = G / nX;
  const int pn = (S & 7) == 0 ? 8 : 1, pm = S / pn;
  const int xcd = blockIdx.x % nX, slot = blockIdx.x / nX;
  const int PMf = MT / pm, PNf = NT / pn;  // full panel rows / columns
  // tile number k (panel order) -> linear index mt * NT + nt
  auto tile_at = [&](int k) {
    int qm = k / (pm * NT);
    if (qm > PMf) qm = PMf;
    const int r = k - qm * pm * NT, h = qm < PMf ? pm : MT - PMf * pm;
    int qn = r / (h * pn);
    if (qn > PNf) qn = PNf;
    const int r2 = r - qn * h * pn, wd = qn < PNf ? pn : NT - PNf * pn;
    const int dm = r2 / wd, dn = r2 - dm * wd;
    return (qm * pm + dm) * NT + qn * pn + dn;
  };
  // this workgroup's i-th tile is number (i * nX + xcd) * S + slot
  int kk = xcd * S + slot;
  const int kstep = nX * S;
  if (kk >= total) return;
  int L = tile_at(kk), L1 = -1, L2 = -1;  // this workgroup's current tile and the two after it
  if (kk + kstep < total) L1 = tile_at(kk + kstep);
  if (kk + 2 * kstep < total) L2 = tile_at(kk + 2 * kstep);
  kk += 2 * kstep;  // number of L2
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps LDS-DMA addressing scalar
  const int wm = w / PK_WAVES_N, wn = w % PK_WAVES_N;
  const int fr = lane & 31, fh = lane >> 5;

  // fragment addressing (the same for every tile): lane reads row (lane & 31), chunk 2*ks + (lane >> 5)
  int a_off[WM], b_off[WN];
  const int fsw = swz(fr);  // fragment rows start at multiples of 32, so the swizzle depends on fr only
#pragma unroll
  for (int i = 0; i < WM; ++i) a_off[i] = ((wm * WM + i) * 32 + fr) * GB_ROW_BYTES;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    int r;
    if (GATED) {
      constexpr int H = WN / 2;
      r = (j < H) ? (wn * H + j) * 32 + fr : BN + (wn * H + (j - H)) * 32 + fr;
    } else {
      r = (wn * WN + j) * 32 + fr;
    }
    b_off[j] = r * GB_ROW_BYTES;
  }

  // per-tile state.  A tile's table entry is fetched two tiles ahead and (GATHER) its token indices
  // one tile ahead, as plain vector loads issued right after a tile's first barrier: they complete
  // in the shadow of the K loop (whose next barrier is a whole K chunk of MFMAs away) and are only
  // touched after it, so no tile ever waits for a table lookup.
  struct Info { int e, m0, rbase, rows_e, fill_e, iroff_e, n0; };
  // Load addressing.  Instruction i of wave w fills stage rows [8 q, 8 q + 8), q = i * NW + w: lane l
  // fetches row 8 q + l / 8.  The swizzle of that row, ((8 q + l / 8) >> 1) & 7, does not depend on i
  // (8 NW is a multiple of 16), so a lane's offsets into one operand differ by a wave-uniform row
  // step from one instruction to the next: one register per operand (A gathered: one per
  // instruction), the step added when the load is issued.
  static_assert((8 * NW) % 16 == 0, "swizzle must not depend on the instruction index");
  constexpr int NVA = GATHER ? NIA : 1;
  // A tile keeps the base and range of its operands; the buffer descriptors are put together from
  // them when loads are issued, through readfirstlane: a descriptor that the register allocator has
  // parked in vector registers would otherwise be treated as divergent and every load wrapped in a
  // waterfall loop.
  struct Tile {
    int e, m0, rbase, rows_e, n0, live;
    int va[NVA], vb;
    unsigned long long pa, pb0, pb1;
    int na;
  };
  auto rsrc_of = [](unsigned long long base, int range) {
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)base);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(base >> 32));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<char *>(((unsigned long long)hi << 32) | lo), 0,
                                             __builtin_amdgcn_readfirstlane(range), BUF_FLAGS);
  };
  const int lrow = w * 8 + (lane >> 3);            // stage row of this lane in instruction 0
  const int lcol = ((lane & 7) ^ swz(lrow)) * 16;  // byte position of its 16-byte chunk in the global row
  const int rstep = NW * 8 * K * 2;                // bytes between the rows of consecutive instructions
  const char *Ab = static_cast<const char *>(P.A);
  auto raw_load = [&](int Lt, int4 &ra, int4 &rb) {
    const int4 *q = reinterpret_cast<const int4 *>(P.tiles + Lt / NT);
    ra = q[0];
    rb = q[1];
  };
  auto finalize = [&](int Lt, const int4 &ra, const int4 &rb) {
    Info f;
    f.e = __builtin_amdgcn_readfirstlane(ra.x);
    f.m0 = __builtin_amdgcn_readfirstlane(ra.y);
    f.rbase = __builtin_amdgcn_readfirstlane(ra.z);
    f.rows_e = __builtin_amdgcn_readfirstlane(ra.w);
    f.fill_e = __builtin_amdgcn_readfirstlane(rb.x);
    f.iroff_e = __builtin_amdgcn_readfirstlane(rb.y);
    f.n0 = (Lt % NT) * BN;
    return f;
  };
  // the dispatch gather (Sec. 3: tokens travel to their experts): the tokens behind this lane's A
  // rows - occupied capacity slots first, then the expert's Intra-GPU rows; -1 = padding
  // Every lane always loads (rows past the expert's end read a valid dummy and are masked when the
  // offsets are built): the number of memory instructions per tile is then fixed, which the counted
  // waits of the K loop rely on.
  auto lookup_tokens = [&](const Info &f, int (&tok)[NIA]) {
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
      const int lr = f.m0 + (i * NW + w) * 8 + (lane >> 3);  // row within the expert
      const int32_t *src = lr < f.fill_e ? P.slot_token + ((size_t)f.e * P.C + lr) : P.ir_token + (f.iroff_e + lr - f.fill_e);
      if (P.row_token) src = P.row_token + (f.rbase + lr);
      if (lr >= f.rows_e) src = P.slot_token;
      tok[i] = *src;
    }
  };
  auto make_tile = [&](const Info &f, const int (&tok)[NIA], Tile &t) {
    t.e = f.e; t.m0 = f.m0; t.rbase = f.rbase; t.rows_e = f.rows_e; t.n0 = f.n0;
    t.live = min(WM, max(0, (f.rows_e - f.m0 - wm * WM * 32 + 31) >> 5));
    const char *B0b = static_cast<const char *>(P.B0) + (size_t)f.e * N * K * 2;
    const char *B1b = GATED ? static_cast<const char *>(P.B1) + (size_t)f.e * N * K * 2 : B0b;
    if (GATHER) {
      t.pa = reinterpret_cast<unsigned long long>(Ab);
      t.na = (int)P.a_bytes;
    } else {
      t.pa = reinterpret_cast<unsigned long long>(Ab + (size_t)f.rbase * K * 2);
      t.na = (int)min((size_t)f.rows_e * K * 2, (size_t)0x7fffffff);
    }
    t.pb0 = reinterpret_cast<unsigned long long>(B0b);
    t.pb1 = reinterpret_cast<unsigned long long>(B1b);
    if (GATHER) {
#pragma unroll
      for (int i = 0; i < NVA; ++i) {
        const bool real = f.m0 + (i * NW + w) * 8 + (lane >> 3) < f.rows_e && tok[i] >= 0;
        t.va[i] = real ? tok[i] * K * 2 + lcol : 0x7ffffff0;  // padding: past the range, reads as zero
      }
    } else {
      t.va[0] = (f.m0 + lrow) * K * 2 + lcol;
    }
    t.vb = (f.n0 + lrow) * K * 2 + lcol;  // gate and up rows (GATED) sit at the same offsets of W1 and W3
  };
  // One K chunk of A (NIA instructions per wave) or of B (NIB) into a stage of its ring.
  constexpr int NIB = NI - NIA;
  auto issue_a = [&](const Tile &t, int kt, int stage) {
    char *st = smem + stage * PK_A_STAGE + w * 1024;
    const int koff = kt * (GB_BK * 2);
    const __amdgpu_buffer_rsrc_t rsA = rsrc_of(t.pa, t.na);
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
      auto lp = (__attribute__((address_space(3))) void *)(st + i * NW * 1024);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, lp, 16, GATHER ? t.va[i < NVA ? i : 0] : t.va[0] + i * rstep, koff, 0,
                                               0);
    }
  };
  auto issue_b = [&](const Tile &t, int kt, int stage) {
    char *st = smem + PK_B_BASE + stage * PK_B_STAGE + w * 1024;
    const int koff = kt * (GB_BK * 2);
    const __amdgpu_buffer_rsrc_t rsB0 = rsrc_of(t.pb0, N * K * 2), rsB1 = rsrc_of(t.pb1, N * K * 2);
#pragma unroll
    for (int i = 0; i < NIB; ++i) {
      // which weight matrix instruction i reads is known at compile time
      auto lp = (__attribute__((address_space(3))) void *)(st + i * NW * 1024);
      if (!GATED || i < NIB0)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB0, lp, 16, t.vb + i * rstep, koff, 0, 0);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB1, lp, 16, t.vb + (i - NIB0) * rstep, koff, 0, 0);
    }
  };
  auto next_b = [](int sb) { return sb == PK_B_STAGES - 1 ? 0 : sb + 1; };

  // LDS rings: A has two stages, B three (160 KB together).  The K chunks of a workgroup's tiles
  // form one stream (chunk KT of a tile is chunk 0 of its next tile).  While chunk c is multiplied,
  // A(c+1), B(c+1) and B(c+2) are in flight or landed: the weights, which stream from HBM, are
  // fetched two chunks ahead, the activations (mostly L2 hits: a row tile is shared by all column
  // tiles) one.  Each chunk issues A(c+1) and then B(c+2), so the barrier that publishes chunk c+1
  // waits for everything but the NIB youngest loads.  KT >= 3.
  f32x16 acc[WM][WN];
  Tile cur, nxt;
  Info info1{}, info2{};                              // table entries of this workgroup's next two tiles
  int4 ra2 = make_int4(0, 0, 0, 0), rb2 = ra2;        // raw table entry of the tile after next
  int tok1[NIA];        // token indices of the next tile's A rows
  int sa = 0, sb = 0;   // ring stages of the current chunk
  {
    int4 ra, rb;
    raw_load(L, ra, rb);
    const Info f0 = finalize(L, ra, rb);
    int tok0[NIA];
#pragma unroll
    for (int i = 0; i < NIA; ++i) tok0[i] = -1;
    if (GATHER) lookup_tokens(f0, tok0);
    make_tile(f0, tok0, cur);
    if (L1 >= 0) {
      raw_load(L1, ra, rb);
      info1 = finalize(L1, ra, rb);
    }
    issue_a(cur, 0, sa);
    issue_b(cur, 0, sb);
    issue_b(cur, 1, next_b(sb));
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NIB) : "memory");  // own A(0), B(0) have landed
  }
  while (true) {
    const bool have1 = L1 >= 0;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    // Everybody's A(0), B(0) have landed: each wave saw its own arrive before it stored the previous
    // tile's results, so the barrier itself waits for no memory operation (the stores and B(1) may
    // still be on their way).
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // table lookups for the tiles to come, issued before this chunk's loads so that they are older
    // than anything a counted wait lets pass
    if (GATHER) lookup_tokens(info1, tok1);
    raw_load(L2 >= 0 ? L2 : L, ra2, rb2);
    int dest[WM];  // DIRECT: where the rows that this lane will store also go (this tile's, used in its epilogue)
#pragma unroll
    for (int i = 0; i < WM; ++i) {
      dest[i] = -1;
      if (DIRECT) {
        const int row = cur.m0 + (wm * WM + i) * 32 + fr;
        dest[i] = P.row_dest[cur.rbase + min(row, cur.rows_e - 1)];
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    issue_a(cur, 1, sa ^ 1);
    issue_b(cur, 2, next_b(next_b(sb)));

    // Ragged row tiles: the last tile of an expert is mostly padding.  A wave skips the fragment
    // loads and MFMAs of its 32-row fragments that lie wholly past the expert's last row (a
    // wave-uniform test), so a padded tile costs MFMA time in proportion to its real rows.  Full
    // tiles take a branch-free copy of the loop (FULL), which keeps its counted LDS waits exact.
    const int live = cur.live;
    auto k_loop = [&](auto full_tag) {
      constexpr bool FULL = decltype(full_tag)::value;
      bf16x8 af[2][WM], bfr[2][WN];
      auto load_frags = [&](const char *sta, const char *stb, int ks, int slot) {
        const int pos = ((2 * ks + fh) ^ fsw) << 4;
#pragma unroll
        for (int i = 0; i < WM; ++i)
          if (FULL || i < live) af[slot][i] = *reinterpret_cast<const bf16x8 *>(sta + a_off[i] + pos);
        if (FULL || live > 0) {
#pragma unroll
          for (int j = 0; j < WN; ++j) bfr[slot][j] = *reinterpret_cast<const bf16x8 *>(stb + b_off[j] + pos);
        }
      };
      auto mfma_step = [&](int slot) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
          if (FULL || i < live) {
#pragma unroll
            for (int j = 0; j < WN; ++j)
              // B fragment first: the accumulator holds the transposed tile (see store_tile_t)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
          }
      };
      // Software pipeline: the fragment loads of the NEXT k-step are spread over the MFMAs of the
      // current one, one LDS read behind each of the first MFMAs.  (With all the reads in front
      // of the MFMAs the LDS pipe is asked for 6 KB per wave in one burst and is then idle for the
      // rest of the step; both waves of a SIMD doing so in turn leaves MFMA slots empty.)  The
      // last k-step of a chunk runs after the barrier; the global loads of the stream go behind
      // its last two MFMAs.  The loop is rotated so that its body starts at the barrier (the
      // compiler's wait counting is exact only inside one basic block).
      auto step = [&](const char *sta, const char *stb, int ks_next, int slot_next, int slot_now) {
        load_frags(sta, stb, ks_next, slot_next);
        mfma_step(slot_now);
        sched_mfma_lds_read<WM + WN>();
        __builtin_amdgcn_sched_barrier(0);
      };
      const char *sta = smem + sa * PK_A_STAGE, *stb = smem + PK_B_BASE + sb * PK_B_STAGE;
      load_frags(sta, stb, 0, 0);
      step(sta, stb, 1, 1, 0);
      step(sta, stb, 2, 0, 1);
      step(sta, stb, 3, 1, 0);
      // The looked-up values are consumed here, unconditionally, rather than where they are first
      // needed: in straight-line code after the lookups the compiler's wait for them is a counted
      // one (the A(1) and B(2) loads behind them stay in flight), and nothing it tracks is pending
      // when the loop is entered or the tile ends - there it would drain every outstanding load
      // and store.  Without a next tile the values are unused.
      make_tile(info1, tok1, nxt);
      info2 = finalize(L2 >= 0 ? L2 : L, ra2, rb2);
      if (DIRECT) {  // consumed here like the other lookups, so that no load is pending when the loop is entered
#pragma unroll
        for (int i = 0; i < WM; ++i) asm volatile("" : "+v"(dest[i]));
      }
      for (int kt = 1; kt < KT; ++kt) {
        // A(kt) and B(kt) have landed - the B issued after A(kt) may still be on its way - and
        // nobody reads the stages of chunk kt-1 any more
        if (kt + 1 < KT || have1) dma_barrier<NIB>();
        else dma_barrier<0>();
        sa ^= 1;
        sb = next_b(sb);
        sta = smem + sa * PK_A_STAGE;
        stb = smem + PK_B_BASE + sb * PK_B_STAGE;
        load_frags(sta, stb, 0, 0);
        mfma_step(1);  // last k-step of chunk kt-1
        sched_mfma_lds_read<WM + WN>();
        sched_mfma_global_load<2, 8>();
        // the stream's next loads: the rest of this tile, then the first two chunks of the next one
        if (kt + 2 < KT) {
          issue_a(cur, kt + 1, sa ^ 1);
          issue_b(cur, kt + 2, next_b(next_b(sb)));
        } else if (kt + 2 == KT) {
          issue_a(cur, kt + 1, sa ^ 1);
          if (have1) issue_b(nxt, 0, next_b(next_b(sb)));
        } else if (have1) {
          issue_a(nxt, 0, sa ^ 1);
          issue_b(nxt, 1, next_b(next_b(sb)));
        }
        __builtin_amdgcn_sched_barrier(0);
        step(sta, stb, 1, 1, 0);
        step(sta, stb, 2, 0, 1);
        step(sta, stb, 3, 1, 0);
      }
      mfma_step(1);
    };
    if (live == WM)
      k_loop(std::true_type{});
    else
      k_loop(std::false_type{});

    // own A(0), B(0) of the next tile have landed (they were issued one and two chunks ago), before
    // the stores below join the queue of outstanding memory operations
    if (have1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NIB) : "memory");
    sa ^= 1;
    sb = next_b(sb);
    store_tile_t<WM, WN, GATED, ACT, DIRECT>(acc, static_cast<uint16_t *>(P.Cout), cur.rbase, cur.rows_e, cur.m0, cur.n0,
                                             N, wm, wn, lane, dest, static_cast<uint16_t *>(P.Out));
    if (!have1) break;
    cur = nxt;
    L = L1;
    L1 = L2;
    kk += kstep;
    L2 = kk < total ? tile_at(kk) : -1;
    info1 = info2;
  }
#endif
}

// ------------------------------------------------------------------ bf16, any K % 8 == 0
// Register-staged loads (global -> registers -> LDS), 4 waves, tile 256 x 256 staged rows, one
// workgroup per tile.  Handles K tails by zero-filling whole 16-byte chunks.
constexpr int GS_THREADS = 256;
template <bool GATED, int ACT>
__global__ __launch_bounds__(GS_THREADS) void gemm_bf16_staged_kernel(GemmArgs P) {
  constexpr int WAVES_N = 2, WM = 4, WN = 4;
  constexpr int BM = 256, BROWS = 256;
  constexpr int BN = GATED ? BROWS / 2 : BROWS;
  constexpr int A_LD = BM / 32, B_LD = BROWS / 32;  // 16-byte loads per thread per chunk
  constexpr int STAGE_BYTES = (BM + BROWS) * GB_ROW_BYTES;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int mt = blockIdx.x / P.NT;
  if (mt >= P.ctl[0]) return;
  const TileInfo ti = P.tiles[mt];
  const int e = ti.expert, m0 = ti.row0, rbase = ti.rbase, rows_e = ti.rows;
  const int n0 = (blockIdx.x - mt * P.NT) * BN;
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
    int r = (tid >> 3) + 32 * i;
    int gr = min(m0 + r, rows_e - 1);
    a_src[i] = Ab + ((size_t)(rbase + gr) * K + lc * 8) * 2;
    lds_off_a[i] = r * GB_ROW_BYTES + ((lc ^ swz(r)) << 4);
  }
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    int r = (tid >> 3) + 32 * i;
    const char *bb = B0b;
    int nr = r;
    if (GATED && r >= BN) { bb = B1b; nr = r - BN; }
    int gn = min(n0 + nr, N - 1);
    b_src[i] = bb + ((size_t)gn * K + lc * 8) * 2;
    lds_off_b[i] = BM * GB_ROW_BYTES + r * GB_ROW_BYTES + ((lc ^ swz(r)) << 4);
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

  const int fr = lane & 31, fh = lane >> 5;
  const int fsw = swz(fr);
  int a_row_off[WM], b_row_off[WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) a_row_off[i] = ((wm * WM + i) * 32 + fr) * GB_ROW_BYTES;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    int r;
    if (GATED) {
      constexpr int H = WN / 2;
      r = (j < H) ? (wn * H + j) * 32 + fr : BN + (wn * H + (j - H)) * 32 + fr;
    } else {
      r = (wn * WN + j) * 32 + fr;
    }
    b_row_off[j] = (BM + r) * GB_ROW_BYTES;
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
      const int pos = ((2 * ks + fh) ^ fsw) << 4;
#pragma unroll
      for (int i = 0; i < WM; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(st + a_row_off[i] + pos);
#pragma unroll
      for (int j = 0; j < WN; ++j) bfr[j] = *reinterpret_cast<const bf16x8 *>(st + b_row_off[j] + pos);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds((kt + 1) & 1);
    __syncthreads();
  }
  store_tile<WM, WN, GATED, ACT>(acc, static_cast<uint16_t *>(P.Cout), rbase, rows_e, m0, n0, N, wm, wn, lane);
}

// ------------------------------------------------------------------ fp32 path
constexpr int GF_BM = 64, GF_BN = 64, GF_BK = 16, GF_LD = GF_BM + 4;

// ACT: -1 none, RR_ACT_GELU, RR_ACT_SWIGLU (gated: B0 = gate, B1 = up)
template <int ACT>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs P) {
  constexpr bool GATED = ACT == RR_ACT_SWIGLU;
  __shared__ float As[GF_BK][GF_LD], Bs0[GF_BK][GF_LD], Bs1[GATED ? GF_BK : 1][GF_LD];
  const int mt = blockIdx.x / P.NT;
  if (mt >= P.ctl[0]) return;
  const TileInfo ti = P.tiles[mt];
  const int e = ti.expert, m0 = ti.row0, rbase = ti.rbase, rows_e = ti.rows;
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

int cu_count() {
  static const int n = [] {  // initialised once, thread-safe (C++11 static)
    int dev = 0, cus = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
    return cus > 0 ? cus : 256;
  }();
  return n;
}

bool persistent_ok(int K) { return K % GB_BK == 0 && K >= 3 * GB_BK; }  // whole K chunks, at least three

}  // namespace

// The bf16 kernels use more dynamic LDS than the default limit.  Raising it is host-side set-up of the
// loaded code object on the current device (no stream work); the caller runs it once per device.
hipError_t ffn_kernel_attributes() {
  hipError_t e = hipSuccess;
  auto set = [&e](auto kern, int bytes) {
    if (e == hipSuccess) e = set_lds(kern, bytes);
  };
  set(gemm_bf16_persistent_kernel<true, -1, true>, PK_SMEM);
  set(gemm_bf16_persistent_kernel<true, -1, false>, PK_SMEM);
  set(gemm_bf16_persistent_kernel<false, RR_ACT_GELU, true>, PK_SMEM);
  set(gemm_bf16_persistent_kernel<false, RR_ACT_GELU, false>, PK_SMEM);
  set(gemm_bf16_persistent_kernel<false, -1, false>, PK_SMEM);
  set(gemm_bf16_persistent_kernel<false, -1, false, true>, PK_SMEM);
  set(gemm_bf16_staged_kernel<true, -1>, PK_LDS);
  set(gemm_bf16_staged_kernel<false, RR_ACT_GELU>, PK_LDS);
  set(gemm_bf16_staged_kernel<false, -1>, PK_LDS);
  return e;
}

bool ffn_writes_single_rows(const Dims &D) { return D.dtype == RR_BF16 && persistent_ok(D.F); }

bool ffn_fuses_gather(const Dims &D) {
  return D.dtype == RR_BF16 && persistent_ok(D.d) && (long long)D.T * D.d * 2 < 0x7ffffff0ll;
}

// which: bit 0 = up projection (+ activation), bit 1 = down projection
hipError_t launch_ffn_part(const Dims &D, const void *x, const rr_tables &tb, const void *w1, const void *w3,
                           const void *w2, const Work &W, void *out, hipStream_t s, int which) {
  const bool fuse = ffn_fuses_gather(D);
  GemmArgs up{fuse ? x : W.x_disp, w1, w3, W.h, D.d, D.F, 0, W.tiles, W.tile_ctl,
              tb.slot_token, tb.ir_token, D.quota ? W.row_token : nullptr, D.C, (long long)D.T * D.d * 2, nullptr, nullptr};
  GemmArgs down{W.h, w2, nullptr, W.y, D.F, D.d, 0, W.tiles, W.tile_ctl, nullptr, nullptr, nullptr, 0, 0, W.row_dest, out};
  if (D.dtype == RR_BF16) {
    const bool gated = D.act == RR_ACT_SWIGLU;
    up.NT = gated ? (D.F + 127) / 128 : (D.F + 255) / 256;
    down.NT = (D.d + 255) / 256;
    const int cus = cu_count();
    if (which & 1) {
      prof_begin(K_FFN_UP, s);
      if (persistent_ok(D.d)) {
        if (gated && fuse) gemm_bf16_persistent_kernel<true, -1, true><<<cus, PK_THREADS, PK_SMEM, s>>>(up);
        else if (gated) gemm_bf16_persistent_kernel<true, -1, false><<<cus, PK_THREADS, PK_SMEM, s>>>(up);
        else if (fuse) gemm_bf16_persistent_kernel<false, RR_ACT_GELU, true><<<cus, PK_THREADS, PK_SMEM, s>>>(up);
        else gemm_bf16_persistent_kernel<false, RR_ACT_GELU, false><<<cus, PK_THREADS, PK_SMEM, s>>>(up);
      } else {
        if (gated) gemm_bf16_staged_kernel<true, -1><<<up.NT * D.max_mtiles, GS_THREADS, PK_LDS, s>>>(up);
        else gemm_bf16_staged_kernel<false, RR_ACT_GELU><<<up.NT * D.max_mtiles, GS_THREADS, PK_LDS, s>>>(up);
      }
      prof_end(K_FFN_UP, s);
    }
    if (which & 2) {
      prof_begin(K_FFN_DOWN, s);
      if (persistent_ok(D.F)) gemm_bf16_persistent_kernel<false, -1, false, true><<<cus, PK_THREADS, PK_SMEM, s>>>(down);
      else gemm_bf16_staged_kernel<false, -1><<<down.NT * D.max_mtiles, GS_THREADS, PK_LDS, s>>>(down);
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

hipError_t launch_ffn(const Dims &D, const void *x, const rr_tables &tb, const void *w1, const void *w3,
                      const void *w2, const Work &W, void *out, hipStream_t s) {
  return launch_ffn_part(D, x, tb, w1, w3, w2, W, out, s, 3);
}

}  // namespace rr
