// Internal declarations shared by the HIP translation units of librr.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rr.h"

namespace rr {

constexpr int kMaxE = 64;
constexpr int kMaxK = 4;
constexpr int kMaxRounds = kMaxK + 1;   // k top-k rounds + the Fill-in round
constexpr int kTokBlock = 128;          // tokens per workgroup in the per-token routing kernels
constexpr int kWave = 64;
// Selection lists (rr_dispatch.hip): up to kSelectRegMax candidates are one workgroup's registers;
// longer lists are cut into segments of kSelectSegLen candidates, one workgroup each, when the batch
// can hold such a list at all and the lists are few enough for the segment map (kept in LDS).
constexpr int kSelectRegMax = 24576;
constexpr int kSelectSegLen = 16384;
__host__ __device__ inline bool select_splits(long long T, int NR, int NL) {
  return T * NR > kSelectRegMax && NL <= 2048;
}

typedef uint32_t u32;

// Everything derived from rr_config on the host.
struct Dims {
  int T, d, F, E, k, G;
  int C;       // slots in an expert's queue (row length of slot_token)
  int Cq;      // slots of one capacity block: C, or with per-group quotas C / G
  int Gq;      // capacity blocks per expert: 1, or G with per-group quotas
  int quota;
  int Eg, Tg;
  int NR;      // routing rounds that place tokens: k (+1 with Fill-in)
  int NCAT;    // NR * E candidate arrays (one per round and expert, ascending token index)
  int NL;      // NCAT * Gq selection lists: list id = (round * E + expert) * Gq + block
  int NB;      // token blocks of kTokBlock
  int cb;      // candidate-count blocks per token block (1, or 4 when the small-batch router counts per 32 tokens)
  int NBc;     // candidate-count blocks: blk_cnt is [NCAT, NBc]
  int ir, fr, arrival;
  int dtype, act;
  int Rmax;        // upper bound on dispatched rows: min(E*C, NR*T) + (ir ? T : 0)
  int max_mtiles;  // upper bound on row tiles of the grouped GEMM
  int BM;          // row-tile height of the grouped GEMM for this dtype
};

// One row tile of the grouped GEMM: rows [row0, row0 + BM) of expert `expert`, whose dispatched rows
// start at `rbase` and number `rows` (`fill` occupied capacity slots, then the Intra-GPU rows, whose
// tokens start at ir_token[ir_offset]).
struct __attribute__((aligned(32))) TileInfo {
  int32_t expert, row0, rbase, rows, fill, ir_offset, pad0, pad1;
};

// Device pointers carved out of the caller's workspace.
struct Work {
  // routing
  u32     *key;          // [T, NR]   order-preserving key of the score of the r-th choice
  float   *ir_score;     // [T]       score of the best expert of the token's own group
  int32_t *ir_cand;      // [T]       that expert
  int32_t *blk_cnt;      // [NCAT, NBc] candidates per (list, count block); scanned in place
  int32_t *cat_cnt;      // [NCAT]    candidates per (round, expert)
  int32_t *grp_fill;     // [E, Gq]   occupied slots of each capacity block after the last round
  int32_t *grp_off;      // [E, Gq]   occupied slots of the expert's earlier blocks (its dispatched rows skip the holes)
  int32_t *row_token;    // [Rmax]    per-group quotas only: token of every dispatched row
  u32     *cand_key;     // [NR*T]    per-list candidates in ascending token index
  int32_t *cand_tok;     // [NR*T]
  u32     *comp_key;     // [NR*T]    split lists only: per segment, the candidates that may be kept, in order
  int32_t *comp_tok;     // [NR*T]
  int32_t *seg_cnt;      // [NL + NR*T / kSelectSegLen] how many of those every segment has
  int32_t *list_done;    // [NL]      segments of a list that have finished (tickets)
  int32_t *ir_blk_cnt;   // [E, NB]   Intra-GPU tokens per (expert, token block); scanned in place
  int32_t *ir_cnt;       // [E]
  int32_t *row_base;     // [E+1]     first dispatched row of each expert (slot rows, then IR rows)
  TileInfo *tiles;       // [max_mtiles] row tiles of the grouped GEMM
  int32_t *tile_ctl;     // [4] [0] = number of row tiles
  // forward only
  float   *logits;       // [T,E] when the caller passes none
  rr_tables tables;      // storage when the caller passes none
  int32_t *row_dest;     // [Rmax] token whose ONLY processed row this is (its output row is written by the down projection), else -1
  void    *x_disp;       // [Rmax, d]
  void    *h;            // [Rmax, F]
  void    *y;            // [Rmax, d]
};

struct Launch {
  hipStream_t stream;
};

// Kernel ids for the profiling record.
enum KernelId {
  K_ROUTER = 0, K_TOPK, K_SCAN_CAND, K_SCATTER_CAND, K_SELECT_SLOT,
  K_IR_COUNT, K_IR_SCAN, K_IR_WEIGHTS, K_GATHER, K_FFN_UP, K_FFN_DOWN, K_COMBINE, K_ROUTER_BWD,
  K_COUNT
};

void prof_begin(KernelId id, hipStream_t s);
void prof_end(KernelId id, hipStream_t s);

// Order-preserving map fp32 -> u32 (IEEE '>' on finite floats == '>' on keys; -0.0 and +0.0 share a key).
__host__ __device__ inline u32 score_key(float a) {
  u32 u = __builtin_bit_cast(u32, a);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__host__ __device__ inline float key_score(u32 key) {
  u32 u = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
  return __builtin_bit_cast(float, u);
}

// Stage launchers (each returns a hipError_t from the launches it made).
// With tb and W the router may also do the per-token ranking that the routing tables start from
// and launch_dispatch is told to skip that step.  The small-batch router counts candidates per 32
// tokens (its workgroup), the others per token block: router_count_blocks(D) = count blocks per token block.
int router_count_blocks(const Dims &D);
hipError_t launch_router(const Dims &D, const void *x, const float *w_router, const float *bias,
                         float *logits, float *probs, int32_t *rank_expert, const rr_tables *tb, const Work *W,
                         hipStream_t s);
// row_dest: only in the forward call (see Work::row_dest), else nullptr
hipError_t launch_dispatch(const Dims &D, const float *logits, const rr_tables &tb, const Work &W, bool ranked,
                           int32_t *row_dest, hipStream_t s);
hipError_t launch_gather(const Dims &D, const void *x, const rr_tables &tb, const Work &W, hipStream_t s);
hipError_t router_kernel_attributes();  // raises the dynamic-LDS limit of the streaming router on the current device
hipError_t ffn_kernel_attributes();     // raises the dynamic-LDS limit of the bf16 GEMM kernels on the current device
bool ffn_fuses_gather(const Dims &D);
bool ffn_writes_single_rows(const Dims &D);  // the down projection writes the output row of a token with one processed assignment itself  // the up projection reads x through the dispatch tables: no gather pass
hipError_t launch_ffn(const Dims &D, const void *x, const rr_tables &tb, const void *w1, const void *w3,
                      const void *w2, const Work &W, void *out, hipStream_t s);
hipError_t launch_combine(const Dims &D, const rr_tables &tb, const Work &W, void *out, hipStream_t s);
// reads the expert outputs, row bases and block offsets that the forward pass left in W
hipError_t launch_router_backward(const Dims &D, const void *dout, const float *logits, const rr_tables &tb,
                                  const Work &W, bool straight_through, float *dcombine_w, float *dlogits,
                                  hipStream_t s);

}  // namespace rr
