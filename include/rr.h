/*
 * rr.h - C ABI of the Rectify-Router MoE-layer forward for AMD MI355X (gfx950).
 *
 * The operations are those of "Turn Waste into Worth: Rectifying Top-k Router of MoE"
 * (arXiv 2402.12399): the top-k router with a fixed expert capacity (Sec. 3, Eq. 1, Eq. 2),
 * Intra-GPU Rectification of dropped tokens (Sec. 4.1, Eq. 3) and Fill-in Rectification of
 * padding slots (Sec. 4.2), followed by the expert FFNs (Sec. 5.1 "Model") and the linear
 * combination of their outputs (Eq. 2 / Eq. 3).  Everything runs on ONE GPU: the paper's
 * expert-parallel GPUs are simulated as G contiguous groups of experts and of tokens
 * (expert j lives on group j / (E/G), token i on group i / (T/G)); the token all-to-all of
 * expert parallelism (Sec. 3) is a permutation in device memory.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates no
 *     device memory and keeps no DATA between calls; scratch comes from `workspace` (one entry
 *     point, rr_rectified_dispatch_static, uses a fixed buffer inside the library instead).
 *     Process state it does keep: per device, whether rr_init has run (kernel attributes, the
 *     address of the static scratch buffer) - set once, thread-safe - and the record of the
 *     benchmarking profiler (rr_profile_*, one thread only).
 *   - Thread safety: calls from several host threads are safe as long as they do not share a
 *     workspace or output buffers (and do not use the profiler or the static scratch buffer).
 *   - Graph capture: every call only enqueues kernels on `stream` (no allocation, no memset, no
 *     synchronisation) and may be captured in a HIP graph, provided rr_init() has run on that
 *     device before the capture starts (the first call on a device otherwise runs it itself,
 *     which is host-side set-up that does not belong in a capture).
 *   - `stream` is a hipStream_t (NULL = the null stream).  Calls enqueue work and return
 *     without waiting for it.
 *   - Return value: RR_OK (0) or a negative rr_status; rr_strerror() names it.  Arguments are
 *     validated on the host before anything is launched; no call aborts or throws.
 *   - Matrices are dense, row-major, without padding.  int32 tables use -1 for "none".
 *   - Logits must be finite; behaviour for NaN/Inf logits is undefined.
 *   - Limits: 1 <= E <= 64, 1 <= k <= 4, T <= 2^24, d_model % 8 == 0, d_ff % 8 == 0, and with
 *     RR_QUOTA_PER_GROUP (T/G) % 128 == 0; with bf16 expert FFNs, (C + T) * max(d_model, d_ff) and
 *     d_model * d_ff below 2^30 elements (one expert's rows and one weight matrix are addressed with
 *     32-bit byte offsets); outside them calls return RR_ERR_UNSUPPORTED.
 */
#ifndef RR_H
#define RR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rr_status {
  RR_OK = 0,
  RR_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive size, E % G, T % G, k > E, Fill-in with k+1 > E */
  RR_ERR_UNSUPPORTED = -2, /* dtype / activation / size outside the limits above */
  RR_ERR_WORKSPACE   = -3, /* workspace NULL, misaligned (256 B) or smaller than rr_workspace_bytes */
  RR_ERR_HIP         = -4, /* a HIP call or kernel launch failed */
  RR_ERR_TOO_LARGE   = -5  /* rr_rectified_dispatch_static: the configuration needs more scratch than
                              RR_STATIC_WORKSPACE_BYTES */
} rr_status;

enum { RR_F32 = 0, RR_BF16 = 1 };             /* rr_config.dtype */
enum { RR_ACT_GELU = 0, RR_ACT_SWIGLU = 1 };  /* rr_config.act   */
enum {                                        /* rr_config.flags */
  RR_INTRA_GPU      = 1u, /* Sec. 4.1: re-route every dropped token inside its own group          */
  RR_FILL_IN        = 2u, /* Sec. 4.2: fill padding slots with the best (k+1)-th-choice tokens     */
  RR_POLICY_ARRIVAL = 4u, /* overflowing experts keep the EARLIEST tokens instead of the
                             highest-scoring ones (Sec. 3 says lowest scores are dropped; the
                             queue picture of Fig. 1 suggests arrival order).  Fill-in always
                             selects by score (Sec. 4.2).                                          */
  RR_QUOTA_PER_GROUP = 8u /* the capacity formula of Sec. 3 read per GPU, as expert-parallel
                             implementations do: every group g owns Cq = rr_capacity(T/G, E, cf)
                             slots of every expert - slots [g Cq, (g+1) Cq) of a queue of G Cq -
                             and only its own tokens compete for them, in the top-k rounds and
                             in Fill-in.  Default: one queue of C slots per expert for all T
                             tokens (Fig. 1).  Requires (T/G) % 128 == 0.                         */
};

/* Problem statement of Sec. 3: T tokens, E experts with router embeddings, top-k, capacity factor,
 * experts spread uniformly over G GPUs. */
typedef struct rr_config {
  int32_t  T;               /* tokens in the batch                                                */
  int32_t  d_model;         /* hidden size of a token                                             */
  int32_t  d_ff;            /* expert FFN inner size (ignored by the routing-only entry points)   */
  int32_t  E;               /* experts                                                            */
  int32_t  k;               /* experts per token                                                  */
  int32_t  G;               /* simulated expert-parallel groups ("GPUs"); E % G == 0, T % G == 0  */
  float    capacity_factor; /* capacity C = rr_capacity(T, E, capacity_factor)                    */
  int32_t  dtype;           /* RR_F32 | RR_BF16: type of x, expert weights and out; router fp32   */
  int32_t  act;             /* RR_ACT_SWIGLU: W2 (silu(W1 x) * (W3 x)); RR_ACT_GELU: W2 gelu(W1 x) */
  uint32_t flags;           /* RR_INTRA_GPU | RR_FILL_IN | RR_POLICY_ARRIVAL | RR_QUOTA_PER_GROUP */
} rr_config;

/* Routing, rectification and dispatch tables.  All device pointers, caller-allocated, every one
 * required.  C = rr_slots_per_expert(cfg): rr_capacity(T, E, cf), or G Cq with RR_QUOTA_PER_GROUP.
 * Column r < k of the [T,k+1] tables is the token's r-th choice (Eq. 1), column k its (k+1)-th
 * choice, the Fill-in nomination (Sec. 4.2 stage 1; -1 if k == E). */
typedef struct rr_tables {
  int32_t *rank_expert; /* [T,k+1] experts by descending score, ties -> lower expert index         */
  int32_t *slot;        /* [T,k+1] slot in that expert's queue, -1 = dropped / not filled in       */
  int32_t *slot_token;  /* [E,C]   token in each capacity slot, -1 = padding.  Kept tokens of a
                                   round take consecutive slots in ascending token index; rounds
                                   0..k-1 first, Fill-in last (with quotas: inside each group's
                                   block of Cq slots)                                              */
  int32_t *fill_topk;   /* [E]     occupied slots after the k top-k rounds (all groups together)   */
  int32_t *fill_total;  /* [E]     occupied slots after Fill-in (all groups together)              */
  int32_t *ir_expert;   /* [T]     Intra-GPU expert h_i of a token dropped >= once, else -1        */
  int32_t *ir_row;      /* [T]     position of the token in ir_expert's Intra-GPU list, else -1    */
  int32_t *ir_offset;   /* [E+1]   CSR offsets of the per-expert Intra-GPU lists in ir_token       */
  int32_t *ir_token;    /* [T]     lists concatenated by expert, ascending token index inside;
                                   only the first ir_offset[E] entries are written                 */
  float   *combine_w;   /* [T,k+2] Eq. 2 / Eq. 3 weights: columns 0..k-1 top-k ranks, k Fill-in,
                                   k+1 Intra-GPU; 0 where unused; a row of zeros = token not
                                   processed by any expert                                         */
} rr_tables;

/* Alignment: x, the expert weights, out, dout, w_router, logits and probs must be 16-byte aligned
 * (rows are moved with 16-byte vector instructions), every other array 4-byte aligned, the workspace
 * 256-byte aligned; a misaligned pointer is RR_ERR_INVALID_ARG (workspace: RR_ERR_WORKSPACE). */

/* One-time, per-device host-side set-up for the current device: raises the dynamic-LDS limit of the
 * grouped-GEMM kernels and looks up the address of the static scratch buffer.  Idempotent and
 * thread-safe.  Every entry point runs it on its first call on a device; call it explicitly before
 * capturing calls in a HIP graph.  Returns RR_OK or RR_ERR_HIP. */
int rr_init(void);

/* Sec. 3: capacity = capacity factor x tokens / experts, rounded up, at least 1.
 * Evaluated as ceil((double)cf * T / E).  Host function; returns -1 on invalid arguments. */
int32_t rr_capacity(int32_t T, int32_t E, float capacity_factor);

/* Slots in an expert's queue = row length of rr_tables.slot_token: rr_capacity(T, E, cf), or
 * G * rr_capacity(T/G, E, cf) with RR_QUOTA_PER_GROUP.  Host function; -1 on invalid arguments. */
int32_t rr_slots_per_expert(const rr_config *cfg);

/* Bytes of scratch that rr_rectified_dispatch and rr_moe_forward need for this configuration
 * (the larger of the two; a multiple of 256).  Host function. */
int rr_workspace_bytes(const rr_config *cfg, size_t *bytes);

/* Eq. 1 scores and argtopk; App. A Eq. 5 softmax over all experts.
 *   x           [T,d_model] of cfg->dtype (bf16 or fp32)
 *   w_router    [E,d_model] fp32, the expert embeddings w_j
 *   bias        [E] fp32 added to every row of scores, or NULL
 *   logits      [T,E] fp32 out: a_ij = w_j . x_i (+ bias_j), accumulated in fp32
 *   probs       [T,E] fp32 out or NULL
 *   rank_expert [T,k+1] int32 out or NULL
 */
int rr_router_scores(const rr_config *cfg, const void *x, const float *w_router, const float *bias,
                     float *logits, float *probs, int32_t *rank_expert, void *stream);

/* Sec. 3 capacity-limited top-k slotting, Sec. 4.1 and Sec. 4.2 rectifications, Eq. 2 / Eq. 3
 * weights: logits [T,E] -> every table of rr_tables.  The ranking is re-derived from `logits`, so
 * that they are the only data input.  All score comparisons use the fp32 logits (-0.0 == +0.0);
 * integer tables are a deterministic function of the logits. */
int rr_rectified_dispatch(const rr_config *cfg, const float *logits, const rr_tables *out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* rr_rectified_dispatch for callers that cannot allocate device memory or size a workspace - code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs and results; the scratch is a buffer of RR_STATIC_WORKSPACE_BYTES that lives in the
 * library's device image (one copy per GPU the library runs on, held until the process ends).  The
 * call allocates nothing.  A configuration whose rr_workspace_bytes (with d_ff = 0) exceeds
 * RR_STATIC_WORKSPACE_BYTES is refused with RR_ERR_TOO_LARGE before anything is launched (at
 * k = 2 with Fill-in and 64 experts that is about 440 K tokens).  All calls on one GPU share
 * that GPU's buffer: calls that overlap on one GPU - two streams, two host threads - race; issue
 * them on one stream.  Nothing in the buffer needs to start at zero (every kernel writes what the
 * next one reads), so the contents left by an earlier call do not matter. */
#define RR_STATIC_WORKSPACE_BYTES (32u << 20)
int rr_rectified_dispatch_static(const rr_config *cfg, const float *logits, const rr_tables *out, void *stream);

/* The whole layer: router -> slotting -> rectifications -> dispatch gather -> per-expert FFN
 * (grouped GEMM) -> weighted combine (Eq. 2 / Eq. 3).
 *   w1 [E,d_ff,d_model], w3 [E,d_ff,d_model] (SwiGLU only, else NULL), w2 [E,d_model,d_ff]: cfg->dtype
 *   out [T,d_model] cfg->dtype; the row of a token that no expert processes is 0 (its value is
 *       carried by the transformer block's residual connection, Sec. 3)
 *   tables: NULL, or tables to fill as rr_rectified_dispatch does
 *   logits: NULL, or [T,E] fp32 out
 * With cfg->d_ff == 0 the call stops after the tables (routing only: router and ranking fused, the
 * logits are not read back): tables and logits are then required, w1, w3, w2 and out are ignored.
 */
int rr_moe_forward(const rr_config *cfg, const void *x, const float *w_router, const float *bias,
                   const void *w1, const void *w3, const void *w2, void *out,
                   const rr_tables *tables, float *logits,
                   void *workspace, size_t workspace_bytes, void *stream);

/* App. A: gradient of a loss L with respect to the router scores through the weights of Eq. 2 /
 * Eq. 3, after an rr_moe_forward call with the same cfg (d_ff > 0) and the same workspace, which
 * must not have been written since: the expert outputs E_j(x_i) and the row layout are read from it.
 * The routing decisions carry no gradient.
 *   dout       [T,d_model] cfg->dtype: dL/d out
 *   logits     the forward call's logits [T,E] fp32; NULL if that call was given none
 *   tables     the forward call's tables; NULL if that call was given none
 *   grad_flags RR_GRAD_STRAIGHT_THROUGH: App. A, Eq. 6 - the weights are n g_ij / S_i with g the
 *              softmax over all experts (Eq. 5), and their normaliser S_i is a constant in the
 *              backward pass, so that a token with a single available expert still has a gradient:
 *                dL/da_il = sum_{p -> expert l} c_ip dL/dc_ip - g_il sum_p c_ip dL/dc_ip.
 *              0: the plain derivative of the normalised weights (g_il replaced by the weight
 *              mass of expert l; zero for a token with a single available expert).
 *   dcombine_w [T,k+2] fp32 out or NULL: dL/dc_ip = <dL/do_i, E_j(x_i)> in the columns of
 *              rr_tables.combine_w, 0 where the token has no such assignment
 *   dlogits    [T,E] fp32 out: dL/da_ij; a row of zeros for a token that no expert processed
 * Dot products and the softmax are accumulated in fp32. */
#define RR_GRAD_STRAIGHT_THROUGH 1u
int rr_router_backward(const rr_config *cfg, const void *dout, const float *logits,
                       const rr_tables *tables, void *workspace, size_t workspace_bytes,
                       uint32_t grad_flags, float *dcombine_w, float *dlogits, void *stream);

/* Per-kernel timing for benchmarks.  While enabled, every kernel the library launches is bracketed
 * by HIP events on the call's stream (events are created on first use and kept).  rr_profile_read
 * synchronises the device, adds up the time of every recorded launch per kernel and clears the
 * record.  Not thread-safe; meant for one benchmarking thread. */
typedef struct rr_kernel_time {
  const char *name;   /* static string, e.g. "ffn_gate_up" */
  int32_t     launches;
  float       total_ms;
} rr_kernel_time;
int rr_profile_enable(int on);
int rr_profile_read(rr_kernel_time *out, int32_t max_entries, int32_t *n_entries);

const char *rr_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* RR_H */
