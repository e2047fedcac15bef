// Host side of librr.so: argument validation, workspace layout, stage sequencing, profiling record.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "rr_internal.h"

// Scratch of rr_rectified_dispatch_static.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address, one per GPU, is looked up once per device (device_setup).
static __device__ __align__(256) unsigned char scratch[RR_STATIC_WORKSPACE_BYTES];

namespace rr {

// ------------------------------------------------------------------ per-device set-up
constexpr int kMaxDevices = 64;
static std::once_flag g_dev_once[kMaxDevices];
static hipError_t g_dev_status[kMaxDevices];
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU

// Runs once per device, with that device current.  Returns the device index, or -1.
static int device_setup() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
  std::call_once(g_dev_once[dev], [dev] {
    hipError_t e = ffn_kernel_attributes();
    if (e == hipSuccess) e = router_kernel_attributes();
    void *p = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    g_scratch_ptr[dev] = e == hipSuccess ? p : nullptr;
    g_dev_status[dev] = e;
  });
  return g_dev_status[dev] == hipSuccess ? dev : -1;
}

// ------------------------------------------------------------------ profiling record
struct ProfSpan { int id; hipEvent_t a, b; };
static bool g_prof_on = false;
static std::vector<ProfSpan> g_spans;       // recorded launches since the last read
static std::vector<hipEvent_t> g_free_events;
static hipEvent_t g_open[K_COUNT];
static const char *const g_kernel_names[K_COUNT] = {
    "router_scores", "topk_rank", "scan_candidates", "scatter_candidates", "select_slot",
    "ir_count", "ir_scan", "ir_weights", "dispatch_gather", "ffn_gate_up", "ffn_down", "combine",
    "router_backward"};

static hipEvent_t get_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

void prof_begin(KernelId id, hipStream_t s) {
  if (!g_prof_on) return;
  hipEvent_t e = get_event();
  g_open[id] = e;
  if (e) (void)hipEventRecord(e, s);
}

void prof_end(KernelId id, hipStream_t s) {
  if (!g_prof_on) return;
  hipEvent_t a = g_open[id];
  hipEvent_t b = get_event();
  if (!a || !b) return;
  (void)hipEventRecord(b, s);
  g_spans.push_back({(int)id, a, b});
}

// ------------------------------------------------------------------ configuration
static int round_up(int a, int b) { return (a + b - 1) / b * b; }

static int make_dims(const rr_config *c, bool need_ffn, Dims *D) {
  if (!c) return RR_ERR_INVALID_ARG;
  if (c->T <= 0 || c->E <= 0 || c->k <= 0 || c->G <= 0 || c->d_model <= 0) return RR_ERR_INVALID_ARG;
  if (c->E % c->G || c->T % c->G || c->k > c->E) return RR_ERR_INVALID_ARG;
  if ((c->flags & RR_FILL_IN) && c->k + 1 > c->E) return RR_ERR_INVALID_ARG;
  if (!(c->capacity_factor > 0.0f) || !isfinite(c->capacity_factor)) return RR_ERR_INVALID_ARG;
  if (c->flags & ~(uint32_t)(RR_INTRA_GPU | RR_FILL_IN | RR_POLICY_ARRIVAL | RR_QUOTA_PER_GROUP)) return RR_ERR_INVALID_ARG;
  if (c->E > kMaxE || c->k > kMaxK || c->T > (1 << 24)) return RR_ERR_UNSUPPORTED;
  if (c->dtype != RR_F32 && c->dtype != RR_BF16) return RR_ERR_UNSUPPORTED;
  if (c->d_model % 8) return RR_ERR_UNSUPPORTED;
  if (need_ffn) {
    if (c->d_ff <= 0) return RR_ERR_INVALID_ARG;
    if (c->d_ff % 8) return RR_ERR_UNSUPPORTED;
    if (c->act != RR_ACT_GELU && c->act != RR_ACT_SWIGLU) return RR_ERR_UNSUPPORTED;
  }
  const int quota = (c->flags & RR_QUOTA_PER_GROUP) ? 1 : 0;
  // token blocks of the candidate counts must not straddle groups
  if (quota && (c->T / c->G) % kTokBlock) return RR_ERR_UNSUPPORTED;
  const int32_t Cq = quota ? rr_capacity(c->T / c->G, c->E, c->capacity_factor)
                           : rr_capacity(c->T, c->E, c->capacity_factor);
  if (Cq < 1) return RR_ERR_INVALID_ARG;
  const int Gq = quota ? c->G : 1;
  if ((int64_t)Cq * Gq * c->E > ((int64_t)1 << 28)) return RR_ERR_UNSUPPORTED;
  const int32_t C = Cq * Gq;
  D->T = c->T; D->d = c->d_model; D->F = c->d_ff > 0 ? c->d_ff : 0; D->E = c->E; D->k = c->k; D->G = c->G; D->C = C;
  D->Cq = Cq; D->Gq = Gq; D->quota = quota;
  D->Eg = c->E / c->G; D->Tg = c->T / c->G;
  D->ir = (c->flags & RR_INTRA_GPU) ? 1 : 0;
  D->fr = (c->flags & RR_FILL_IN) ? 1 : 0;
  D->arrival = (c->flags & RR_POLICY_ARRIVAL) ? 1 : 0;
  D->NR = c->k + D->fr;
  D->NCAT = D->NR * c->E;
  D->NL = D->NCAT * Gq;
  D->NB = (c->T + kTokBlock - 1) / kTokBlock;
  D->cb = 1;
  D->NBc = D->NB;
  D->dtype = c->dtype; D->act = c->act;
  int64_t slots = (int64_t)C * c->E, assigns = (int64_t)D->NR * c->T;
  int64_t rmax = (slots < assigns ? slots : assigns) + (D->ir ? c->T : 0);
  if (rmax > ((int64_t)1 << 28)) return RR_ERR_UNSUPPORTED;
  D->Rmax = (int)rmax;
  if (need_ffn && c->dtype == RR_BF16) {
    // the grouped GEMM addresses one expert's rows, and one expert's weight matrix, with 32-bit byte offsets
    int64_t rows_max = (int64_t)C + (D->ir ? c->T : 0);
    if (rows_max > rmax) rows_max = rmax;
    const int64_t kmax = c->d_model > c->d_ff ? c->d_model : c->d_ff;
    if (rows_max * kmax * 2 >= ((int64_t)1 << 31) || (int64_t)c->d_model * c->d_ff * 2 >= ((int64_t)1 << 31))
      return RR_ERR_UNSUPPORTED;
  }
  D->BM = c->dtype == RR_BF16 ? 256 : 64;
  D->max_mtiles = need_ffn ? D->Rmax / D->BM + c->E : 0;  // routing-only calls cut no GEMM row tiles
  return RR_OK;
}

// Lays the Work arrays out in the workspace; with base == nullptr only measures.
struct Carver {
  char *base; size_t off;
  template <typename Tp> Tp *take(size_t n) {
    size_t bytes = (n * sizeof(Tp) + 255) / 256 * 256;
    Tp *p = base ? reinterpret_cast<Tp *>(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

static size_t carve(const Dims &D, bool forward, void *ws, Work *W) {
  Carver cv{static_cast<char *>(ws), 0};
  size_t T = D.T, NR = D.NR, E = D.E;
  W->key = cv.take<u32>(T * NR);
  W->ir_score = cv.take<float>(T);
  W->ir_cand = cv.take<int32_t>(T);
  W->blk_cnt = cv.take<int32_t>((size_t)D.NCAT * D.NB * router_count_blocks(D));
  W->cat_cnt = cv.take<int32_t>(D.NCAT);
  W->grp_fill = cv.take<int32_t>(E * D.Gq);
  W->grp_off = cv.take<int32_t>(E * D.Gq);
  W->row_token = D.quota ? cv.take<int32_t>(D.Rmax) : nullptr;
  W->cand_key = cv.take<u32>(T * NR);
  W->cand_tok = cv.take<int32_t>(T * NR);
  const bool splits = select_splits(D.T, D.NR, D.NL);
  W->comp_key = splits ? cv.take<u32>(T * NR) : nullptr;
  W->comp_tok = splits ? cv.take<int32_t>(T * NR) : nullptr;
  W->seg_cnt = splits ? cv.take<int32_t>(D.NL + T * NR / kSelectSegLen + 1) : nullptr;
  W->list_done = splits ? cv.take<int32_t>(D.NL) : nullptr;
  W->ir_blk_cnt = cv.take<int32_t>(E * D.NB);
  W->ir_cnt = cv.take<int32_t>(E);
  W->row_base = cv.take<int32_t>(E + 1);
  W->tiles = cv.take<TileInfo>(D.max_mtiles + 1);
  W->tile_ctl = cv.take<int32_t>(4);
  if (forward) {
    size_t K1 = D.k + 1, es = D.dtype == RR_BF16 ? 2 : 4;
    W->logits = cv.take<float>(T * E);
    W->tables.rank_expert = cv.take<int32_t>(T * K1);
    W->tables.slot = cv.take<int32_t>(T * K1);
    W->tables.slot_token = cv.take<int32_t>(E * D.C);
    W->tables.fill_topk = cv.take<int32_t>(E);
    W->tables.fill_total = cv.take<int32_t>(E);
    W->tables.ir_expert = cv.take<int32_t>(T);
    W->tables.ir_row = cv.take<int32_t>(T);
    W->tables.ir_offset = cv.take<int32_t>(E + 1);
    W->tables.ir_token = cv.take<int32_t>(T);
    W->tables.combine_w = cv.take<float>(T * (D.k + 2));
    W->row_dest = cv.take<int32_t>(D.Rmax);
    W->x_disp = cv.take<char>((size_t)D.Rmax * D.d * es);
    W->h = cv.take<char>((size_t)D.Rmax * D.F * es);
    W->y = cv.take<char>((size_t)D.Rmax * D.d * es);
  }
  return cv.off;
}

// The kernels read and write rows with 16-byte vector instructions: data pointers must be 16-byte
// aligned (row lengths already are: d_model, d_ff % 8 == 0, E floats per row are accessed 4-byte
// wise unless the row itself is a multiple of 16 bytes).  NULL (optional arguments) passes.
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
static bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }
static bool tables_aligned(const rr_tables *t) {
  return aligned4(t->rank_expert) && aligned4(t->slot) && aligned4(t->slot_token) && aligned4(t->fill_topk) &&
         aligned4(t->fill_total) && aligned4(t->ir_expert) && aligned4(t->ir_row) && aligned4(t->ir_offset) &&
         aligned4(t->ir_token) && aligned4(t->combine_w);
}

static bool tables_complete(const rr_tables *t) {
  return t && t->rank_expert && t->slot && t->slot_token && t->fill_topk && t->fill_total && t->ir_expert &&
         t->ir_row && t->ir_offset && t->ir_token && t->combine_w;
}

static int check_ws(const Dims &D, bool forward, void *ws, size_t ws_bytes, Work *W) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return RR_ERR_WORKSPACE;
  Work probe;
  size_t need = carve(D, forward, nullptr, &probe);
  if (ws_bytes < need) return RR_ERR_WORKSPACE;
  carve(D, forward, ws, W);
  return RR_OK;
}

}  // namespace rr

using namespace rr;

extern "C" {

int32_t rr_capacity(int32_t T, int32_t E, float capacity_factor) {
  if (T <= 0 || E <= 0 || !(capacity_factor > 0.0f) || !isfinite(capacity_factor)) return -1;
  double c = ceil((double)capacity_factor * (double)T / (double)E);
  if (c < 1.0) c = 1.0;
  if (c > 2147483647.0) return -1;
  return (int32_t)c;
}

int32_t rr_slots_per_expert(const rr_config *cfg) {
  Dims D;
  if (make_dims(cfg, false, &D) != RR_OK) return -1;
  return D.C;
}

int rr_workspace_bytes(const rr_config *cfg, size_t *bytes) {
  if (!bytes) return RR_ERR_INVALID_ARG;
  Dims D;
  int rc = make_dims(cfg, cfg && cfg->d_ff > 0, &D);
  if (rc != RR_OK) return rc;
  Work W;
  *bytes = carve(D, D.F > 0, nullptr, &W);
  return RR_OK;
}

int rr_router_scores(const rr_config *cfg, const void *x, const float *w_router, const float *bias, float *logits,
                     float *probs, int32_t *rank_expert, void *stream) {
  Dims D;
  int rc = make_dims(cfg, false, &D);
  if (rc != RR_OK) return rc;
  if (!x || !w_router || !logits) return RR_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(w_router) || !aligned16(logits) || !aligned16(probs) || !aligned4(bias) ||
      !aligned4(rank_expert))
    return RR_ERR_INVALID_ARG;
  if (device_setup() < 0) return RR_ERR_HIP;
  hipError_t e = launch_router(D, x, w_router, bias, logits, probs, rank_expert, nullptr, nullptr,
                               static_cast<hipStream_t>(stream));
  return e == hipSuccess ? RR_OK : RR_ERR_HIP;
}

int rr_init(void) { return device_setup() >= 0 ? RR_OK : RR_ERR_HIP; }

int rr_rectified_dispatch_static(const rr_config *cfg, const float *logits, const rr_tables *out, void *stream) {
  Dims D;
  int rc = make_dims(cfg, false, &D);
  if (rc != RR_OK) return rc;
  if (!logits || !tables_complete(out)) return RR_ERR_INVALID_ARG;
  if (!aligned16(logits) || !tables_aligned(out)) return RR_ERR_INVALID_ARG;
  Work probe;
  if (carve(D, false, nullptr, &probe) > (size_t)RR_STATIC_WORKSPACE_BYTES) return RR_ERR_TOO_LARGE;
  const int dev = device_setup();
  if (dev < 0 || !g_scratch_ptr[dev]) return RR_ERR_HIP;
  Work W;
  memset(&W, 0, sizeof(W));
  carve(D, false, g_scratch_ptr[dev], &W);
  hipError_t e = launch_dispatch(D, logits, *out, W, false, nullptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? RR_OK : RR_ERR_HIP;
}

int rr_rectified_dispatch(const rr_config *cfg, const float *logits, const rr_tables *out, void *workspace,
                          size_t workspace_bytes, void *stream) {
  Dims D;
  int rc = make_dims(cfg, false, &D);
  if (rc != RR_OK) return rc;
  if (!logits || !tables_complete(out)) return RR_ERR_INVALID_ARG;
  if (!aligned16(logits) || !tables_aligned(out)) return RR_ERR_INVALID_ARG;
  Work W;
  memset(&W, 0, sizeof(W));
  rc = check_ws(D, false, workspace, workspace_bytes, &W);
  if (rc != RR_OK) return rc;
  hipError_t e = launch_dispatch(D, logits, *out, W, false, nullptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? RR_OK : RR_ERR_HIP;
}

int rr_moe_forward(const rr_config *cfg, const void *x, const float *w_router, const float *bias, const void *w1,
                   const void *w3, const void *w2, void *out, const rr_tables *tables, float *logits,
                   void *workspace, size_t workspace_bytes, void *stream) {
  if (!cfg) return RR_ERR_INVALID_ARG;
  const bool routing_only = cfg->d_ff == 0;  // router + tables, no expert FFN
  Dims D;
  int rc = make_dims(cfg, !routing_only, &D);
  if (rc != RR_OK) return rc;
  if (!x || !w_router) return RR_ERR_INVALID_ARG;
  if (routing_only) {
    if (!tables || !logits) return RR_ERR_INVALID_ARG;
  } else {
    if (!w1 || !w2 || !out) return RR_ERR_INVALID_ARG;
    if (cfg->act == RR_ACT_SWIGLU && !w3) return RR_ERR_INVALID_ARG;
  }
  if (tables && (!tables_complete(tables) || !tables_aligned(tables))) return RR_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(w_router) || !aligned4(bias) || !aligned16(logits)) return RR_ERR_INVALID_ARG;
  if (!routing_only && (!aligned16(w1) || !aligned16(w3) || !aligned16(w2) || !aligned16(out))) return RR_ERR_INVALID_ARG;
  Work W;
  memset(&W, 0, sizeof(W));
  rc = check_ws(D, !routing_only, workspace, workspace_bytes, &W);
  if (rc != RR_OK) return rc;
  if (device_setup() < 0) return RR_ERR_HIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const rr_tables &tb = tables ? *tables : W.tables;
  float *lg = logits ? logits : W.logits;
  D.cb = router_count_blocks(D);  // the router ranks and counts: per 32 tokens for small batches
  D.NBc = (D.T + kTokBlock / D.cb - 1) / (kTokBlock / D.cb);
  hipError_t e = launch_router(D, x, w_router, bias, lg, nullptr, nullptr, &tb, &W, s);
  const bool direct = !routing_only && ffn_writes_single_rows(D);
  if (e == hipSuccess) e = launch_dispatch(D, lg, tb, W, true, direct ? W.row_dest : nullptr, s);
  if (routing_only) return e == hipSuccess ? RR_OK : RR_ERR_HIP;
  if (e == hipSuccess && !ffn_fuses_gather(D)) e = launch_gather(D, x, tb, W, s);
  if (e == hipSuccess) e = launch_ffn(D, x, tb, w1, w3, w2, W, out, s);
  if (e == hipSuccess) e = launch_combine(D, tb, W, out, s);
  return e == hipSuccess ? RR_OK : RR_ERR_HIP;
}

int rr_router_backward(const rr_config *cfg, const void *dout, const float *logits, const rr_tables *tables,
                       void *workspace, size_t workspace_bytes, uint32_t grad_flags, float *dcombine_w,
                       float *dlogits, void *stream) {
  if (!cfg) return RR_ERR_INVALID_ARG;
  Dims D;
  int rc = make_dims(cfg, true, &D);  // the expert outputs of a full forward call are needed
  if (rc != RR_OK) return rc;
  if (!dout || !dlogits) return RR_ERR_INVALID_ARG;
  if (grad_flags & ~(uint32_t)RR_GRAD_STRAIGHT_THROUGH) return RR_ERR_INVALID_ARG;
  if (tables && (!tables_complete(tables) || !tables_aligned(tables))) return RR_ERR_INVALID_ARG;
  if (!aligned16(dout) || !aligned4(logits) || !aligned4(dcombine_w) || !aligned4(dlogits)) return RR_ERR_INVALID_ARG;
  Work W;
  memset(&W, 0, sizeof(W));
  rc = check_ws(D, true, workspace, workspace_bytes, &W);
  if (rc != RR_OK) return rc;
  const rr_tables &tb = tables ? *tables : W.tables;
  const float *lg = logits ? logits : W.logits;
  hipError_t e = launch_router_backward(D, dout, lg, tb, W, (grad_flags & RR_GRAD_STRAIGHT_THROUGH) != 0, dcombine_w,
                                        dlogits, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? RR_OK : RR_ERR_HIP;
}

int rr_profile_enable(int on) {
  g_prof_on = on != 0;
  return RR_OK;
}

int rr_profile_read(rr_kernel_time *out, int32_t max_entries, int32_t *n_entries) {
  if (!out || !n_entries || max_entries < K_COUNT) return RR_ERR_INVALID_ARG;
  if (hipDeviceSynchronize() != hipSuccess) return RR_ERR_HIP;
  for (int i = 0; i < K_COUNT; ++i) out[i] = {g_kernel_names[i], 0, 0.0f};
  for (const ProfSpan &sp : g_spans) {
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) {
      out[sp.id].launches += 1;
      out[sp.id].total_ms += ms;
    }
    g_free_events.push_back(sp.a);
    g_free_events.push_back(sp.b);
  }
  g_spans.clear();
  *n_entries = K_COUNT;
  return RR_OK;
}

const char *rr_strerror(int code) {
  switch (code) {
    case RR_OK: return "ok";
    case RR_ERR_INVALID_ARG: return "invalid argument";
    case RR_ERR_UNSUPPORTED: return "unsupported configuration";
    case RR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RR_ERR_HIP: return "HIP runtime or launch failure";
    case RR_ERR_TOO_LARGE: return "configuration needs more scratch than the library's static buffer (RR_STATIC_WORKSPACE_BYTES)";
    default: return "unknown rr_status";
  }
}

}  // extern "C"
