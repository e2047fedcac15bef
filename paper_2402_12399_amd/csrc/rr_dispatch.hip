// Capacity-limited top-k slotting (Sec. 3), Intra-GPU Rectification (Sec. 4.1), Fill-in
// Rectification (Sec. 4.2) and the Eq. 2 / Eq. 3 combine weights: logits -> tables.
//
// Structure.  The number of tokens an expert keeps in round r depends only on how many candidates
// it received in rounds 0..r (kept = min(candidates, C - filled)), never on WHICH ones were kept.
// So all k top-k rounds and the Fill-in round (the (k+1)-th round at unchanged capacity, Sec. 4.2)
// are planned from candidate counts alone and then resolved concurrently, one workgroup per
// (round, expert) list:
//   topk_rank          per token: ranked experts, score keys, best expert of its own group,
//                      candidate counts per (list, token block)
//   scan_candidates    exclusive scan of those counts over token blocks, per list
//   scatter_candidates stable split of the tokens into per-list arrays (ascending token index);
//                      lists whose kept set follows from the counts (nobody, everybody, the first m
//                      in token order) get their slots here and are not materialised
//   select_slot        per remaining list: kept count and first free slot from the counts,
//                      radix-select of the score threshold of the kept set (ties -> lower token
//                      index), then a prefix scan in token order hands out consecutive slots
//   ir_count / ir_scan / ir_weights
//                      per-expert Intra-GPU lists (stable, token order), dispatched-row layout and
//                      row tiles for the grouped GEMM, combine weights
// Plans that are a few dozen numbers (array bases, kept counts, row layout) are recomputed by every
// workgroup that needs them instead of being a launch of their own: a dependent launch costs about
// 6 us on this part, more than any of these kernels needs for a small batch.
// Every table is a deterministic function of the logits: integer atomics are only used for counts.
#include "rr_device.h"

namespace rr {

namespace {

constexpr int TS = kMaxE + 1;  // LDS row stride of a [token][expert] tile

constexpr int kDirectMaxT = 16384;  // tokens up to which the selection lists are not materialised (see select_direct_kernel)
constexpr int kIrSelfMax = 4096;  // experts x token blocks up to which ir_weights does the block scan itself

struct DispatchArgs {
  int T, E, k, C, NR, NCAT, NB, Eg, Tg, ir, fr, arrival, BM, max_mtiles;
  int Cq, Gq, NL;  // capacity blocks: Gq per expert (1, or one per group with per-group quotas) of Cq slots
  int NBc, cb;     // candidate counts come per count block: cb of them per token block, NBc in all
  int ir_self;     // small batches: ir_weights sums the Intra-GPU block counts itself (no scan launch)
  int direct;      // small batches, one capacity block per expert: select_direct_kernel finds its candidates itself
};

// lanes of this wave whose (valid, e) equals the caller's; e < 64
__device__ inline unsigned long long same_expert_mask(bool valid, int e) {
  unsigned long long mask = __ballot(valid);
#pragma unroll
  for (int b = 0; b < 6; ++b) {
    bool bit = (e >> b) & 1;
    unsigned long long bb = __ballot(valid && bit);
    mask &= bit ? bb : ~bb;
  }
  return mask;
}

__device__ inline int lanes_below(unsigned long long mask) {
  int lane = lane_id();
  return __popcll(mask & ((1ull << lane) - 1ull));
}

// ------------------------------------------------------------------ topk_rank
__global__ __launch_bounds__(kTokBlock) void topk_rank_kernel(const float *__restrict__ logits, DispatchArgs A,
                                                              int32_t *__restrict__ rank_expert,
                                                              int32_t *__restrict__ slot, u32 *__restrict__ key,
                                                              float *__restrict__ ir_score,
                                                              int32_t *__restrict__ ir_cand,
                                                              int32_t *__restrict__ blk_cnt) {
  __shared__ float tile[kTokBlock * TS];
  __shared__ int cnt[kMaxRounds * kMaxE];
  const int tid = threadIdx.x, b = blockIdx.x;
  const int t0 = b * kTokBlock;
  const int ntok = min(kTokBlock, A.T - t0);
  const int E = A.E;
  const float *src = logits + (size_t)t0 * E;  // 16-byte aligned: t0 is a multiple of 128
  const int nvec = (ntok * E) >> 2;
  for (int v = tid; v < nvec; v += kTokBlock) {
    const float4 q = reinterpret_cast<const float4 *>(src)[v];
    const float qq[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int idx = 4 * v + u, row = idx / E, e = idx - row * E;
      tile[row * TS + e] = qq[u];
    }
  }
  for (int idx = 4 * nvec + tid; idx < ntok * E; idx += kTokBlock) {
    int row = idx / E, e = idx - row * E;
    tile[row * TS + e] = src[idx];
  }
  for (int c = tid; c < A.NCAT; c += kTokBlock) cnt[c] = 0;
  __syncthreads();
  if (tid < ntok) {
    const int i = t0 + tid;
    const float *row = tile + tid * TS;
    const int n = min(A.k + 1, E);
    unsigned long long top[kMaxRank];
    top_keys_of_range<kMaxRank>(row, 0, E, top);
#pragma unroll
    for (int q = 0; q < kMaxRank; ++q) {
      const int e = rank_key_expert(top[q]);  // -1 past the number of experts
      if (q <= A.k) rank_expert[(size_t)i * (A.k + 1) + q] = (q < n) ? e : -1;
      if (q < A.NR) {
        key[(size_t)i * A.NR + q] = rank_key_score(top[q]);
        atomicAdd(&cnt[q * E + e], 1);
      }
    }
    if (!A.fr) slot[(size_t)i * (A.k + 1) + A.k] = -1;
    const int g = i / A.Tg;
    float best;
    int arg;
    best_in_group(row, g * A.Eg, (g + 1) * A.Eg, best, arg);
    ir_score[i] = best;
    ir_cand[i] = arg;
  }
  __syncthreads();
  for (int c = tid; c < A.NCAT; c += kTokBlock) blk_cnt[(size_t)c * A.NBc + b] = cnt[c];  // here cb == 1
}

// ------------------------------------------------------------------ scan over token blocks
// One workgroup per list: exclusive scan of a[list][0..NB) in place, total to tot[list].  A thread
// scans SC_PER consecutive entries in registers, so 8192 entries are one trip with two barriers.
constexpr int SC_THREADS = 1024, SC_PER = 8, SC_WAVES = SC_THREADS / kWave;
// zero: nullptr, or an array of which every workgroup clears nzero entries from blockIdx.x * nzero on.
__global__ __launch_bounds__(SC_THREADS) void scan_blocks_kernel(int32_t *__restrict__ a, int32_t *__restrict__ tot,
                                                                 int NB, int32_t *__restrict__ zero, int nzero) {
  __shared__ int wsum[SC_WAVES];
  if (zero)
    for (int q = threadIdx.x; q < nzero; q += SC_THREADS) zero[(size_t)blockIdx.x * nzero + q] = 0;
  int32_t *p = a + (size_t)blockIdx.x * NB;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const bool vec = (NB & 3) == 0;  // then every list starts 16-byte aligned
  int running = 0;
  for (int base = 0; base < NB; base += SC_THREADS * SC_PER) {
    const int idx = base + tid * SC_PER;
    int v[SC_PER];
    if (vec && idx + SC_PER <= NB) {
      const int4 q0 = *reinterpret_cast<const int4 *>(p + idx), q1 = *reinterpret_cast<const int4 *>(p + idx + 4);
      v[0] = q0.x; v[1] = q0.y; v[2] = q0.z; v[3] = q0.w; v[4] = q1.x; v[5] = q1.y; v[6] = q1.z; v[7] = q1.w;
    } else {
#pragma unroll
      for (int u = 0; u < SC_PER; ++u) v[u] = idx + u < NB ? p[idx + u] : 0;
    }
    int sum = 0;
#pragma unroll
    for (int u = 0; u < SC_PER; ++u) {  // v[u] becomes the exclusive prefix inside the thread
      const int t = v[u];
      v[u] = sum;
      sum += t;
    }
    int incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      int t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int q = 0; q < SC_WAVES; ++q) {
      int s = wsum[q];
      if (q < w) before += s;
      total += s;
    }
    const int off0 = running + before + incl - sum;
    if (vec && idx + SC_PER <= NB) {
      *reinterpret_cast<int4 *>(p + idx) = make_int4(off0 + v[0], off0 + v[1], off0 + v[2], off0 + v[3]);
      *reinterpret_cast<int4 *>(p + idx + 4) = make_int4(off0 + v[4], off0 + v[5], off0 + v[6], off0 + v[7]);
    } else {
#pragma unroll
      for (int u = 0; u < SC_PER; ++u)
        if (idx + u < NB) p[idx + u] = off0 + v[u];
    }
    running += total;
    __syncthreads();
  }
  if (tid == 0) tot[blockIdx.x] = running;
}

// ------------------------------------------------------------------ scatter_candidates
// Besides splitting the tokens into per-list arrays this kernel settles every list whose outcome
// follows from the candidate counts alone: nobody kept (the capacity block is full), everybody kept,
// or the first m in token order (arrival order).  A candidate's position in its list is known here,
// so its slot is too: the token's slot entry is written with the rest of its row (whole cache
// lines) and the candidate never enters the arrays.  Only the lists that are selected by score
// (Sec. 3: the lowest scores are dropped; Sec. 4.2: Fill-in takes the highest) are materialised for
// select_slot.
__global__ __launch_bounds__(kTokBlock) void scatter_candidates_kernel(DispatchArgs A,
                                                                       const int32_t *__restrict__ rank_expert,
                                                                       const u32 *__restrict__ key,
                                                                       const int32_t *__restrict__ blk_off,
                                                                       const int32_t *__restrict__ cat_cnt,
                                                                       u32 *__restrict__ cand_key,
                                                                       int32_t *__restrict__ cand_tok,
                                                                       int32_t *__restrict__ slot,
                                                                       int32_t *__restrict__ slot_token) {
  constexpr int NW = kTokBlock / kWave;
  __shared__ int wcnt[kMaxRounds][NW][kMaxE];
  __shared__ int s_base[kMaxRounds * kMaxE];
  // per list of this block's capacity block: first candidate (position in the candidate array), kept
  // count (-1: selected by score, the list goes to select_slot) and first slot
  __shared__ int s_lo[kMaxRounds * kMaxE], s_keep[kMaxRounds * kMaxE], s_fill0[kMaxRounds * kMaxE];
  const int tid = threadIdx.x, b = xcd_block(blockIdx.x, A.NB), w = tid >> 6, lane = tid & 63;
  const int i = b * kTokBlock + tid;
  const bool valid = i < A.T;
  for (int c = tid; c < kMaxRounds * NW * kMaxE; c += kTokBlock) (&wcnt[0][0][0])[c] = 0;
  // the token's experts are fetched in the same round trip as the array counts below (loads do not
  // move across barriers by themselves)
  int e_r[kMaxRounds], rank_r[kMaxRounds], off_r[kMaxRounds];
  u32 key_r[kMaxRounds];
#pragma unroll
  for (int r = 0; r < kMaxRounds; ++r) {
    e_r[r] = 0;
    if (valid && r < A.NR) e_r[r] = rank_expert[(size_t)i * (A.k + 1) + r];
  }
  // every token is a candidate of exactly one array per round: round r's arrays tile [r T, (r+1) T)
  // in expert order (a dozen counts: recomputed by every workgroup rather than by a launch of its own)
  for (int r = w; r < A.NR; r += NW) {
    const int c = lane < A.E ? cat_cnt[r * A.E + lane] : 0;
    int incl = c;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      int t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane < A.E) s_base[r * A.E + lane] = r * A.T + incl - c;
  }
  // the plan of the lists that this block's tokens can be candidates of: capacity block g of every
  // (round, expert); kept = min(candidates, free slots) round after round, as in select_slot
  {
    const int bpg = A.NB / A.Gq * A.cb, g = b / (A.NB / A.Gq);
    for (int c = tid; c < A.NCAT; c += kTokBlock) {
      const int r = c / A.E, j = c - r * A.E;
      int n = 0, m = 0, fill = 0, lo = 0;
      for (int rr = 0; rr <= r; ++rr) {
        const int cc = rr * A.E + j;
        fill += m;
        lo = g == 0 ? 0 : blk_off[(size_t)cc * A.NBc + g * bpg];
        const int hi = g == A.Gq - 1 ? cat_cnt[cc] : blk_off[(size_t)cc * A.NBc + (g + 1) * bpg];
        n = hi - lo;
        m = min(n, A.Cq - fill);
      }
      const bool by_score = !A.arrival || r == A.k;
      s_lo[c] = lo;
      s_keep[c] = (m == n || m == 0 || !by_score) ? m : -1;
      s_fill0[c] = g * A.Cq + fill;
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kMaxRounds; ++r) {
    rank_r[r] = 0;
    off_r[r] = 0;
    key_r[r] = 0;
    if (r < A.NR) {
      const int e = e_r[r];
      // in flight across the barrier, and only what the list's plan needs: nothing for a list that keeps
      // nobody, the position for a list that keeps by position, the key as well for a score-selected one
      const int keep = s_keep[r * A.E + e];
      if (valid && keep != 0) off_r[r] = blk_off[(size_t)(r * A.E + e) * A.NBc + b * A.cb];
      if (valid && keep < 0) key_r[r] = key[(size_t)i * A.NR + r];
      unsigned long long mask = same_expert_mask(valid, e);
      int below = lanes_below(mask);
      if (valid && below == 0) wcnt[r][w][e] = __popcll(mask);
      rank_r[r] = below;
    }
  }
  __syncthreads();
  if (!valid) return;
#pragma unroll
  for (int r = 0; r < kMaxRounds; ++r) {
    if (r < A.NR) {
      int e = e_r[r], cat = r * A.E + e;
      int at = off_r[r] + rank_r[r];  // position in the (round, expert) array
      for (int q = 0; q < w; ++q) at += wcnt[r][q][e];
      const int keep = s_keep[cat], idx = at - s_lo[cat];
      int sl = -1;  // "dropped" until select_slot says otherwise (it only touches the entries of the tokens it keeps)
      if (keep < 0) {
        cand_key[s_base[cat] + at] = key_r[r];
        cand_tok[s_base[cat] + at] = i;
      } else if (keep > 0 && idx < keep) {  // (keep == 0: the position was not even fetched)
        sl = s_fill0[cat] + idx;
        slot_token[(size_t)e * A.C + sl] = i;
      }
      slot[(size_t)i * (A.k + 1) + r] = sl;
    }
  }
}

// ------------------------------------------------------------------ select_slot
constexpr int SS_THREADS = 1024;
constexpr int SS_WAVES = SS_THREADS / kWave;
constexpr int SS_PER = kSelectRegMax / SS_THREADS;  // keys a thread keeps in registers (24)
constexpr int kHistCopies = 32;  // counters per histogram bin (see radix_select)
constexpr int kHistWords = 256 * (1 + kHistCopies);

// m-th largest key among those that `each` enumerates, by 8-bit digits from the top (Sec. 3: the
// lowest scores are dropped).  Returns the threshold key; need_eq = how many of the keys equal to it
// are kept (the first ones in token order).  `each(f)` calls f(key, valid) for every key slot of the
// calling thread, the same number of times in every lane of a wave (invalid slots with valid = false);
// all threads of the workgroup call this together.
// Scores of one list share their leading digits, so most lanes of a wave hit the same histogram
// bin, and LDS atomics of one instruction on one address are served one lane after the other: every
// bin has kHistCopies counters, lane l adds to copy l % kHistCopies (consecutive words, different
// banks), and the copies are added up before the bins are scanned.
// last_pass > 0 stops after the digits above it: the result is then the threshold with its lower digits
// cleared - a lower bound of the m-th largest key that is off by less than one step of the last digit
// taken (need_eq is meaningless then).
template <class Each>
__device__ inline u32 radix_select(int m, Each each, u32 *hist, u32 *s_pick, u32 &need_eq, int last_pass = 0) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  u32 *copies = hist + 256;  // [256][kHistCopies]
  u32 prefix = 0, remaining = (u32)m;
  for (int pass = 3; pass >= last_pass; --pass) {
    const int shift = pass * 8;
#pragma unroll
    for (int q = 0; q < 256 * kHistCopies / SS_THREADS; ++q) copies[q * SS_THREADS + tid] = 0;
    __syncthreads();
    each([&](u32 kx, bool valid) {
      if (valid && (pass == 3 || ((kx ^ prefix) >> (shift + 8)) == 0))
        atomicAdd(&copies[((kx >> shift) & 255u) * kHistCopies + (lane & (kHistCopies - 1))], 1u);
    });
    __syncthreads();
    {  // thread t adds up a quarter of the copies of bin t / 4
      static_assert(SS_THREADS == 4 * 256 && kHistCopies % 4 == 0, "four threads per bin");
      const u32 *c = copies + (tid >> 2) * kHistCopies + (tid & 3) * (kHistCopies / 4);
      u32 sum = 0;
#pragma unroll
      for (int q = 0; q < kHistCopies / 4; ++q) sum += c[q];
      sum += __shfl_xor(sum, 1);
      sum += __shfl_xor(sum, 2);
      if ((tid & 3) == 0) hist[tid >> 2] = sum;
    }
    __syncthreads();
    if (w == 0) {
      // lane l owns bins 255-4l .. 252-4l, i.e. bins in descending order across lanes
      u32 c0 = hist[255 - 4 * lane], c1 = hist[254 - 4 * lane], c2 = hist[253 - 4 * lane], c3 = hist[252 - 4 * lane];
      u32 sum = c0 + c1 + c2 + c3, incl = sum;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        u32 t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      u32 excl = incl - sum;
      if (excl < remaining && remaining <= incl) {
        u32 rem = remaining - excl;
        int bkt = 255 - 4 * lane;
        if (rem > c0) { rem -= c0; --bkt;
          if (rem > c1) { rem -= c1; --bkt;
            if (rem > c2) { rem -= c2; --bkt; } } }
        s_pick[0] = (u32)bkt;
        s_pick[1] = rem;
      }
    }
    __syncthreads();  // the picks are next written two barriers from here: no barrier needed after reading them
    prefix |= s_pick[0] << shift;
    remaining = s_pick[1];
  }
  need_eq = remaining;
  return prefix;
}

// Shared memory of the selection kernels.
struct SelectSmem {
  u32 hist[kHistWords];
  u32 pick[2];
  int2 wtot[SS_PER][SS_WAVES];  // (kept-for-sure, equal-to-threshold) counts per (trip, wave)
  int2 wsum[8];
};

// Selection and slotting of a list of n <= SS_THREADS * SS_PER candidates held in registers: candidate
// idx = u * SS_THREADS + tid is element u of thread tid (`load(idx, key, tok)` fetches it), so the
// candidates are met in token order.  by_score: the m highest keys are kept, equal keys in token order
// (radix select of the threshold, four digit passes on registers); otherwise the first m in token
// order.  Kept candidates take slots fill0, fill0 + 1, ... in token order: one scan over the
// (trip, wave) totals of the kept flags.  Only kept candidates are written (every slot entry starts
// as -1).
template <class Load>
__device__ inline void select_in_registers(const DispatchArgs &A, int n, int m, bool by_score, int r, int j, int fill0,
                                           Load load, SelectSmem &S, int32_t *__restrict__ slot,
                                           int32_t *__restrict__ slot_token) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const unsigned long long below = (1ull << lane) - 1ull;
  const int nu = (n + SS_THREADS - 1) / SS_THREADS;
  u32 kreg[SS_PER];
  int treg[SS_PER];
#pragma unroll
  for (int u = 0; u < SS_PER; ++u) {
    const int idx = u * SS_THREADS + tid;
    kreg[u] = 0;
    treg[u] = 0;
    if (u < nu && idx < n) load(idx, kreg[u], treg[u]);
  }
  u32 thr = 0, need_eq = 0;
  if (by_score)
    thr = radix_select(m, [&](auto f) {
#pragma unroll
      for (int u = 0; u < SS_PER; ++u)
        if (u < nu) f(kreg[u], u * SS_THREADS + tid < n);
    }, S.hist, S.pick, need_eq);

  int pre[SS_PER];  // lanes of this wave before this one: kept-for-sure | equal << 8
#pragma unroll
  for (int u = 0; u < SS_PER; ++u) {
    pre[u] = 0;
    if (u < nu) {
      const int idx = u * SS_THREADS + tid;
      const bool valid = idx < n;
      bool gt, eq = false;
      if (by_score) { gt = valid && kreg[u] > thr; eq = valid && kreg[u] == thr; }
      else gt = valid && idx < m;
      const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
      pre[u] = __popcll(bgt & below) | (__popcll(beq & below) << 8) | (gt ? 1 << 16 : 0) | (eq ? 1 << 17 : 0);
      if (lane == 0) S.wtot[u][w] = make_int2(__popcll(bgt), __popcll(beq));
    }
  }
  __syncthreads();
  // exclusive scan of the nu * SS_WAVES totals in (trip, wave) order = token order
  const int ne = nu * SS_WAVES;
  int2 mine = make_int2(0, 0), incl = mine;
  if (tid < ne) mine = (&S.wtot[0][0])[tid];
  if (tid < 8 * kWave) {  // SS_PER * SS_WAVES = 384 entries fit 6 waves
    incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int tx = __shfl_up(incl.x, off), ty = __shfl_up(incl.y, off);
      if (lane >= off) { incl.x += tx; incl.y += ty; }
    }
    if (lane == 63) S.wsum[w] = incl;
  }
  __syncthreads();
  if (tid < ne) {
    int2 before = make_int2(0, 0);
    for (int q = 0; q < w; ++q) { before.x += S.wsum[q].x; before.y += S.wsum[q].y; }
    (&S.wtot[0][0])[tid] = make_int2(before.x + incl.x - mine.x, before.y + incl.y - mine.y);
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < SS_PER; ++u) {
    if (u < nu && u * SS_THREADS + tid < n) {
      const int2 base = S.wtot[u][w];
      const bool gt = (pre[u] >> 16) & 1, eq = (pre[u] >> 17) & 1;
      const int eqs = base.y + ((pre[u] >> 8) & 255);  // equal keys before this one
      if (gt || (eq && (u32)eqs < need_eq)) {
        const int sl = fill0 + base.x + (pre[u] & 255) + min(eqs, (int)need_eq);
        slot[(size_t)treg[u] * (A.k + 1) + r] = sl;
        slot_token[(size_t)j * A.C + sl] = treg[u];
      }
    }
  }
}

// The same for a list of any length, streamed from memory by one workgroup: the threshold by four
// digit passes over the keys, then a pass that hands out the slots 1024 candidates at a time.  The
// path for lists that fit neither the registers nor the split scheme below; exact for any input.
__device__ inline void select_streaming(const DispatchArgs &A, int n, int m, bool by_score, int r, int j, int fill0,
                                        const u32 *__restrict__ keys, const int32_t *__restrict__ toks, SelectSmem &S,
                                        int32_t *__restrict__ slot, int32_t *__restrict__ slot_token) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const unsigned long long below = (1ull << lane) - 1ull;
  u32 thr = 0, need_eq = 0;
  if (by_score)
    thr = radix_select(m, [&](auto f) {
      for (int base = 0; base < n; base += SS_THREADS) {
        const int idx = base + tid;
        f(idx < n ? keys[idx] : 0u, idx < n);
      }
    }, S.hist, S.pick, need_eq);
  int run_gt = 0, run_eq = 0;
  for (int base = 0; base < n; base += SS_THREADS) {
    const int idx = base + tid;
    const bool valid = idx < n;
    u32 kx = 0;
    int tok = 0;
    if (valid) { kx = keys[idx]; tok = toks[idx]; }
    bool gt, eq = false;
    if (by_score) { gt = valid && kx > thr; eq = valid && kx == thr; }
    else gt = valid && idx < m;
    unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    int gt_before = __popcll(bgt & below), eq_before = __popcll(beq & below);
    if (lane == 0) S.wtot[0][w] = make_int2(__popcll(bgt), __popcll(beq));
    __syncthreads();
    int tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int q = 0; q < SS_WAVES; ++q) {
      const int2 t = S.wtot[0][q];
      if (q < w) { gt_before += t.x; eq_before += t.y; }
      tot_gt += t.x; tot_eq += t.y;
    }
    if (valid) {
      int eqs = run_eq + eq_before;                       // equal keys before this one
      if (gt || (eq && (u32)eqs < need_eq)) {
        int sl = fill0 + run_gt + gt_before + min(eqs, (int)need_eq);
        slot[(size_t)tok * (A.k + 1) + r] = sl;
        slot_token[(size_t)j * A.C + sl] = tok;
      }
    }
    run_gt += tot_gt;
    run_eq += tot_eq;
    __syncthreads();
  }
}

// A selection list is the piece of a (round, expert) candidate array that competes for one capacity
// block: the whole array and the expert's whole queue by default; with per-group quotas (Sec. 3's
// capacity read per GPU) the candidates of group g - a contiguous piece, since candidates are in
// ascending token index and groups are token ranges that end on block boundaries - and the group's
// Cq slots.  The kept count of a round is min(candidates, free slots of the block), so every round
// (Fill-in, the (k+1)-th, included) is planned from the candidate counts alone; each workgroup derives
// its own list's numbers from them, and the workgroup of an expert's last round and first block also
// writes the expert's fill counts.
//
// Lists of up to SS_THREADS * SS_PER candidates are one workgroup's work (select_in_registers).  A
// longer list - a skewed router sends most tokens to a few experts - is cut into segments of
// kSegLen candidates, one workgroup each (the first workgroups of the grid are the segments after a
// list's first; each derives its (list, segment) from the candidate counts):
//   * nobody, everybody or the first m in token order kept: scatter_candidates has handed out the
//     slots already, the list's workgroups leave at once;
//   * the m highest scores kept: every segment workgroup takes the same sample of the list's keys
//     (runs of 64 consecutive candidates, spread evenly) and selects in it a key L that, with a
//     margin of several standard deviations, lies below the list's m-th highest key; it then copies its segment's candidates with key >= L,
//     in order, to a second pair of arrays and counts them.  The workgroup that finishes last
//     (a ticket from an atomic counter - nobody waits for anybody) adds up the counts: if they
//     number at least m and fit the registers, the kept set is among them and it finishes the
//     list with select_in_registers; otherwise (the sample misled, or the scores are tied en
//     masse) it streams the original list.  The result is exact either way.
constexpr int kSegLen = kSelectSegLen;           // 16384
constexpr int kSegPer = kSegLen / SS_THREADS;    // candidates per thread of a segment workgroup
constexpr int kSampleLen = kSegLen;              // keys in the sample
constexpr int kRegMax = kSelectRegMax;           // candidates that fit the registers of one workgroup
constexpr int kMapLists = 2048;                  // lists up to which long lists are split (the map is kept in LDS)

// Exclusive scan of one value per thread over the workgroup (two barriers); total = sum over all threads.
__device__ inline int block_scan_exclusive(int v, int *s_wave, int &total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  if (lane == 63) s_wave[w] = incl;
  __syncthreads();
  int before = 0;
  total = 0;
#pragma unroll
  for (int q = 0; q < SS_WAVES; ++q) {
    const int t = s_wave[q];
    if (q < w) before += t;
    total += t;
  }
  __syncthreads();
  return before + incl - v;
}

__global__ __launch_bounds__(SS_THREADS) void select_slot_kernel(DispatchArgs A, const int32_t *__restrict__ cat_cnt,
                                                                 const int32_t *__restrict__ blk_off,
                                                                 const u32 *__restrict__ cand_key,
                                                                 const int32_t *__restrict__ cand_tok,
                                                                 u32 *__restrict__ comp_key,
                                                                 int32_t *__restrict__ comp_tok,
                                                                 int32_t *__restrict__ seg_cnt,
                                                                 int32_t *__restrict__ list_done,
                                                                 int32_t *__restrict__ slot,
                                                                 int32_t *__restrict__ slot_token,
                                                                 int32_t *__restrict__ grp_fill,
                                                                 int32_t *__restrict__ grp_off,
                                                                 int32_t *__restrict__ fill_topk,
                                                                 int32_t *__restrict__ fill_total) {
  __shared__ SelectSmem S;
  __shared__ int s_extra[kMapLists + 1];  // exclusive scan over the lists of their segments after the first
  __shared__ int s_wave[SS_WAVES];
  __shared__ int s_bcast;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int bpg = A.NB / A.Gq * A.cb;  // count blocks per group (exact with quotas; all of them otherwise)
  // candidates [lo, hi) of (round rr, expert jj) that belong to group gg
  auto piece = [&](int rr, int jj, int gg, int &lo, int &hi) {
    const int c = rr * A.E + jj;
    lo = gg == 0 ? 0 : blk_off[(size_t)c * A.NBc + gg * bpg];
    hi = gg == A.Gq - 1 ? cat_cnt[c] : blk_off[(size_t)c * A.NBc + (gg + 1) * bpg];
  };

  // ---- which (list, segment) is this workgroup.  The workgroups of the further segments come first
  // in the grid (those that turn out to have no segment leave at once): a split list is finished
  // by the last of its segments, so they should not queue behind the one-workgroup lists.
  const bool can_split = select_splits(A.T, A.NR, A.NL);  // otherwise the grid has one workgroup per list
  const int n_extra = (int)gridDim.x - A.NL;
  int lst = (int)blockIdx.x - n_extra, seg = 0, extra_base = 0;
  if (can_split) {
    int carry = 0;
    for (int l0 = 0; l0 < A.NL; l0 += SS_THREADS) {
      const int l = l0 + tid;
      int ex = 0;
      if (l < A.NL) {
        const int c = l / A.Gq, gg = l - c * A.Gq, rr = c / A.E;
        int lo, hi;
        piece(rr, c - rr * A.E, gg, lo, hi);
        ex = hi - lo > kRegMax ? (hi - lo + kSegLen - 1) / kSegLen - 1 : 0;
      }
      int total;
      const int excl = block_scan_exclusive(ex, s_wave, total);
      if (l < A.NL) s_extra[l] = carry + excl;
      carry += total;
    }
    if (tid == 0) s_extra[A.NL] = carry;
    __syncthreads();
    if ((int)blockIdx.x < n_extra) {
      const int x = blockIdx.x;
      if (x >= s_extra[A.NL]) return;  // no such segment
      int a = 0, b = A.NL - 1;  // the last list whose scan value is <= x (lists without extra segments repeat their successor's value)
      while (a < b) {
        const int mid = (a + b + 1) >> 1;
        if (s_extra[mid] <= x) a = mid; else b = mid - 1;
      }
      lst = a;
      seg = x - s_extra[lst] + 1;
    }
    extra_base = s_extra[lst];
  }

  // ---- the list: (round r, expert j, capacity block g); n candidates, m of them kept, in slots fill0 ..
  const int cat = lst / A.Gq, g = lst - cat * A.Gq, r = cat / A.E, j = cat - r * A.E;
  int n = 0, m = 0, fill = 0, lo = 0;
  for (int rr = 0; rr <= r; ++rr) {
    int hi;
    fill += m;
    piece(rr, j, g, lo, hi);
    n = hi - lo;
    m = min(n, A.Cq - fill);
  }
  const int fill0 = g * A.Cq + fill;
  int base = r * A.T + lo;  // round r's arrays tile [r T, (r+1) T) in expert order
  for (int jj = 0; jj < j; ++jj) base += cat_cnt[r * A.E + jj];
  const u32 *keys = cand_key + base;
  const int32_t *toks = cand_tok + base;
  if (seg == 0) {
    if (r == A.NR - 1 && g == 0 && w == 0) {
      // lane gg: occupied slots of block gg after the top-k rounds and after every round
      int topk = 0, total = 0;
      if (lane < A.Gq) {
        for (int rr = 0; rr < A.NR; ++rr) {
          int l, h;
          piece(rr, j, lane, l, h);
          total += min(h - l, A.Cq - total);
          if (rr == A.k - 1) topk = total;
        }
      }
      int incl = total, sum_topk = topk;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sum_topk += __shfl_xor(sum_topk, off);
      if (lane < A.Gq) {
        grp_fill[j * A.Gq + lane] = total;
        grp_off[j * A.Gq + lane] = incl - total;
      }
      if (lane == 63) fill_total[j] = incl;
      if (lane == 0) fill_topk[j] = sum_topk;
    }
    // the last round pads the rest of the capacity block (Sec. 3: zero padding)
    if (r == A.NR - 1)
      for (int sl = fill0 + m + tid; sl < (g + 1) * A.Cq; sl += SS_THREADS) slot_token[(size_t)j * A.C + sl] = -1;
  }
  if (m == 0) return;  // nobody kept: every slot entry already says so
  const bool by_score = !A.arrival || r == A.k;  // the Fill-in round always selects by score (Sec. 4.2)
  if (m == n || !by_score) return;  // everybody, or the first m in token order: settled by scatter_candidates
  const bool is_long = n > kRegMax;          // then, if can_split, the list has a workgroup per segment
  if (!is_long) {
    select_in_registers(A, n, m, true, r, j, fill0, [&](int idx, u32 &kx, int &tok) { kx = keys[idx]; tok = toks[idx]; },
                        S, slot, slot_token);
    return;
  }

  // ---- long list, the m highest scores: sample, copy the candidates that may be kept, last one finishes
  const int nseg = (n + kSegLen - 1) / kSegLen;
  // rank in the sample: the expected number of sampled keys among the list's m highest, plus five
  // standard deviations and a few; the candidates with key >= L then number about n / kSampleLen times that
  const float expect = (float)m * (float)kSampleLen / (float)n;
  const int qsel = (int)(expect + 5.0f * sqrtf(expect) + 16.0f);
  const bool split = can_split && qsel < kSampleLen && (long long)qsel * n / kSampleLen <= kRegMax * 7 / 8;
  if (!split) {
    if (seg == 0) select_streaming(A, n, m, true, r, j, fill0, keys, toks, S, slot, slot_token);
    return;
  }
  u32 L;
  {
    // the sample: kSampleLen / 64 runs of 64 consecutive candidates, spread evenly over the list (a wave
    // instruction then reads one run - two cache lines - where single candidates a stride apart would
    // touch 64 lines: 19 -> 5 us for a list of 900 K candidates)
    static_assert(kSegPer * SS_WAVES * kWave == kSampleLen, "one run per (trip, wave)");
    const int run = n / (kSampleLen / kWave);  // > 64: n > kRegMax
    u32 sk[kSegPer];
#pragma unroll
    for (int u = 0; u < kSegPer; ++u) sk[u] = keys[(size_t)(u * SS_WAVES + w) * run + lane];
    u32 dummy;
    // the two leading digits are enough: L only has to lie below the list's m-th highest key, and the keys of
    // one 16-bit step (2^-7 of a score) are a handful of candidates more
    L = radix_select(qsel, [&](auto f) {
#pragma unroll
      for (int u = 0; u < kSegPer; ++u) f(sk[u], true);
    }, S.hist, S.pick, dummy, 2);
  }
  {
    const unsigned long long below = (1ull << lane) - 1ull;
    const int i0 = seg * kSegLen, len = min(n - i0, kSegLen);
    u32 kreg[kSegPer];
    int pre[kSegPer];
#pragma unroll
    for (int u = 0; u < kSegPer; ++u) {
      const int idx = u * SS_THREADS + tid;
      kreg[u] = idx < len ? keys[i0 + idx] : 0u;
      const bool ge = idx < len && kreg[u] >= L;
      const unsigned long long bge = __ballot(ge);
      pre[u] = __popcll(bge & below) | (ge ? 1 << 16 : 0);
      if (lane == 0) S.wtot[u][w] = make_int2(__popcll(bge), 0);
    }
    __syncthreads();
    // exclusive scan of the kSegPer * SS_WAVES wave totals in (trip, wave) order = token order
    int mine = 0, incl = 0;
    if (tid < kSegPer * SS_WAVES) mine = (&S.wtot[0][0])[tid].x;
    if (tid < 4 * kWave) {  // kSegPer * SS_WAVES = 256 entries = 4 waves
      incl = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      if (lane == 63) S.wsum[w].x = incl;
    }
    __syncthreads();
    int count = 0;
    if (tid < kSegPer * SS_WAVES) {
      int before = 0;
      for (int q = 0; q < w; ++q) before += S.wsum[q].x;
      (&S.wtot[0][0])[tid].x = before + incl - mine;
    }
    count = S.wsum[0].x + S.wsum[1].x + S.wsum[2].x + S.wsum[3].x;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kSegPer; ++u) {
      if ((pre[u] >> 16) & 1) {
        const int idx = u * SS_THREADS + tid, pos = base + i0 + S.wtot[u][w].x + (pre[u] & 255);
        comp_key[pos] = kreg[u];
        comp_tok[pos] = toks[i0 + idx];
      }
    }
    // publish: count, then the ticket.  Every wave waits until its own copies have been written (a
    // store counts as done when the L2 has it), the barrier collects the waves, and ONE device-scope
    // fence (a write-back of the L2, which the other XCDs do not see into) goes before the ticket.
    // Whoever draws the last ticket fences once more before it reads the other segments' copies.
    const int seg_id = seg == 0 ? lst : A.NL + extra_base + seg - 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      seg_cnt[seg_id] = count;
      __threadfence();
      s_bcast = atomicAdd(&list_done[lst], 1);
      if (s_bcast == nseg - 1) __threadfence();
    }
    __syncthreads();
    if (s_bcast != nseg - 1) return;
  }
  // ---- the last workgroup of the list: segments' counts -> offsets of their copies (s_extra is free now)
  __syncthreads();
  int total = 0;
  {
    int carry = 0;
    for (int q0 = 0; q0 < nseg; q0 += SS_THREADS) {  // nseg <= 2^24 / kSegLen + 1 fits s_extra
      const int q = q0 + tid;
      const int c = q < nseg ? seg_cnt[q == 0 ? lst : A.NL + extra_base + q - 1] : 0;
      int tot;
      const int excl = block_scan_exclusive(c, s_wave, tot);
      if (q < nseg) s_extra[q] = carry + excl;
      carry += tot;
    }
    total = carry;
    __syncthreads();
  }
  if (total < m || total > kRegMax) {
    select_streaming(A, n, m, true, r, j, fill0, keys, toks, S, slot, slot_token);
    return;
  }
  const int *s_off = s_extra;  // first copy of every segment
  select_in_registers(A, total, m, true, r, j, fill0, [&](int idx, u32 &kx, int &tok) {
    int a = 0, b = nseg - 1;  // segment whose copies hold position idx
    while (a < b) {
      const int mid = (a + b + 1) >> 1;
      if (s_off[mid] <= idx) a = mid; else b = mid - 1;
    }
    const int pos = base + a * kSegLen + (idx - s_off[a]);
    kx = comp_key[pos];
    tok = comp_tok[pos];
  }, S, slot, slot_token);
}

// ------------------------------------------------------------------ select_slot, small batches
// Up to SS_THREADS * SS_PER tokens and one capacity block per expert: the workgroup of list
// (round r, expert j) finds its candidates itself - it reads column r of rank_expert for every token,
// idx = u * SS_THREADS + tid being element u of thread tid, so candidates are met in token order -
// and counts expert j's candidates of the earlier rounds on the way (the kept count of a round is
// min(candidates, free slots)).  No candidate counts, no scan, no scatter: three launches fewer.
// The selection itself is that of select_slot_kernel's register path.
__global__ __launch_bounds__(SS_THREADS) void select_direct_kernel(DispatchArgs A,
                                                                   const int32_t *__restrict__ rank_expert,
                                                                   const u32 *__restrict__ key,
                                                                   int32_t *__restrict__ slot,
                                                                   int32_t *__restrict__ slot_token,
                                                                   int32_t *__restrict__ grp_fill,
                                                                   int32_t *__restrict__ grp_off,
                                                                   int32_t *__restrict__ fill_topk,
                                                                   int32_t *__restrict__ fill_total) {
  __shared__ u32 hist[kHistWords];
  __shared__ u32 s_pick[2];
  __shared__ int2 wtot[SS_PER][SS_WAVES];
  __shared__ int2 wsum[8];
  __shared__ int s_cnt[kMaxRounds];
  const int r = blockIdx.x / A.E, j = blockIdx.x - r * A.E;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nu = (A.T + SS_THREADS - 1) / SS_THREADS;
  if (tid < kMaxRounds) s_cnt[tid] = 0;
  __syncthreads();
  u32 member = 0;  // bit u: token u * SS_THREADS + tid is a candidate of this list
  u32 kreg[SS_PER];  // score keys of round r, fetched for every token in the same round trip as the ranks
  int c_rr[kMaxRounds];
#pragma unroll
  for (int rr = 0; rr < kMaxRounds; ++rr) c_rr[rr] = 0;
#pragma unroll
  for (int u = 0; u < SS_PER; ++u) {
    const int idx = u * SS_THREADS + tid;
    kreg[u] = 0;
    if (u < nu && idx < A.T) {
      kreg[u] = key[(size_t)idx * A.NR + r];
#pragma unroll
      for (int rr = 0; rr < kMaxRounds; ++rr)
        if (rr <= r && rank_expert[(size_t)idx * (A.k + 1) + rr] == j) {
          ++c_rr[rr];
          if (rr == r) member |= 1u << u;
        }
    }
  }
#pragma unroll
  for (int rr = 0; rr < kMaxRounds; ++rr) {
    if (rr <= r) {  // r is uniform over the workgroup
      int v = c_rr[rr];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
      if (lane == 0 && v) atomicAdd(&s_cnt[rr], v);
    }
  }
  __syncthreads();
  int n = 0, m = 0, fill = 0, topk = 0;
  for (int rr = 0; rr <= r; ++rr) {
    fill += m;
    n = s_cnt[rr];
    m = min(n, A.Cq - fill);
    if (rr == A.k - 1) topk = fill + m;
  }
  const int fill0 = fill;
  if (r == A.NR - 1 && tid == 0) {  // the expert's last round also writes its fill counts
    grp_fill[j] = fill + m;
    grp_off[j] = 0;
    fill_total[j] = fill + m;
    fill_topk[j] = topk;
  }
  const bool by_score = !A.arrival || r == A.k;  // the Fill-in round always selects by score (Sec. 4.2)
  const unsigned long long below = (1ull << lane) - 1ull;
  // mode 0: nobody kept; 1: everybody kept; 2: the first m in token order; 3: by score threshold
  const int mode = m == 0 ? 0 : (m == n ? 1 : (by_score ? 3 : 2));
  u32 thr = 0, need_eq = 0;
  if (mode == 3)
    thr = radix_select(m, [&](auto f) {
#pragma unroll
      for (int u = 0; u < SS_PER; ++u)
        if (u < nu) f(kreg[u], (member >> u) & 1u);
    }, hist, s_pick, need_eq);
  if (mode == 2) need_eq = (u32)m;  // arrival order: every candidate "ties", the first m of them are kept

  int pre[SS_PER];  // lanes of this wave before this one: kept-for-sure | equal << 8
#pragma unroll
  for (int u = 0; u < SS_PER; ++u) {
    pre[u] = 0;
    if (u < nu) {
      const bool cand = (member >> u) & 1u;
      bool gt = false, eq = false;
      if (mode == 3) { gt = cand && kreg[u] > thr; eq = cand && kreg[u] == thr; }
      else if (mode == 2) eq = cand;
      else gt = cand && mode == 1;
      const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
      pre[u] = __popcll(bgt & below) | (__popcll(beq & below) << 8) | (gt ? 1 << 16 : 0) | (eq ? 1 << 17 : 0);
      if (lane == 0) wtot[u][w] = make_int2(__popcll(bgt), __popcll(beq));
    }
  }
  __syncthreads();
  // exclusive scan of the nu * SS_WAVES totals in (trip, wave) order = token order
  const int ne = nu * SS_WAVES;
  int2 mine = make_int2(0, 0), incl = mine;
  if (tid < ne) mine = (&wtot[0][0])[tid];
  if (tid < 8 * kWave) {
    incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int tx = __shfl_up(incl.x, off), ty = __shfl_up(incl.y, off);
      if (lane >= off) { incl.x += tx; incl.y += ty; }
    }
    if (lane == 63) wsum[w] = incl;
  }
  __syncthreads();
  if (tid < ne) {
    int2 before = make_int2(0, 0);
    for (int q = 0; q < w; ++q) { before.x += wsum[q].x; before.y += wsum[q].y; }
    (&wtot[0][0])[tid] = make_int2(before.x + incl.x - mine.x, before.y + incl.y - mine.y);
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < SS_PER; ++u) {
    if (u < nu && ((member >> u) & 1u)) {
      const int tok = u * SS_THREADS + tid;
      const int2 base = wtot[u][w];
      const bool gt = (pre[u] >> 16) & 1, eq = (pre[u] >> 17) & 1;
      const int eqs = base.y + ((pre[u] >> 8) & 255);  // equal keys before this one
      const bool kept = gt || (eq && (u32)eqs < need_eq);
      const int sl = fill0 + base.x + (pre[u] & 255) + min(eqs, (int)need_eq);
      slot[(size_t)tok * (A.k + 1) + r] = kept ? sl : -1;
      if (kept) slot_token[(size_t)j * A.C + sl] = tok;
    }
  }
  // the last round pads the rest of the queue (Sec. 3: zero padding)
  if (r == A.NR - 1)
    for (int sl = fill0 + m + tid; sl < A.Cq; sl += SS_THREADS) slot_token[(size_t)j * A.C + sl] = -1;
}

// ------------------------------------------------------------------ Intra-GPU lists
__device__ inline int drops_of_token(const int32_t *slot, int i, int k) {
  int n = 0;
  for (int r = 0; r < k; ++r) n += slot[(size_t)i * (k + 1) + r] < 0;
  return n;
}

__global__ __launch_bounds__(kTokBlock) void ir_count_kernel(DispatchArgs A, const int32_t *__restrict__ slot,
                                                             const int32_t *__restrict__ ir_cand,
                                                             int32_t *__restrict__ ir_blk_cnt) {
  __shared__ int cnt[kMaxE];
  // neighbouring blocks write neighbouring words of the per-expert count rows: XCD-aware block order
  const int tid = threadIdx.x, b = xcd_block(blockIdx.x, A.NB);
  const int i = b * kTokBlock + tid;
  if (tid < kMaxE) cnt[tid] = 0;
  __syncthreads();
  if (i < A.T && drops_of_token(slot, i, A.k) > 0) atomicAdd(&cnt[ir_cand[i]], 1);
  __syncthreads();
  if (tid < A.E) ir_blk_cnt[(size_t)tid * A.NB + b] = cnt[tid];
}

// Dispatched-row layout: expert e owns rows [row_base[e], row_base[e+1]): its occupied capacity
// slots first, then its Intra-GPU rows.  One wave, lane e = expert e: the offsets of the experts'
// Intra-GPU lists go to s_off (LDS, every workgroup of ir_weights needs them); the wave that `writes`
// also stores them with row_base and cuts every expert's rows into tiles of BM rows (skipped when
// max_mtiles == 0: routing-only calls have no grouped GEMM).
__device__ inline void row_plan_wave(const DispatchArgs &A, bool writes, const int32_t *__restrict__ fill_total,
                                     const int32_t *__restrict__ ir_cnt, int *s_off, int *s_rbase,
                                     int32_t *__restrict__ ir_offset,
                                     int32_t *__restrict__ row_base, TileInfo *__restrict__ tiles,
                                     int32_t *__restrict__ tile_ctl) {
  const int e = threadIdx.x & 63;
  const bool on = e < A.E;
  const int nir = (on && A.ir) ? ir_cnt[e] : 0;
  const int fill = on ? fill_total[e] : 0;
  const int rows = fill + nir;
  const int ntile = A.max_mtiles > 0 ? (rows + A.BM - 1) / A.BM : 0;
  int s_ir = nir, s_rows = rows, s_tiles = ntile;  // inclusive scans over experts
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int a = __shfl_up(s_ir, off), b = __shfl_up(s_rows, off), c = __shfl_up(s_tiles, off);
    if (e >= off) { s_ir += a; s_rows += b; s_tiles += c; }
  }
  if (on) {
    s_off[e] = s_ir - nir;
    s_rbase[e] = s_rows - rows;
  }
  if (!writes) return;
  if (on) {
    ir_offset[e] = s_ir - nir;
    row_base[e] = s_rows - rows;
    int t = s_tiles - ntile;
    for (int m0 = 0; m0 < rows && ntile > 0 && t < A.max_mtiles; m0 += A.BM, ++t)
      tiles[t] = TileInfo{e, m0, s_rows - rows, rows, fill, s_ir - nir, 0, 0};
  }
  if (e == A.E - 1) {
    ir_offset[A.E] = s_ir;
    row_base[A.E] = s_rows;
    tile_ctl[0] = min(s_tiles, A.max_mtiles);
  }
}

// Per-group quotas only: the occupied slots of an expert are not a prefix of its queue, so the
// token behind every dispatched row is written out once (rows skip the holes between blocks).
__global__ __launch_bounds__(256) void row_token_kernel(DispatchArgs A, const int32_t *__restrict__ slot_token,
                                                        const int32_t *__restrict__ grp_fill,
                                                        const int32_t *__restrict__ grp_off,
                                                        const int32_t *__restrict__ fill_total,
                                                        const int32_t *__restrict__ ir_offset,
                                                        const int32_t *__restrict__ ir_token,
                                                        const int32_t *__restrict__ row_base,
                                                        int32_t *__restrict__ row_token) {
  const int e = blockIdx.x, base = row_base[e];
  for (int s = threadIdx.x; s < A.C; s += 256) {
    const int g = s / A.Cq, p = s - g * A.Cq;
    if (p < grp_fill[e * A.Gq + g]) row_token[base + grp_off[e * A.Gq + g] + p] = slot_token[(size_t)e * A.C + s];
  }
  const int nir = ir_offset[e + 1] - ir_offset[e], first = base + fill_total[e];
  for (int t = threadIdx.x; t < nir; t += 256) row_token[first + t] = ir_token[ir_offset[e] + t];
}

// Per token: Intra-GPU list position (Sec. 4.1) and the Eq. 2 / Eq. 3 weights.
__global__ __launch_bounds__(kTokBlock) void ir_weights_kernel(DispatchArgs A, const int32_t *__restrict__ slot,
                                                               const u32 *__restrict__ key,
                                                               const float *__restrict__ ir_score,
                                                               const int32_t *__restrict__ ir_cand,
                                                               const int32_t *__restrict__ ir_blk_off,
                                                               const int32_t *__restrict__ ir_cnt,
                                                               const int32_t *__restrict__ fill_total,
                                                               int32_t *__restrict__ ir_offset,
                                                               int32_t *__restrict__ row_base,
                                                               TileInfo *__restrict__ tiles,
                                                               int32_t *__restrict__ tile_ctl,
                                                               int32_t *__restrict__ ir_expert,
                                                               int32_t *__restrict__ ir_row,
                                                               int32_t *__restrict__ ir_token,
                                                               float *__restrict__ combine_w,
                                                               const int32_t *__restrict__ rank_expert,
                                                               const int32_t *__restrict__ grp_off,
                                                               int32_t *__restrict__ row_dest) {
  constexpr int NW = kTokBlock / kWave;
  __shared__ int wcnt[NW][kMaxE];
  __shared__ int s_off[kMaxE], s_rbase[kMaxE];
  const int tid = threadIdx.x, b = xcd_block(blockIdx.x, A.NB), w = tid >> 6;
  const int i = b * kTokBlock + tid;
  const bool valid = i < A.T;
  for (int c = tid; c < NW * kMaxE; c += kTokBlock) (&wcnt[0][0])[c] = 0;
  __shared__ int s_cnt[kMaxE], s_before[kMaxE];
  const bool self = A.ir_self && A.ir;
  if (self && tid < kMaxE) s_cnt[tid] = s_before[tid] = 0;
  // everything this token needs from global memory is fetched here, in one round trip, ahead of the
  // barriers (loads do not move across them)
  int slot_r[kMaxRank], cand = 0, ndrop = 0;
  u32 key_r[kMaxRank];
  float score_h = 0.0f;
#pragma unroll
  for (int r = 0; r < kMaxRank; ++r) {
    slot_r[r] = -1;
    key_r[r] = 0;
    if (valid && r < A.NR) {
      slot_r[r] = slot[(size_t)i * (A.k + 1) + r];
      key_r[r] = key[(size_t)i * A.NR + r];
    }
  }
  if (valid && A.ir) {
    cand = ir_cand[i];
    score_h = ir_score[i];
  }
  int e_r[kMaxRank];  // only for row_dest: the experts behind the token's slots
#pragma unroll
  for (int r = 0; r < kMaxRank; ++r) {
    e_r[r] = 0;
    if (row_dest && valid && r < A.NR) e_r[r] = rank_expert[(size_t)i * (A.k + 1) + r];
  }
#pragma unroll
  for (int r = 0; r < kMaxRank; ++r)
    if (r < A.k) ndrop += slot_r[r] < 0;
  const bool has_ir = valid && A.ir && ndrop > 0;
  const int h = has_ir ? cand : 0;
  unsigned long long mask = same_expert_mask(has_ir, h);
  const int below = lanes_below(mask);
  __syncthreads();
  if (has_ir && below == 0) wcnt[w][h] = __popcll(mask);
  // Small batches: ir_blk_off holds the raw per-block counts (at most a few thousand numbers) and
  // every workgroup adds up what it needs - the tokens of each expert's list in earlier blocks and
  // in all blocks - instead of a scan launch of its own in front of this kernel.
  if (self) {
    for (int idx = tid; idx < A.E * A.NB; idx += kTokBlock) {
      const int e = idx / A.NB, bb = idx - e * A.NB, v = ir_blk_off[idx];
      if (v) {
        atomicAdd(&s_cnt[e], v);
        if (bb < b) atomicAdd(&s_before[e], v);
      }
    }
    __syncthreads();
  }
  // the row plan is a few dozen numbers: every workgroup recomputes the list offsets it needs, the
  // first one also writes the plan out for the kernels that follow
  if (w == 0)
    row_plan_wave(A, blockIdx.x == 0, fill_total, self ? s_cnt : ir_cnt, s_off, s_rbase, ir_offset, row_base, tiles, tile_ctl);
  __syncthreads();
  if (!valid) return;
  float a_h = 0.0f;
  int my_ir_row = -1;
  if (has_ir) {
    int row = (A.ir_self ? s_before[h] : ir_blk_off[(size_t)h * A.NB + b]) + below;
    for (int q = 0; q < w; ++q) row += wcnt[q][h];
    ir_expert[i] = h;
    ir_row[i] = row;
    ir_token[s_off[h] + row] = i;
    a_h = score_h;
    my_ir_row = row;
  } else {
    ir_expert[i] = -1;
    ir_row[i] = -1;
  }
  if (row_dest) {
    // Every dispatched row belongs to one (token, assignment): the token marks each of its rows - with
    // its own index if this is the token's only row (Eq. 2 / Eq. 3 then give it weight exactly 1 and the
    // expert's output row IS the layer's output row: the down projection stores it there), else with -1.
    int nrows = has_ir ? 1 : 0;
#pragma unroll
    for (int r = 0; r < kMaxRank; ++r) nrows += (r < A.NR && slot_r[r] >= 0) ? 1 : 0;
    const int mark = nrows == 1 ? i : -1;
#pragma unroll
    for (int r = 0; r < kMaxRank; ++r) {
      if (r < A.NR && slot_r[r] >= 0) {
        const int e = e_r[r], g = slot_r[r] / A.Cq;
        row_dest[s_rbase[e] + grp_off[e * A.Gq + g] + (slot_r[r] - g * A.Cq)] = mark;
      }
    }
    if (has_ir) row_dest[s_rbase[h] + fill_total[h] + my_ir_row] = mark;
  }
  // Eq. 2 / Eq. 3: softmax over the successfully routed experts, a placed Fill-in expert, and the
  // Intra-GPU expert counted (k - |R_i|) times
  float a_r[kMaxRank];
  bool kept[kMaxRank];
  float mx = has_ir ? a_h : -INFINITY;
#pragma unroll
  for (int r = 0; r < kMaxRank; ++r) {
    kept[r] = false;
    a_r[r] = 0.0f;
    if (r < A.NR) {
      kept[r] = slot_r[r] >= 0;
      if (kept[r]) {
        a_r[r] = key_score(key_r[r]);
        mx = fmaxf(mx, a_r[r]);
      }
    }
  }
  float term[kMaxRank], t_ir = has_ir ? (float)ndrop * expf(a_h - mx) : 0.0f, Z = t_ir;
#pragma unroll
  for (int r = 0; r < kMaxRank; ++r) {
    term[r] = kept[r] ? expf(a_r[r] - mx) : 0.0f;
    Z += term[r];
  }
  const float inv = Z > 0.0f ? 1.0f / Z : 0.0f;
  float *cw = combine_w + (size_t)i * (A.k + 2);
#pragma unroll
  for (int r = 0; r < kMaxRank; ++r)
    if (r <= A.k) cw[r] = term[r] * inv;
  cw[A.k + 1] = t_ir * inv;
}

}  // namespace

hipError_t launch_dispatch(const Dims &D, const float *logits, const rr_tables &tb, const Work &W, bool ranked,
                           int32_t *row_dest, hipStream_t s) {
  DispatchArgs A{D.T, D.E, D.k, D.C, D.NR, D.NCAT, D.NB, D.Eg, D.Tg, D.ir, D.fr, D.arrival, D.BM, D.max_mtiles,
                 D.Cq, D.Gq, D.NL, D.NBc, D.cb, D.E * D.NB <= kIrSelfMax ? 1 : 0,
                 D.Gq == 1 && D.T <= kDirectMaxT ? 1 : 0};
  if (!ranked) {  // otherwise the router's epilogue has already written what topk_rank writes
    prof_begin(K_TOPK, s);
    topk_rank_kernel<<<D.NB, kTokBlock, 0, s>>>(logits, A, tb.rank_expert, tb.slot, W.key, W.ir_score, W.ir_cand,
                                                W.blk_cnt);
    prof_end(K_TOPK, s);
  }
  if (A.direct) {
    prof_begin(K_SELECT_SLOT, s);
    select_direct_kernel<<<D.NCAT, SS_THREADS, 0, s>>>(A, tb.rank_expert, W.key, tb.slot, tb.slot_token, W.grp_fill,
                                                       W.grp_off, tb.fill_topk, tb.fill_total);
    prof_end(K_SELECT_SLOT, s);
  } else {
    prof_begin(K_SCAN_CAND, s);
    // (also clears the tickets of the lists' segments: Gq lists per candidate array)
    scan_blocks_kernel<<<D.NCAT, SC_THREADS, 0, s>>>(W.blk_cnt, W.cat_cnt, D.NBc, W.list_done, D.Gq);
    prof_end(K_SCAN_CAND, s);
    prof_begin(K_SCATTER_CAND, s);
    scatter_candidates_kernel<<<D.NB, kTokBlock, 0, s>>>(A, tb.rank_expert, W.key, W.blk_cnt, W.cat_cnt, W.cand_key,
                                                         W.cand_tok, tb.slot, tb.slot_token);
    prof_end(K_SCATTER_CAND, s);
    prof_begin(K_SELECT_SLOT, s);
    // one workgroup per list, plus one for every further segment that a long list can have
    const int sel_grid = D.NL + (select_splits(D.T, D.NR, D.NL) ? (int)((long long)D.T * D.NR / kSelectSegLen) : 0);
    select_slot_kernel<<<sel_grid, SS_THREADS, 0, s>>>(A, W.cat_cnt, W.blk_cnt, W.cand_key, W.cand_tok, W.comp_key,
                                                       W.comp_tok, W.seg_cnt, W.list_done, tb.slot, tb.slot_token,
                                                       W.grp_fill, W.grp_off, tb.fill_topk, tb.fill_total);
    prof_end(K_SELECT_SLOT, s);
  }
  if (D.ir) {
    prof_begin(K_IR_COUNT, s);
    ir_count_kernel<<<D.NB, kTokBlock, 0, s>>>(A, tb.slot, W.ir_cand, W.ir_blk_cnt);
    prof_end(K_IR_COUNT, s);
    if (!A.ir_self) {
      prof_begin(K_IR_SCAN, s);
      scan_blocks_kernel<<<D.E, SC_THREADS, 0, s>>>(W.ir_blk_cnt, W.ir_cnt, D.NB, nullptr, 0);
      prof_end(K_IR_SCAN, s);
    }
  }
  prof_begin(K_IR_WEIGHTS, s);
  ir_weights_kernel<<<D.NB, kTokBlock, 0, s>>>(A, tb.slot, W.key, W.ir_score, W.ir_cand, W.ir_blk_cnt, W.ir_cnt,
                                               tb.fill_total, tb.ir_offset, W.row_base, W.tiles, W.tile_ctl,
                                               tb.ir_expert, tb.ir_row, tb.ir_token, tb.combine_w, tb.rank_expert,
                                               W.grp_off, row_dest);
  prof_end(K_IR_WEIGHTS, s);
  if (D.quota && D.max_mtiles > 0)  // the forward pass addresses dispatched rows through row_token
    row_token_kernel<<<D.E, 256, 0, s>>>(A, tb.slot_token, W.grp_fill, W.grp_off, tb.fill_total, tb.ir_offset,
                                         tb.ir_token, W.row_base, W.row_token);
  return hipGetLastError();
}

}  // namespace rr
