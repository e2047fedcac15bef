"""CPU oracle for the Rectify-Router MoE layer forward (arXiv 2402.12399).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
HIP path is checked against.  Only tests, the smoke check and the CPU-baseline
leg of the benchmark may import it; the product path never does.  It shares no
code with the HIP library and imports nothing from the package.

All floating-point arithmetic is float64 (numpy) except that
  * router scores are rounded once to float32 after the float64 dot product
    (they are the fp32 "logits" that every routing decision compares), and
  * every comparison between scores is done on those float32 values with
    IEEE `>` / `==` (so -0.0 and +0.0 tie).

Each function follows one passage of the paper, in the paper's order:

  capacity()            Sec. 3, capacity formula
  router_scores()       Sec. 3, Eq. 1 (a_ij = w_j^T x_i)
  rank_experts()        Sec. 3, Eq. 1 (argtopk) and Sec. 4.2 stage 1 ((k+1)-th)
  topk_capacity_rounds() Sec. 3 "Dropped Tokens and Padding"; Sec. 4.1
                        ("first routing", "second routing")
  intra_gpu_rectification()  Sec. 4.1
  fill_in_rectification()    Sec. 4.2 (stage 1: nomination, stage 2: selection)
  topk_capacity_rounds_quota(), fill_in_rectification_quota()
                        the same two steps with the capacity of Sec. 3 read per GPU
  combine_weights()     Eq. 2 and Eq. 3
  expert_ffn()          Sec. 5.1 "Model": experts are LLaMA FFNs (SwiGLU)
  moe_output()          Eq. 2 / Eq. 3 applied to expert outputs
  router_score_gradient()  App. A (Eq. 5, Eq. 6): gradient of a loss with respect to
                        the router scores through the Eq. 2 / Eq. 3 weights

Readings taken where the paper is silent (each one is also a flag or a
documented rule of the HIP library):
  * scores compared across tokens are the raw a_ij, never the softmax;
  * ties between experts -> lower expert index; between tokens -> lower token
    index;
  * capacity = ceil(capacity_factor * T / E) evaluated in float64 with the
    capacity factor first rounded to float32, minimum 1;
  * rank-major rounds: every token's r-th choice is placed before any token's
    (r+1)-th choice; an expert keeps its best candidates of the round (policy
    "score") or its earliest candidates (policy "arrival");
  * kept tokens of a round occupy consecutive slots in ascending token index;
  * token i lives on group i // (T/G), expert j on group j // (E/G);
  * Intra-GPU Rectification excludes no expert of the group (it may pick an
    expert that already serves, or that dropped, the token);
  * every token nominates its (k+1)-th expert for Fill-in, kept or not;
  * with both rectifications, (k - |R_i|) counts top-k drops only and a placed
    fill-in joins the sum over R_i;
  * capacity competition is global by default (one queue of C slots per expert
    over all T tokens, Fig. 1).  The variant quota=True reads the capacity
    formula of Sec. 3 per GPU, as expert-parallel implementations do: every
    group g owns Cq = capacity(T/G, E, capacity_factor) slots of every expert,
    slots [g Cq, (g+1) Cq) of that expert's queue of G Cq slots, and only the
    group's own tokens compete for them, in the top-k rounds and in Fill-in.

  * App. A, Eq. 6 (printed garbled): the weight of a processed assignment is
    n g_ij / S_i with g the softmax over ALL experts (Eq. 5), n its
    multiplicity (1, or k - |R_i| for the Intra-GPU expert) and
    S_i = sum over the token's processed assignments of n g_ij; the forward
    value is that of Eq. 2 / Eq. 3.  In the backward pass S_i is a constant.
    The routing decisions themselves (which experts, which tokens are kept)
    carry no gradient.

Parity pins (tests/test_oracle_*.py): a hand-worked capacity-3 example
(tests/golden/), brute-force subset enumeration on tiny inputs, the
"top-(k+1) router at unchanged capacity" formulation of Fill-in, the G=1
special case of Intra-GPU Rectification, counting identities, the
no-drop dense-mixture closed form, and the identical-experts closed form;
for router_score_gradient() central differences of the loss it differentiates,
automatic differentiation of the same expressions, the dense-mixture softmax
gradient and the single-expert cases App. A describes.
The choice between the alternative readings listed above is "parity unpinned":
the paper prints no number that discriminates them.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

POLICY_SCORE = "score"
POLICY_ARRIVAL = "arrival"


# ----------------------------------------------------------------------------
# Sec. 3: capacity = capacity factor x tokens / experts
# ----------------------------------------------------------------------------
def capacity(T: int, E: int, capacity_factor: float) -> int:
    cf = float(np.float32(capacity_factor))
    return max(1, int(math.ceil(cf * float(T) / float(E))))


# ----------------------------------------------------------------------------
# Sec. 3, Eq. 1: a_ij = w_j^T x_i  (+ optional per-expert bias used by the
# synthetic workloads to skew the load; the paper has no bias)
# ----------------------------------------------------------------------------
def router_scores(x: np.ndarray, w_router: np.ndarray, bias: np.ndarray | None = None) -> np.ndarray:
    a = np.asarray(x, dtype=np.float64) @ np.asarray(w_router, dtype=np.float64).T
    if bias is not None:
        a = a + np.asarray(bias, dtype=np.float64)[None, :]
    return a.astype(np.float32)


def softmax_probs(a: np.ndarray) -> np.ndarray:
    """App. A, Eq. 5: g_ij = exp(a_ij) / sum_j exp(a_ij) over all experts."""
    a64 = np.asarray(a, dtype=np.float64)
    z = np.exp(a64 - a64.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


# ----------------------------------------------------------------------------
# Eq. 1 argtopk, extended by one rank for Fill-in stage 1 (Sec. 4.2)
# ----------------------------------------------------------------------------
def rank_experts(a: np.ndarray, n_ranks: int) -> np.ndarray:
    """Experts of each token by descending score, ties -> lower expert index.

    Returns int32 [T, n_ranks]; columns beyond E are -1.
    """
    a = np.asarray(a, dtype=np.float32)
    T, E = a.shape
    order = np.argsort(-a, axis=1, kind="stable")  # stable: equal scores keep ascending j
    out = np.full((T, n_ranks), -1, dtype=np.int32)
    n = min(n_ranks, E)
    out[:, :n] = order[:, :n]
    return out


def _best_first(cand: np.ndarray, score: np.ndarray, policy: str) -> np.ndarray:
    """Candidates (ascending token index) reordered best-first for one expert."""
    if policy == POLICY_ARRIVAL:
        return cand
    # primary key: score descending; secondary: token index ascending
    return cand[np.lexsort((cand, -score))]


# ----------------------------------------------------------------------------
# Sec. 3 "Dropped Tokens and Padding" + Sec. 4.1: k routing rounds under a
# fixed capacity.  Overflowing experts drop their lowest-scoring candidates.
# ----------------------------------------------------------------------------
def topk_capacity_rounds(a, rank_expert, k, C, policy=POLICY_SCORE):
    a = np.asarray(a, dtype=np.float32)
    T, E = a.shape
    slot = np.full((T, k + 1), -1, dtype=np.int32)
    slot_token = np.full((E, C), -1, dtype=np.int32)
    fill = np.zeros(E, dtype=np.int32)
    for r in range(k):
        for j in range(E):
            cand = np.flatnonzero(rank_expert[:, r] == j)
            m = min(len(cand), C - int(fill[j]))
            kept = np.sort(_best_first(cand, a[cand, j], policy)[:m])
            slot[kept, r] = fill[j] + np.arange(m, dtype=np.int32)
            slot_token[j, fill[j]:fill[j] + m] = kept
            fill[j] += m
    return slot, slot_token, fill


# ----------------------------------------------------------------------------
# Sec. 4.1: every token dropped at least once goes to the best-scoring expert
# of its own GPU (group); once per token; no capacity limit.
# ----------------------------------------------------------------------------
def intra_gpu_rectification(a, slot, k, G):
    a = np.asarray(a, dtype=np.float32)
    T, E = a.shape
    Eg, Tg = E // G, T // G
    n_drop = (slot[:, :k] < 0).sum(axis=1).astype(np.int32)
    ir_expert = np.full(T, -1, dtype=np.int32)
    ir_row = np.full(T, -1, dtype=np.int32)
    lists = [[] for _ in range(E)]
    for i in np.flatnonzero(n_drop > 0):
        g = i // Tg
        h = g * Eg + int(np.argmax(a[i, g * Eg:(g + 1) * Eg]))  # first maximum -> lower j
        ir_expert[i] = h
        ir_row[i] = len(lists[h])
        lists[h].append(i)
    ir_offset = np.zeros(E + 1, dtype=np.int32)
    for j in range(E):
        ir_offset[j + 1] = ir_offset[j] + len(lists[j])
    ir_token = np.array([i for l in lists for i in l], dtype=np.int32)
    return n_drop, ir_expert, ir_row, ir_offset, ir_token


# ----------------------------------------------------------------------------
# Sec. 4.2: stage 1 - each token nominates its (k+1)-th expert; stage 2 - each
# expert replaces its padding with the highest-scoring nominees.
# ----------------------------------------------------------------------------
def fill_in_rectification(a, rank_expert, k, C, slot, slot_token, fill_topk):
    a = np.asarray(a, dtype=np.float32)
    T, E = a.shape
    slot = slot.copy()
    slot_token = slot_token.copy()
    fill = fill_topk.copy()
    nominee = rank_expert[:, k]
    for j in range(E):
        cand = np.flatnonzero(nominee == j)
        vacancy = C - int(fill_topk[j])
        m = min(len(cand), vacancy)
        chosen = np.sort(_best_first(cand, a[cand, j], POLICY_SCORE)[:m])
        slot[chosen, k] = fill_topk[j] + np.arange(m, dtype=np.int32)
        slot_token[j, fill_topk[j]:fill_topk[j] + m] = chosen
        fill[j] += m
    return slot, slot_token, fill


# ----------------------------------------------------------------------------
# Eq. 2 (top-k, normalised over the successfully routed set R_i) and Eq. 3
# (Intra-GPU term weighted by k - |R_i|).
# ----------------------------------------------------------------------------
def combine_weights(a, rank_expert, slot, k, n_drop, ir_expert):
    """float64 [T, k+2]: columns 0..k-1 top-k ranks, k fill-in, k+1 Intra-GPU."""
    a64 = np.asarray(a, dtype=np.float32).astype(np.float64)
    T, E = a64.shape
    row_max = a64.max(axis=1)
    terms = np.zeros((T, k + 2), dtype=np.float64)
    tok = np.arange(T)
    for r in range(k + 1):
        kept = slot[:, r] >= 0
        terms[kept, r] = np.exp(a64[tok[kept], rank_expert[kept, r]] - row_max[kept])
    has_ir = ir_expert >= 0
    terms[has_ir, k + 1] = n_drop[has_ir] * np.exp(a64[tok[has_ir], ir_expert[has_ir]] - row_max[has_ir])
    Z = terms.sum(axis=1)
    cw = np.zeros_like(terms)
    live = Z > 0
    cw[live] = terms[live] / Z[live, None]
    return cw


# ----------------------------------------------------------------------------
# Sec. 3 capacity read per GPU (quota variant): the rounds of topk_capacity_rounds
# and the selection of fill_in_rectification, run for every (group, expert) pair
# on the group's own tokens and the group's own Cq slots of the expert's queue.
# ----------------------------------------------------------------------------
def topk_capacity_rounds_quota(a, rank_expert, k, Cq, G, policy=POLICY_SCORE):
    a = np.asarray(a, dtype=np.float32)
    T, E = a.shape
    Tg = T // G
    slot = np.full((T, k + 1), -1, dtype=np.int32)
    slot_token = np.full((E, G * Cq), -1, dtype=np.int32)
    fill = np.zeros((G, E), dtype=np.int32)  # occupied slots of group g's block of expert j
    group = np.arange(T) // Tg
    for r in range(k):
        for g in range(G):
            for j in range(E):
                cand = np.flatnonzero((rank_expert[:, r] == j) & (group == g))
                m = min(len(cand), Cq - int(fill[g, j]))
                kept = np.sort(_best_first(cand, a[cand, j], policy)[:m])
                first = g * Cq + int(fill[g, j])
                slot[kept, r] = first + np.arange(m, dtype=np.int32)
                slot_token[j, first:first + m] = kept
                fill[g, j] += m
    return slot, slot_token, fill


def fill_in_rectification_quota(a, rank_expert, k, Cq, G, slot, slot_token, fill_topk):
    a = np.asarray(a, dtype=np.float32)
    T, E = a.shape
    Tg = T // G
    slot = slot.copy()
    slot_token = slot_token.copy()
    fill = fill_topk.copy()
    nominee = rank_expert[:, k]
    group = np.arange(T) // Tg
    for g in range(G):
        for j in range(E):
            cand = np.flatnonzero((nominee == j) & (group == g))
            m = min(len(cand), Cq - int(fill_topk[g, j]))
            chosen = np.sort(_best_first(cand, a[cand, j], POLICY_SCORE)[:m])
            first = g * Cq + int(fill_topk[g, j])
            slot[chosen, k] = first + np.arange(m, dtype=np.int32)
            slot_token[j, first:first + m] = chosen
            fill[g, j] += m
    return slot, slot_token, fill


def route(a, k, G, capacity_factor, intra_gpu=True, fill_in=True, policy=POLICY_SCORE, quota=False):
    """Logits -> every routing / rectification / dispatch table (Sec. 3, 4).

    quota=True: per-group capacity; C in the result is then the number of slots per expert, G Cq,
    and fill_topk / fill_total are summed over groups (fill_topk_group / fill_total_group [G,E]
    hold the per-group counts)."""
    a = np.asarray(a, dtype=np.float32)
    assert np.isfinite(a).all(), "logits must be finite"
    T, E = a.shape
    assert E % G == 0 and T % G == 0 and 1 <= k <= E
    assert not fill_in or k + 1 <= E
    if quota:
        return _route_quota(a, k, G, capacity_factor, intra_gpu, fill_in, policy)
    C = capacity(T, E, capacity_factor)
    rank_expert = rank_experts(a, k + 1)
    slot, slot_token, fill_topk = topk_capacity_rounds(a, rank_expert, k, C, policy)
    if intra_gpu:
        n_drop, ir_expert, ir_row, ir_offset, ir_token = intra_gpu_rectification(a, slot, k, G)
    else:
        n_drop = (slot[:, :k] < 0).sum(axis=1).astype(np.int32)
        ir_expert = np.full(T, -1, dtype=np.int32)
        ir_row = np.full(T, -1, dtype=np.int32)
        ir_offset = np.zeros(E + 1, dtype=np.int32)
        ir_token = np.zeros(0, dtype=np.int32)
    if fill_in:
        slot, slot_token, fill_total = fill_in_rectification(a, rank_expert, k, C, slot, slot_token, fill_topk)
    else:
        fill_total = fill_topk.copy()
    cw = combine_weights(a, rank_expert, slot, k, n_drop, ir_expert)
    return dict(C=C, rank_expert=rank_expert, slot=slot, slot_token=slot_token,
                fill_topk=fill_topk, fill_total=fill_total, n_drop=n_drop,
                ir_expert=ir_expert, ir_row=ir_row, ir_offset=ir_offset, ir_token=ir_token,
                combine_w=cw)


def _route_quota(a, k, G, capacity_factor, intra_gpu, fill_in, policy):
    T, E = a.shape
    Cq = capacity(T // G, E, capacity_factor)
    rank_expert = rank_experts(a, k + 1)
    slot, slot_token, fill_topk_g = topk_capacity_rounds_quota(a, rank_expert, k, Cq, G, policy)
    if intra_gpu:
        n_drop, ir_expert, ir_row, ir_offset, ir_token = intra_gpu_rectification(a, slot, k, G)
    else:
        n_drop = (slot[:, :k] < 0).sum(axis=1).astype(np.int32)
        ir_expert = np.full(T, -1, dtype=np.int32)
        ir_row = np.full(T, -1, dtype=np.int32)
        ir_offset = np.zeros(E + 1, dtype=np.int32)
        ir_token = np.zeros(0, dtype=np.int32)
    if fill_in:
        slot, slot_token, fill_total_g = fill_in_rectification_quota(a, rank_expert, k, Cq, G, slot, slot_token,
                                                                     fill_topk_g)
    else:
        fill_total_g = fill_topk_g.copy()
    cw = combine_weights(a, rank_expert, slot, k, n_drop, ir_expert)
    return dict(C=G * Cq, Cq=Cq, rank_expert=rank_expert, slot=slot, slot_token=slot_token,
                fill_topk=fill_topk_g.sum(axis=0).astype(np.int32), fill_total=fill_total_g.sum(axis=0).astype(np.int32),
                fill_topk_group=fill_topk_g, fill_total_group=fill_total_g, n_drop=n_drop,
                ir_expert=ir_expert, ir_row=ir_row, ir_offset=ir_offset, ir_token=ir_token, combine_w=cw)


# ----------------------------------------------------------------------------
# Sec. 5.1: each expert is a LLaMA FFN (gate/up/down, SiLU, no bias).  The tiny
# fp32 workload uses a two-matrix GELU FFN (exact erf form) instead.
# ----------------------------------------------------------------------------
def expert_ffn(x_rows, w1, w3, w2, act):
    """x_rows [n,d]; w1,w3 [F,d]; w2 [d,F].  float64 in, float64 out."""
    x_rows = np.asarray(x_rows, dtype=np.float64)
    g = x_rows @ np.asarray(w1, dtype=np.float64).T
    if act == "swiglu":
        u = x_rows @ np.asarray(w3, dtype=np.float64).T
        h = g / (1.0 + np.exp(-g)) * u
    elif act == "gelu":
        h = 0.5 * g * (1.0 + _erf(g / math.sqrt(2.0)))
    else:
        raise ValueError(act)
    return h @ np.asarray(w2, dtype=np.float64).T


# ----------------------------------------------------------------------------
# Eq. 2 / Eq. 3: o_i = sum of weighted expert outputs; a token that no expert
# processes gets 0 (its value travels by the block's residual connection).
# ----------------------------------------------------------------------------
def moe_output(x, tables, k, w1, w3, w2, act, tokens=None):
    """Outputs for `tokens` (default: all). Returns float64 [len(tokens), d]."""
    x = np.asarray(x)
    T, d = x.shape
    E = w1.shape[0]
    tokens = np.arange(T) if tokens is None else np.asarray(tokens)
    rank_expert, slot, cw = tables["rank_expert"], tables["slot"], tables["combine_w"]
    ir_expert = tables["ir_expert"]
    out = np.zeros((len(tokens), d), dtype=np.float64)
    for j in range(E):
        w = np.zeros(len(tokens), dtype=np.float64)
        for r in range(k + 1):
            sel = (rank_expert[tokens, r] == j) & (slot[tokens, r] >= 0)
            w[sel] += cw[tokens[sel], r]
        sel = ir_expert[tokens] == j
        w[sel] += cw[tokens[sel], k + 1]
        rows = np.flatnonzero(w != 0.0)
        if len(rows) == 0:
            continue
        y = expert_ffn(x[tokens[rows]], w1[j], None if w3 is None else w3[j], w2[j], act)
        out[rows] += w[rows, None] * y
    return out


def moe_forward(x, w_router, bias, w1, w3, w2, k, G, capacity_factor, act,
                intra_gpu=True, fill_in=True, policy=POLICY_SCORE, tokens=None, quota=False):
    a = router_scores(x, w_router, bias)
    tables = route(a, k, G, capacity_factor, intra_gpu, fill_in, policy, quota)
    out = moe_output(x, tables, k, w1, w3, w2, act, tokens)
    return a, tables, out


# ----------------------------------------------------------------------------
# App. A: gradient of a loss L with respect to the router scores a_ij, through
# the weights of Eq. 2 / Eq. 3 only (routing decisions are piecewise constant).
# The processed assignments of token i are p = (expert e_p, multiplicity n_p):
# kept top-k ranks and a placed fill-in with n = 1, the Intra-GPU expert with
# n = k - |R_i| (Eq. 3).  Eq. 2 / Eq. 3: o_i = sum_p c_ip E_{e_p}(x_i), so
#   dL/dc_ip = <dL/do_i, E_{e_p}(x_i)>.
# ----------------------------------------------------------------------------
def processed_assignments(tables, k, i):
    """[(column of combine_w, expert, multiplicity)] of token i."""
    out = []
    for r in range(k + 1):
        if tables["slot"][i, r] >= 0:
            out.append((r, int(tables["rank_expert"][i, r]), 1.0))
    if tables["ir_expert"][i] >= 0:
        out.append((k + 1, int(tables["ir_expert"][i]), float(tables["n_drop"][i])))
    return out


def router_score_gradient(x, a, tables, k, w1, w3, w2, act, dout, straight_through=True, tokens=None):
    """Returns (dL/dc [n, k+2], dL/da [n, E]) for `tokens` (default: all), float64.

    straight_through=True: App. A, Eq. 6.  c_ip = n_p g_{i,e_p} / S_i with g the softmax over all
    experts (Eq. 5); S_i is held constant, so dL/dg_ij = sum_{p: e_p = j} n_p dL/dc_ip / S_i, and
    dL/da_il = sum_j dL/dg_ij dg_ij/da_il with the softmax Jacobian dg_ij/da_il = g_ij ([j = l] - g_il).
    straight_through=False: the plain derivative of the normalised weights
    c_ip = n_p exp(a_{i,e_p}) / Z_i, Z_i = sum_q n_q exp(a_{i,e_q}) (quotient rule)."""
    x = np.asarray(x)
    a64 = np.asarray(a, dtype=np.float32).astype(np.float64)
    T, E = a64.shape
    tokens = np.arange(T) if tokens is None else np.asarray(tokens)
    g = softmax_probs(a64)
    dc = np.zeros((len(tokens), k + 2), dtype=np.float64)
    da = np.zeros((len(tokens), E), dtype=np.float64)
    assigned = [processed_assignments(tables, k, i) for i in tokens]
    # dL/dc_ip = <dL/do_i, E_j(x_i)>, one expert at a time over the tokens it processes
    for j in range(E):
        users = [(n, col) for n, P in enumerate(assigned) for col, e, _ in P if e == j]
        if not users:
            continue
        rows = np.array(sorted({n for n, _ in users}))
        y = expert_ffn(x[tokens[rows]], w1[j], None if w3 is None else w3[j], w2[j], act)
        proj = dict(zip(rows.tolist(), (y * np.asarray(dout[tokens[rows]], dtype=np.float64)).sum(axis=1)))
        for n, col in users:
            dc[n, col] = proj[n]
    for n, i in enumerate(tokens):
        P = assigned[n]
        if not P:
            continue
        if straight_through:
            S = sum(mult * g[i, e] for _, e, mult in P)
            dg = np.zeros(E, dtype=np.float64)
            for col, e, mult in P:
                dg[e] += mult * dc[n, col] / S
            jac = np.diag(g[i]) - np.outer(g[i], g[i])  # jac[j, l] = dg_ij / da_il
            da[n] = dg @ jac
        else:
            t = np.array([mult * math.exp(a64[i, e] - a64[i].max()) for _, e, mult in P])
            Z = t.sum()
            c = t / Z
            for p, (col, e, mult) in enumerate(P):
                # dc_p/da_l = [e_p = l] c_p - c_p * sum_{q: e_q = l} c_q
                da[n, e] += dc[n, col] * c[p]
                for q, (_, eq, _) in enumerate(P):
                    da[n, eq] -= dc[n, col] * c[p] * c[q]
    return dc, da
