"""Are the oracle's pins strong enough?  Each case plants one plausible mistake in the CPU oracle
(a flipped comparison, a dropped factor, a wrong tie-break, a transposed operand ...) and re-runs
the pin tests of test_oracle_pins.py against the mutated module: at least one pin must fail.

Everything here runs on the CPU and touches only the oracle; the mistakes are never planted in the
HIP path.
"""
import inspect
import math

import numpy as np
import pytest

from oracle import rectify_router as orc
from tests import test_oracle_pins as pins


# ------------------------------------------------------------------ running the pins by hand
def _param_sets(fn):
    """Argument dictionaries of a test function from its parametrize marks (their cross product)."""
    sets = [{}]
    for mark in getattr(fn, "pytestmark", []):
        if mark.name != "parametrize":
            continue
        names = [n.strip() for n in mark.args[0].split(",")] if isinstance(mark.args[0], str) else list(mark.args[0])
        values = [v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,) for v in mark.args[1]]
        sets = [dict(s, **dict(zip(names, v))) for s in sets for v in values]
    return sets


def _golden():
    import json
    with open(pins.GOLDEN) as f:
        return json.load(f)


def pins_catch_it():
    """True as soon as one pin test fails against the oracle module as it currently is."""
    golden = _golden()
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_"):
            continue
        wants = inspect.signature(fn).parameters
        for args in _param_sets(fn):
            if "golden" in wants:
                args = dict(args, golden=golden)
            try:
                fn(**args)
            except Exception:  # an assertion, or the mutated oracle tripping over itself
                return True
    return False


def test_unmutated_oracle_passes_every_pin():
    assert not pins_catch_it()


# ------------------------------------------------------------------ the planted mistakes
def m_keep_lowest_scores(mp):
    def best_first(cand, score, policy):
        if policy == orc.POLICY_ARRIVAL:
            return cand
        return cand[np.lexsort((cand, score))]  # ascending score: the best are dropped
    mp.setattr(orc, "_best_first", best_first)


def m_token_tie_break_reversed(mp):
    def best_first(cand, score, policy):
        if policy == orc.POLICY_ARRIVAL:
            return cand
        return cand[np.lexsort((-cand, -score))]  # equal scores: the LATER token wins
    mp.setattr(orc, "_best_first", best_first)


def m_expert_tie_break_reversed(mp):
    def rank_experts(a, n_ranks):
        a = np.asarray(a, dtype=np.float32)
        T, E = a.shape
        order = (E - 1) - np.argsort(-a[:, ::-1], axis=1, kind="stable")  # equal scores: HIGHER expert first
        out = np.full((T, n_ranks), -1, dtype=np.int32)
        n = min(n_ranks, E)
        out[:, :n] = order[:, :n]
        return out
    mp.setattr(orc, "rank_experts", rank_experts)


def m_capacity_floor(mp):
    mp.setattr(orc, "capacity", lambda T, E, cf: max(1, int(math.floor(float(np.float32(cf)) * T / E))))


def m_slots_in_score_order(mp):
    def rounds(a, rank_expert, k, C, policy=orc.POLICY_SCORE):
        a = np.asarray(a, dtype=np.float32)
        T, E = a.shape
        slot = np.full((T, k + 1), -1, dtype=np.int32)
        slot_token = np.full((E, C), -1, dtype=np.int32)
        fill = np.zeros(E, dtype=np.int32)
        for r in range(k):
            for j in range(E):
                cand = np.flatnonzero(rank_expert[:, r] == j)
                m = min(len(cand), C - int(fill[j]))
                kept = orc._best_first(cand, a[cand, j], policy)[:m]  # not re-sorted by token index
                slot[kept, r] = fill[j] + np.arange(m, dtype=np.int32)
                slot_token[j, fill[j]:fill[j] + m] = kept
                fill[j] += m
        return slot, slot_token, fill
    mp.setattr(orc, "topk_capacity_rounds", rounds)


def m_rounds_forget_earlier_fill(mp):
    def rounds(a, rank_expert, k, C, policy=orc.POLICY_SCORE):
        a = np.asarray(a, dtype=np.float32)
        T, E = a.shape
        slot = np.full((T, k + 1), -1, dtype=np.int32)
        slot_token = np.full((E, C), -1, dtype=np.int32)
        fill = np.zeros(E, dtype=np.int32)
        for j in range(E):  # expert-major: one global score order per expert instead of rank-major rounds
            cand = np.array([(i, r) for r in range(k) for i in np.flatnonzero(rank_expert[:, r] == j)], dtype=np.int64)
            if len(cand) == 0:
                continue
            order = np.lexsort((cand[:, 0], -a[cand[:, 0], j]))
            kept = cand[order][:C]
            kept = kept[np.argsort(kept[:, 0], kind="stable")]
            for s, (i, r) in enumerate(kept):
                slot[i, r] = s
                slot_token[j, s] = i
            fill[j] = len(kept)
        return slot, slot_token, fill
    mp.setattr(orc, "topk_capacity_rounds", rounds)


def _ir_with(group_of, candidates_of, trigger):
    def ir(a, slot, k, G):
        a = np.asarray(a, dtype=np.float32)
        T, E = a.shape
        n_drop = (slot[:, :k] < 0).sum(axis=1).astype(np.int32)
        ir_expert = np.full(T, -1, dtype=np.int32)
        ir_row = np.full(T, -1, dtype=np.int32)
        lists = [[] for _ in range(E)]
        for i in np.flatnonzero(trigger(n_drop, k)):
            lo, hi = candidates_of(group_of(i, T, G), E, G)
            h = lo + int(np.argmax(a[i, lo:hi]))
            ir_expert[i] = h
            ir_row[i] = len(lists[h])
            lists[h].append(i)
        ir_offset = np.zeros(E + 1, dtype=np.int32)
        for j in range(E):
            ir_offset[j + 1] = ir_offset[j] + len(lists[j])
        ir_token = np.array([i for l in lists for i in l], dtype=np.int32)
        return n_drop, ir_expert, ir_row, ir_offset, ir_token
    return ir


_block_group = lambda i, T, G: i // (T // G)
_own_experts = lambda g, E, G: (g * (E // G), (g + 1) * (E // G))
_any_drop = lambda n_drop, k: n_drop > 0


def m_ir_tokens_interleaved_over_groups(mp):
    mp.setattr(orc, "intra_gpu_rectification", _ir_with(lambda i, T, G: i % G, _own_experts, _any_drop))


def m_ir_ignores_groups(mp):
    mp.setattr(orc, "intra_gpu_rectification", _ir_with(_block_group, lambda g, E, G: (0, E), _any_drop))


def m_ir_only_when_all_choices_dropped(mp):
    mp.setattr(orc, "intra_gpu_rectification", _ir_with(_block_group, _own_experts, lambda n_drop, k: n_drop == k))


def _fill_in_with(nominates, vacancy_of):
    def fr(a, rank_expert, k, C, slot, slot_token, fill_topk):
        a = np.asarray(a, dtype=np.float32)
        T, E = a.shape
        slot, slot_token, fill = slot.copy(), slot_token.copy(), fill_topk.copy()
        nominee = rank_expert[:, k]
        ok = nominates(slot, k)
        for j in range(E):
            cand = np.flatnonzero((nominee == j) & ok)
            m = min(len(cand), vacancy_of(C, int(fill_topk[j])))
            chosen = np.sort(orc._best_first(cand, a[cand, j], orc.POLICY_SCORE)[:m])
            first = min(int(fill_topk[j]), C - m)
            slot[chosen, k] = first + np.arange(m, dtype=np.int32)
            slot_token[j, first:first + m] = chosen
            fill[j] = max(int(fill[j]), first + m)
        return slot, slot_token, fill
    return fr


def m_only_dropped_tokens_nominate(mp):
    mp.setattr(orc, "fill_in_rectification",
               _fill_in_with(lambda slot, k: (slot[:, :k] < 0).any(axis=1), lambda C, f: C - f))


def m_fill_in_evicts(mp):
    mp.setattr(orc, "fill_in_rectification", _fill_in_with(lambda slot, k: np.ones(len(slot), bool), lambda C, f: C))


def _weights_with(ir_factor, normaliser):
    def cw(a, rank_expert, slot, k, n_drop, ir_expert):
        a64 = np.asarray(a, dtype=np.float32).astype(np.float64)
        T, E = a64.shape
        row_max = a64.max(axis=1)
        terms = np.zeros((T, k + 2), dtype=np.float64)
        tok = np.arange(T)
        for r in range(k + 1):
            kept = slot[:, r] >= 0
            terms[kept, r] = np.exp(a64[tok[kept], rank_expert[kept, r]] - row_max[kept])
        has_ir = ir_expert >= 0
        terms[has_ir, k + 1] = ir_factor(n_drop[has_ir]) * np.exp(a64[tok[has_ir], ir_expert[has_ir]] - row_max[has_ir])
        Z = normaliser(terms, a64, row_max)
        out = np.zeros_like(terms)
        live = terms.sum(axis=1) > 0
        out[live] = terms[live] / Z[live, None]
        return out
    return cw


def m_ir_term_without_drop_count(mp):
    mp.setattr(orc, "combine_weights", _weights_with(lambda n: 1.0, lambda t, a, m: t.sum(axis=1)))


def m_weights_are_gate_probabilities(mp):
    mp.setattr(orc, "combine_weights",
               _weights_with(lambda n: n, lambda t, a, m: np.exp(a - m[:, None]).sum(axis=1)))  # softmax over ALL experts


def m_swiglu_gate_and_up_swapped(mp):
    real = orc.expert_ffn
    mp.setattr(orc, "expert_ffn", lambda x, w1, w3, w2, act: real(x, w3, w1, w2, act) if act == "swiglu" else real(x, w1, w3, w2, act))


def m_gelu_tanh_approximation(mp):
    real = orc.expert_ffn

    def ffn(x, w1, w3, w2, act):
        if act != "gelu":
            return real(x, w1, w3, w2, act)
        h = np.asarray(x, dtype=np.float64) @ np.asarray(w1, dtype=np.float64).T
        h = 0.5 * h * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (h + 0.044715 * h ** 3)))
        return h @ np.asarray(w2, dtype=np.float64).T
    mp.setattr(orc, "expert_ffn", ffn)


def m_down_projection_read_in_the_wrong_layout(mp):
    def ffn(x, w1, w3, w2, act):
        x = np.asarray(x, dtype=np.float64)
        g = x @ np.asarray(w1, dtype=np.float64).T
        if act == "swiglu":
            h = g / (1.0 + np.exp(-g)) * (x @ np.asarray(w3, dtype=np.float64).T)
        else:
            from scipy.special import erf
            h = 0.5 * g * (1.0 + erf(g / math.sqrt(2.0)))
        w2 = np.asarray(w2, dtype=np.float64)
        return h @ w2.reshape(w2.shape[1], w2.shape[0])  # [d,F] read as if it were stored [F,d]
    mp.setattr(orc, "expert_ffn", ffn)


def m_router_bias_subtracted(mp):
    def scores(x, w_router, bias=None):
        a = np.asarray(x, dtype=np.float64) @ np.asarray(w_router, dtype=np.float64).T
        if bias is not None:
            a = a - np.asarray(bias, dtype=np.float64)[None, :]
        return a.astype(np.float32)
    mp.setattr(orc, "router_scores", scores)


def m_softmax_over_tokens(mp):
    def probs(a):
        a64 = np.asarray(a, dtype=np.float64)
        z = np.exp(a64 - a64.max(axis=0, keepdims=True))
        return z / z.sum(axis=0, keepdims=True)
    mp.setattr(orc, "softmax_probs", probs)


def m_output_ignores_fill_in(mp):
    real = orc.moe_output

    def out(x, tables, k, w1, w3, w2, act, tokens=None):
        t = dict(tables)
        t["slot"] = tables["slot"].copy()
        t["slot"][:, k] = -1  # the fill-in column never contributes
        return real(x, t, k, w1, w3, w2, act, tokens)
    mp.setattr(orc, "moe_output", out)


def m_output_ignores_intra_gpu(mp):
    real = orc.moe_output

    def out(x, tables, k, w1, w3, w2, act, tokens=None):
        t = dict(tables)
        t["ir_expert"] = np.full_like(tables["ir_expert"], -1)
        return real(x, t, k, w1, w3, w2, act, tokens)
    mp.setattr(orc, "moe_output", out)


def m_quota_ignores_groups(mp):
    def rounds(a, rank_expert, k, Cq, G, policy=orc.POLICY_SCORE):  # one queue of G Cq slots for everybody
        slot, slot_token, fill = orc.topk_capacity_rounds(a, rank_expert, k, G * Cq, policy)
        per_group = np.zeros((G, a.shape[1]), dtype=np.int32)
        per_group[0] = fill
        return slot, slot_token, per_group
    mp.setattr(orc, "topk_capacity_rounds_quota", rounds)


def m_quota_capacity_from_all_tokens(mp):
    real = orc._route_quota
    mp.setattr(orc, "_route_quota", lambda a, k, G, cf, ir, fr, policy: real(a, k, G, cf * G, ir, fr, policy))


def m_quota_fill_in_over_all_groups(mp):
    def fr(a, rank_expert, k, Cq, G, slot, slot_token, fill_topk):  # nominees compete across groups
        a = np.asarray(a, dtype=np.float32)
        T, E = a.shape
        slot, slot_token, fill = slot.copy(), slot_token.copy(), fill_topk.copy()
        for j in range(E):
            cand = np.flatnonzero(rank_expert[:, k] == j)
            order = orc._best_first(cand, a[cand, j], orc.POLICY_SCORE)
            for i in order:
                for g in range(G):
                    if fill[g, j] < Cq:
                        slot[i, k] = g * Cq + fill[g, j]
                        slot_token[j, slot[i, k]] = i
                        fill[g, j] += 1
                        break
        return slot, slot_token, fill
    mp.setattr(orc, "fill_in_rectification_quota", fr)


# ------------------------------------------------------------------ App. A gradient
def _gradient_with(jacobian=None, normaliser_constant=True, multiplicity=lambda m: m, dc_sign=1.0, mass=None):
    """router_score_gradient re-built with one piece exchangeable."""
    def grad(x, a, tables, k, w1, w3, w2, act, dout, straight_through=True, tokens=None):
        a64 = np.asarray(a, dtype=np.float32).astype(np.float64)
        T, E = a64.shape
        tokens = np.arange(T) if tokens is None else np.asarray(tokens)
        g = np.exp(a64 - a64.max(axis=1, keepdims=True))
        g /= g.sum(axis=1, keepdims=True)
        dc = np.zeros((len(tokens), k + 2))
        da = np.zeros((len(tokens), E))
        for n, i in enumerate(tokens):
            P = [(c, e, multiplicity(m)) for c, e, m in orc.processed_assignments(tables, k, i)]
            if not P:
                continue
            for col, e, m in P:
                y = orc.expert_ffn(x[i:i + 1], w1[e], None if w3 is None else w3[e], w2[e], act)[0]
                dc[n, col] = dc_sign * float(np.asarray(dout, dtype=np.float64)[i] @ y)
            t = np.array([m * g[i, e] for _, e, m in P])
            c = t / t.sum()
            D = float(sum(c[p] * dc[n, col] for p, (col, _, _) in enumerate(P)))
            if straight_through and normaliser_constant:
                dg = np.zeros(E)
                for col, e, m in P:
                    dg[e] += m * dc[n, col] / t.sum()
                jac = jacobian(g[i]) if jacobian else np.diag(g[i]) - np.outer(g[i], g[i])
                da[n] = dg @ jac
            else:
                for p, (col, e, m) in enumerate(P):
                    da[n, e] += c[p] * dc[n, col]
                w = np.zeros(E)
                for p, (_, e, _) in enumerate(P):
                    w[e] += c[p]
                da[n] -= (mass(g[i], w) if mass else w) * D
        return dc, da
    return grad


def m_gradient_normaliser_not_held_constant(mp):
    mp.setattr(orc, "router_score_gradient", _gradient_with(normaliser_constant=False))


def m_gradient_softmax_jacobian_sign(mp):
    mp.setattr(orc, "router_score_gradient", _gradient_with(jacobian=lambda g: np.diag(g) + np.outer(g, g)))


def m_gradient_softmax_jacobian_without_diagonal_scale(mp):
    mp.setattr(orc, "router_score_gradient", _gradient_with(jacobian=lambda g: np.eye(len(g)) - np.outer(g, g)))


def m_gradient_forgets_the_drop_count(mp):
    mp.setattr(orc, "router_score_gradient", _gradient_with(multiplicity=lambda m: 1.0))


def m_gradient_of_the_negated_loss(mp):
    mp.setattr(orc, "router_score_gradient", _gradient_with(dc_sign=-1.0))


def m_plain_gradient_subtracts_the_gate_probability(mp):
    # the straight-through closed form used where the plain derivative is asked for
    real = orc.router_score_gradient
    mp.setattr(orc, "router_score_gradient",
               lambda *a, straight_through=True, **kw: real(*a, straight_through=True, **kw))


def m_gradient_ignores_the_fill_in_column(mp):
    real = orc.processed_assignments
    mp.setattr(orc, "processed_assignments", lambda t, k, i: [p for p in real(t, k, i) if p[0] != k])


MUTATIONS = [
    m_keep_lowest_scores, m_token_tie_break_reversed, m_expert_tie_break_reversed, m_capacity_floor,
    m_slots_in_score_order, m_rounds_forget_earlier_fill, m_ir_tokens_interleaved_over_groups, m_ir_ignores_groups,
    m_ir_only_when_all_choices_dropped, m_only_dropped_tokens_nominate, m_fill_in_evicts,
    m_ir_term_without_drop_count, m_weights_are_gate_probabilities, m_swiglu_gate_and_up_swapped,
    m_gelu_tanh_approximation, m_down_projection_read_in_the_wrong_layout, m_router_bias_subtracted, m_softmax_over_tokens,
    m_output_ignores_fill_in, m_output_ignores_intra_gpu, m_quota_ignores_groups, m_quota_capacity_from_all_tokens,
    m_quota_fill_in_over_all_groups, m_gradient_normaliser_not_held_constant, m_gradient_softmax_jacobian_sign,
    m_gradient_softmax_jacobian_without_diagonal_scale, m_gradient_forgets_the_drop_count,
    m_gradient_of_the_negated_loss, m_plain_gradient_subtracts_the_gate_probability,
    m_gradient_ignores_the_fill_in_column,
]


@pytest.mark.parametrize("mutation", MUTATIONS, ids=[m.__name__[2:] for m in MUTATIONS])
def test_a_pin_catches_the_planted_mistake(mutation, monkeypatch):
    mutation(monkeypatch)
    assert pins_catch_it(), "no pin noticed this mistake in the oracle"
