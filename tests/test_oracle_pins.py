"""Pins for the CPU oracle: each test checks it against something other than itself.

  * a hand-worked capacity-3 example (tests/golden/capacity3_example.json),
  * counting definitions evaluated by brute force in pure Python,
  * the second formulation of Fill-in (a top-(k+1) router at unchanged capacity, Sec. 4.2),
  * special cases that reduce to plain library routines (Sec. 4.1: all experts on one
    GPU -> top-1 routing; capacity >= T -> dense softmax mixture; identical experts ->
    one dense FFN, Sec. 5.1),
  * counting identities (Sec. 3: capacity factor k -> #dropped = #padding).
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import rectify_router as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "capacity3_example.json")


@pytest.fixture(scope="module")
def golden():
    with open(GOLDEN) as f:
        return json.load(f)


def _route(g, policy, ir, fr):
    a = np.array(g["logits"], dtype=np.float32)
    return orc.route(a, g["k"], g["G"], g["capacity_factor"], intra_gpu=ir, fill_in=fr, policy=policy)


# ---------------------------------------------------------------- hand-worked example
def test_golden_capacity_and_ranking(golden):
    t = _route(golden, "score", False, False)
    assert t["C"] == golden["C"] == 3
    assert t["rank_expert"].tolist() == golden["rank_expert"]


def test_golden_vanilla_score(golden):
    t = _route(golden, "score", False, False)
    want = golden["score"]["vanilla"]
    assert t["slot_token"].tolist() == want["slot_token"]
    assert t["slot"][:, 0].tolist() == want["slot_rank0"]
    assert np.flatnonzero(t["slot"][:, 0] < 0).tolist() == want["dropped_tokens"]
    assert t["fill_topk"].tolist() == want["fill_topk"]
    assert (t["slot"][:, 1] == -1).all()
    assert (t["ir_expert"] == -1).all()
    # vanilla top-1: a kept token's single weight is exactly 1, a dropped token's is 0
    kept = t["slot"][:, 0] >= 0
    assert np.array_equal(t["combine_w"][:, 0], kept.astype(np.float64))
    assert (t["combine_w"][:, 1:] == 0).all()


def test_golden_vanilla_arrival(golden):
    t = _route(golden, "arrival", False, False)
    want = golden["arrival"]["vanilla"]
    assert t["slot_token"].tolist() == want["slot_token"]
    assert np.flatnonzero(t["slot"][:, 0] < 0).tolist() == want["dropped_tokens"]
    t = _route(golden, "arrival", True, False)
    assert t["ir_expert"].tolist() == golden["arrival"]["intra_gpu"]["ir_expert"]


def test_golden_intra_gpu(golden):
    t = _route(golden, "score", True, False)
    want = golden["score"]["intra_gpu"]
    assert t["ir_expert"].tolist() == want["ir_expert"]
    assert t["ir_row"].tolist() == want["ir_row"]
    assert t["ir_offset"].tolist() == want["ir_offset"]
    assert t["ir_token"].tolist() == want["ir_token"]
    for tok, w in want["ir_weight"].items():
        assert t["combine_w"][int(tok), golden["k"] + 1] == pytest.approx(w, abs=1e-15)
        assert t["combine_w"][int(tok), :golden["k"] + 1].sum() == 0
    # top-k tables are untouched by the rectification
    assert t["slot_token"].tolist() == golden["score"]["vanilla"]["slot_token"]


def test_golden_fill_in(golden):
    t = _route(golden, "score", False, True)
    want = golden["score"]["fill_in"]
    assert t["slot_token"].tolist() == want["slot_token"]
    assert t["slot"][:, 1].tolist() == want["slot_rank1"]
    assert t["fill_total"].tolist() == want["fill_total"]
    assert t["fill_topk"].tolist() == golden["score"]["vanilla"]["fill_topk"]
    for tok, w in want["weights"].items():
        assert t["combine_w"][int(tok), :2].tolist() == pytest.approx(w, abs=1e-12)
        assert t["combine_w"][int(tok), 2] == 0


def test_golden_both(golden):
    t = _route(golden, "score", True, True)
    want = golden["score"]["both"]
    cw = t["combine_w"]
    assert cw[9].tolist() == pytest.approx([0.0, want["t9_fill_weight"], want["t9_ir_weight"]], abs=1e-12)
    assert cw[3].tolist() == pytest.approx([0.0, 0.0, want["t3_ir_weight"]], abs=1e-12)
    assert cw[6].tolist() == pytest.approx([0.0, 0.0, want["t6_ir_weight"]], abs=1e-12)
    assert t["slot_token"].tolist() == golden["score"]["fill_in"]["slot_token"]
    assert t["ir_expert"].tolist() == golden["score"]["intra_gpu"]["ir_expert"]


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("T,E,cf,want", [
    (256, 8, 1.0, 32), (8192, 16, 1.0, 512), (16384, 8, 1.25, 2560), (1 << 20, 64, 0.75, 12288),
    (32768, 32, 0.5, 512), (12, 4, 1.0, 3), (10, 4, 1.0, 3), (3, 8, 1.0, 1), (7, 2, 0.5, 2), (100, 8, 2.0, 25),
])
def test_capacity_formula(T, E, cf, want):
    assert orc.capacity(T, E, cf) == want


def test_router_scores_exact_on_integers():
    # integer-valued inputs: the dot products are exact, so Eq. 1 can be checked with Python ints
    rng = np.random.default_rng(0)
    x = rng.integers(-8, 9, size=(7, 5))
    w = rng.integers(-8, 9, size=(3, 5))
    b = rng.integers(-8, 9, size=3)
    a = orc.router_scores(x.astype(np.float32), w.astype(np.float32), b.astype(np.float32))
    assert a.dtype == np.float32 and a.shape == (7, 3)
    for i in range(7):
        for j in range(3):
            assert a[i, j] == sum(int(x[i, d]) * int(w[j, d]) for d in range(5)) + int(b[j])
    a0 = orc.router_scores(x.astype(np.float32), w.astype(np.float32), None)
    assert a0[2, 1] == sum(int(x[2, d]) * int(w[1, d]) for d in range(5))


def test_rank_experts_against_python_sort():
    rng = np.random.default_rng(1)
    a = np.round(rng.standard_normal((50, 6)) * 2).astype(np.float32) / 2  # many ties
    a[3, 2], a[3, 4] = -0.0, 0.0
    ranks = orc.rank_experts(a, 4)
    for i in range(50):
        want = sorted(range(6), key=lambda j: (-float(a[i, j]), j))[:4]
        assert ranks[i].tolist() == want
    assert orc.rank_experts(a[:, :2], 3)[:, 2].tolist() == [-1] * 50


def test_softmax_probs_definition():
    a = np.array([[1.0, 2.0, 3.0], [-1.0, 0.0, 50.0]], dtype=np.float32)
    g = orc.softmax_probs(a)
    for i in range(2):
        den = sum(math.exp(float(v)) for v in a[i])
        for j in range(3):
            assert g[i, j] == pytest.approx(math.exp(float(a[i, j])) / den, rel=1e-12)


def test_expert_ffn_elementwise_definitions():
    # W1 = W3 = W2 = identity: SwiGLU reduces to silu(x) * x, GELU FFN to gelu(x), per element
    x = np.array([[-2.0, -0.5, 0.0, 1.0, 3.0]])
    eye = np.eye(5)
    y = orc.expert_ffn(x, eye, eye, eye, "swiglu")
    for c, v in enumerate(x[0]):
        assert y[0, c] == pytest.approx(v / (1 + math.exp(-v)) * v, rel=1e-13, abs=1e-15)
    y = orc.expert_ffn(x, eye, None, eye, "gelu")
    for c, v in enumerate(x[0]):
        assert y[0, c] == pytest.approx(0.5 * v * (1 + math.erf(v / math.sqrt(2))), rel=1e-13, abs=1e-15)
    assert orc.expert_ffn(np.array([[1.0]]), np.eye(1), None, np.eye(1), "gelu")[0, 0] == pytest.approx(0.8413447460685429)


def test_expert_ffn_operand_orientation():
    # non-square integer weights, checked with explicit Python loops: W1,W3 are [F,d], W2 is [d,F]
    rng = np.random.default_rng(2)
    d, F = 3, 4
    x = rng.integers(-2, 3, size=(2, d)).astype(np.float64)
    w1 = rng.integers(-2, 3, size=(F, d)).astype(np.float64)
    w3 = rng.integers(-2, 3, size=(F, d)).astype(np.float64)
    w2 = rng.integers(-2, 3, size=(d, F)).astype(np.float64)
    y = orc.expert_ffn(x, w1, w3, w2, "swiglu")
    for n in range(2):
        h = []
        for f in range(F):
            g = sum(x[n, c] * w1[f, c] for c in range(d))
            u = sum(x[n, c] * w3[f, c] for c in range(d))
            h.append(g / (1 + math.exp(-g)) * u)
        for c in range(d):
            assert y[n, c] == pytest.approx(sum(h[f] * w2[c, f] for f in range(F)), rel=1e-12, abs=1e-12)


# ---------------------------------------------------------------- brute force on tiny inputs
def _beats(a, j, i1, i2):
    """token i1 outranks token i2 at expert j (higher score, ties -> lower token index)"""
    return (a[i1, j] > a[i2, j]) or (a[i1, j] == a[i2, j] and i1 < i2)


def _brute_round(a, choice, fill, C, by_score=True):
    """One routing round by definition: enumerate every subset of each expert's candidates and
    keep the unique subset of the allowed size that no outside candidate outranks."""
    T, E = a.shape
    kept_of = {}
    for j in range(E):
        cand = [i for i in range(T) if choice[i] == j]
        m = min(len(cand), C - fill[j])
        winners = []
        for sub in itertools.combinations(cand, m):
            inside = set(sub)
            if by_score:
                ok = all(not _beats(a, j, o, i) for i in inside for o in cand if o not in inside)
            else:
                ok = all(not (o < i) for i in inside for o in cand if o not in inside)
            if ok:
                winners.append(sub)
        assert len(winners) == 1
        kept_of[j] = sorted(winners[0])
    return kept_of


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("policy", ["score", "arrival"])
def test_brute_force_tiny(seed, policy):
    rng = np.random.default_rng(100 + seed)
    T, E, G = 8, 4, 2
    k = 1 + seed % 2
    cf = [0.5, 1.0, 1.5][seed % 3]
    a = np.round(rng.standard_normal((T, E)) * 1.5).astype(np.float32) / 2  # coarse -> ties
    t = orc.route(a, k, G, cf, intra_gpu=True, fill_in=True, policy=policy)
    C = t["C"]
    # ranking by counting: expert j has rank r for token i iff exactly r experts outrank it
    rank_expert = np.full((T, k + 1), -1)
    for i in range(T):
        for j in range(E):
            r = sum(1 for o in range(E) if a[i, o] > a[i, j] or (a[i, o] == a[i, j] and o < j))
            if r <= k:
                rank_expert[i, r] = j
    assert np.array_equal(rank_expert, t["rank_expert"])
    fill = [0] * E
    slot = np.full((T, k + 1), -1)
    slot_token = np.full((E, C), -1)
    for r in range(k + 1):
        fill_in_round = r == k
        kept_of = _brute_round(a, rank_expert[:, r], fill, C, by_score=(policy == "score") or fill_in_round)
        if fill_in_round:
            assert t["fill_topk"].tolist() == fill
        for j, kept in kept_of.items():
            for p, i in enumerate(kept):
                slot[i, r] = fill[j] + p
                slot_token[j, fill[j] + p] = i
            fill[j] += len(kept)
    assert np.array_equal(slot, t["slot"])
    assert np.array_equal(slot_token, t["slot_token"])
    assert t["fill_total"].tolist() == fill
    # Intra-GPU Rectification by definition
    Eg, Tg = E // G, T // G
    for i in range(T):
        n = sum(1 for r in range(k) if slot[i, r] < 0)
        assert t["n_drop"][i] == n
        if n == 0:
            assert t["ir_expert"][i] == -1 and t["ir_row"][i] == -1
            continue
        local = list(range((i // Tg) * Eg, (i // Tg + 1) * Eg))
        h = [j for j in local if all(a[i, j] > a[i, o] or (a[i, j] == a[i, o] and j <= o) for o in local)]
        assert len(h) == 1 and t["ir_expert"][i] == h[0]
        earlier = [q for q in range(i) if t["ir_expert"][q] == h[0]]
        assert t["ir_row"][i] == len(earlier)
        assert t["ir_token"][t["ir_offset"][h[0]] + len(earlier)] == i
    # Eq. 2 / Eq. 3 with math.exp, no max subtraction
    for i in range(T):
        terms = [math.exp(float(a[i, rank_expert[i, r]])) if slot[i, r] >= 0 else 0.0 for r in range(k + 1)]
        n = int(t["n_drop"][i])
        terms.append(n * math.exp(float(a[i, t["ir_expert"][i]])) if n > 0 else 0.0)
        Z = sum(terms)
        want = [v / Z for v in terms] if Z > 0 else terms
        assert t["combine_w"][i].tolist() == pytest.approx(want, rel=1e-12, abs=1e-15)


# ---------------------------------------------------------------- second formulation of Fill-in
@pytest.mark.parametrize("seed", range(6))
def test_fill_in_equals_top_k_plus_1_router(seed):
    # Sec. 4.2: Fill-in == extending top-k to top-(k+1) with the capacity unchanged
    rng = np.random.default_rng(200 + seed)
    T, E = 96, 8
    k = 1 + seed % 3
    cf = [0.75, 1.0, 2.0][seed % 3]
    a = (rng.standard_normal((T, E)) + rng.standard_normal(E)).astype(np.float32)
    if seed % 2:
        a = np.round(a * 2) / 2
    t = orc.route(a, k, 2, cf, intra_gpu=False, fill_in=True)
    C = orc.capacity(T, E, cf)
    ranks = orc.rank_experts(a, k + 2)
    slot, slot_token, fill = orc.topk_capacity_rounds(a, ranks, k + 1, C)
    assert np.array_equal(slot[:, :k + 1], t["slot"])
    assert np.array_equal(slot_token, t["slot_token"])
    assert np.array_equal(fill, t["fill_total"])


# ---------------------------------------------------------------- special cases and identities
def test_single_group_ir_is_top1_routing():
    # Sec. 4.1: with all experts on one GPU, Intra-GPU Rectification is exactly top-1 routing
    rng = np.random.default_rng(3)
    a = rng.standard_normal((64, 8)).astype(np.float32)
    a[:, 0] += 3.0  # overload expert 0 so that many tokens are dropped
    t = orc.route(a, 1, 1, 1.0, intra_gpu=True, fill_in=False)
    dropped = t["slot"][:, 0] < 0
    assert dropped.sum() > 10
    assert np.array_equal(t["ir_expert"][dropped], np.argmax(a, axis=1)[dropped])
    assert (t["ir_expert"][~dropped] == -1).all()
    assert np.array_equal(t["combine_w"][dropped, 2], np.ones(dropped.sum()))


@pytest.mark.parametrize("k,cf", [(1, 1.0), (2, 2.0), (3, 3.0)])
def test_capacity_factor_k_drops_equal_padding(k, cf):
    # Sec. 3: with capacity factor k (and E*C == k*T), #dropped assignments == #padding slots
    rng = np.random.default_rng(4)
    T, E = 128, 8
    a = (rng.standard_normal((T, E)) + 1.5 * rng.standard_normal(E)).astype(np.float32)
    t = orc.route(a, k, 2, cf, intra_gpu=False, fill_in=False)
    drops = int((t["slot"][:, :k] < 0).sum())
    padding = int((t["slot_token"] < 0).sum())
    assert E * t["C"] == k * T
    assert drops == padding > 0
    assert int((t["slot"][:, :k] >= 0).sum()) + drops == k * T


def test_top1_fill_in_half_unsuccessful():
    # App. C.2: with Fill-in, top-1 at CF 1 is top-2 routing at CF 1 -> at least 50 % of
    # the 2T assignments cannot be placed in T slots
    rng = np.random.default_rng(5)
    T, E = 256, 8
    a = (rng.standard_normal((T, E)) + rng.standard_normal(E)).astype(np.float32)
    t = orc.route(a, 1, 2, 1.0, intra_gpu=False, fill_in=True)
    placed = int((t["slot"] >= 0).sum())
    assert placed <= T and (2 * T - placed) / (2 * T) >= 0.5


def test_rectifications_commute():
    # Sec. 1: the two rectifications are orthogonal
    rng = np.random.default_rng(6)
    a = (rng.standard_normal((120, 12)) + rng.standard_normal(12)).astype(np.float32)
    both = orc.route(a, 2, 3, 1.0, True, True)
    ir = orc.route(a, 2, 3, 1.0, True, False)
    fr = orc.route(a, 2, 3, 1.0, False, True)
    for name in ("ir_expert", "ir_row", "ir_offset", "ir_token", "n_drop", "fill_topk"):
        assert np.array_equal(both[name], ir[name]), name
    for name in ("slot", "slot_token", "fill_total", "rank_expert"):
        assert np.array_equal(both[name], fr[name]), name
    assert np.array_equal(ir["slot"][:, :2], fr["slot"][:, :2])


def _dense_mixture(x, a, n_top, w1, w3, w2):
    """softmax-renormalised mixture of the n_top best experts, no capacity: plain matmuls."""
    T, E = a.shape
    out = np.zeros((T, x.shape[1]))
    for i in range(T):
        top = sorted(range(E), key=lambda j: (-float(a[i, j]), j))[:n_top]
        e = np.array([math.exp(float(a[i, j])) for j in top])
        for wgt, j in zip(e / e.sum(), top):
            g = w1[j].astype(np.float64) @ x[i]
            u = w3[j].astype(np.float64) @ x[i]
            out[i] += wgt * (w2[j].astype(np.float64) @ (g / (1 + np.exp(-g)) * u))
    return out


def test_no_drop_case_is_dense_top_k_plus_1_mixture():
    # capacity >= T: nothing is dropped, Intra-GPU is a no-op and Fill-in places every
    # nominee, so the layer is the dense top-(k+1) mixture
    rng = np.random.default_rng(7)
    T, d, F, E, k = 24, 6, 10, 4, 2
    x = rng.standard_normal((T, d))
    wr = rng.standard_normal((E, d)) * 0.5
    w1, w3 = rng.standard_normal((E, F, d)) * 0.3, rng.standard_normal((E, F, d)) * 0.3
    w2 = rng.standard_normal((E, d, F)) * 0.3
    a, t, out = orc.moe_forward(x, wr, None, w1, w3, w2, k, 2, float(E), "swiglu", True, True)
    assert t["C"] >= T and (t["slot"] >= 0).all() and (t["ir_expert"] == -1).all()
    assert np.allclose(out, _dense_mixture(x, a, k + 1, w1, w3, w2), rtol=1e-11, atol=1e-13)
    # vanilla (no rectification): dense top-k mixture
    a, t, out = orc.moe_forward(x, wr, None, w1, w3, w2, k, 2, float(E), "swiglu", False, False)
    assert np.allclose(out, _dense_mixture(x, a, k, w1, w3, w2), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("act", ["swiglu", "gelu"])
def test_identical_experts_closed_form(act):
    # Sec. 5.1: experts are initialised as copies of one dense FFN.  Then every processed
    # token's output is that FFN's output (weights sum to 1) and, with Intra-GPU
    # Rectification on, every token is processed.
    rng = np.random.default_rng(8)
    T, d, F, E, k = 64, 8, 12, 8, 2
    x = rng.standard_normal((T, d))
    wr = rng.standard_normal((E, d))
    b = rng.standard_normal(E) * 2
    f1, f3, f2 = rng.standard_normal((F, d)) * 0.3, rng.standard_normal((F, d)) * 0.3, rng.standard_normal((d, F)) * 0.3
    w1, w3, w2 = np.tile(f1, (E, 1, 1)), np.tile(f3, (E, 1, 1)), np.tile(f2, (E, 1, 1))
    if act == "gelu":
        w3 = None
    g = x @ f1.T
    if act == "swiglu":
        dense = (g / (1 + np.exp(-g)) * (x @ f3.T)) @ f2.T
    else:
        from scipy.special import erf
        dense = (0.5 * g * (1 + erf(g / math.sqrt(2)))) @ f2.T
    a, t, out = orc.moe_forward(x, wr, b, w1, w3, w2, k, 2, 0.75, act, True, True)
    assert (t["slot"][:, :k] < 0).any()
    assert np.allclose(t["combine_w"].sum(axis=1), 1.0, atol=1e-14)
    assert np.allclose(out, dense, rtol=1e-11, atol=1e-13)
    # vanilla: tokens dropped everywhere output exactly 0, the others the dense FFN
    a, t, out = orc.moe_forward(x, wr, b, w1, w3, w2, k, 2, 0.75, act, False, False)
    unprocessed = (t["slot"] < 0).all(axis=1)
    assert unprocessed.any()
    assert (out[unprocessed] == 0).all()
    assert np.allclose(out[~unprocessed], dense[~unprocessed], rtol=1e-11, atol=1e-13)
    # a sampled subset of tokens gives the same rows
    sample = np.array([5, 17, 40])
    _, _, sub = orc.moe_forward(x, wr, b, w1, w3, w2, k, 2, 0.75, act, False, False, tokens=sample)
    assert np.allclose(sub, out[sample], rtol=1e-13, atol=1e-15)


def test_ir_weight_scales_with_number_of_drops():
    # Eq. 3, routing worked by hand.  T=8, E=4, G=2 (tokens 0-3 with experts 0,1; tokens 4-7
    # with experts 2,3), top-2, C = 1.
    #   t0..t3 (3,2,0,0): expert 0 then expert 1; only t0 fits in each -> t1,t2,t3 dropped twice,
    #                     best local expert: 0.
    #   t4 (2.5,1,0,0.5): loses expert 0 and expert 1 to t0 -> dropped twice, local experts
    #                     2|3 score 0 | 0.5 -> expert 3.
    #   t5..t7 (0,0,1,2): expert 3 then expert 2; only t5 fits -> t6,t7 dropped twice -> expert 3.
    a = np.array([[3.0, 2.0, 0.0, 0.0]] * 4 + [[2.5, 1.0, 0.0, 0.5]] + [[0.0, 0.0, 1.0, 2.0]] * 3, dtype=np.float32)
    t = orc.route(a, 2, 2, 0.5, intra_gpu=True, fill_in=False)
    assert t["C"] == 1
    assert t["n_drop"].tolist() == [0, 2, 2, 2, 2, 0, 2, 2]
    assert t["ir_expert"].tolist() == [-1, 0, 0, 0, 3, -1, 3, 3]
    assert t["ir_row"].tolist() == [-1, 0, 1, 2, 0, -1, 1, 2]
    assert t["ir_offset"].tolist() == [0, 3, 3, 3, 6] and t["ir_token"].tolist() == [1, 2, 3, 4, 6, 7]
    for i in (1, 2, 3, 4, 6, 7):  # factor (k - |R_i|) = 2 normalises to weight exactly 1
        assert t["combine_w"][i].tolist() == [0.0, 0.0, 0.0, 1.0]
    assert t["combine_w"][0].tolist() == pytest.approx([1 / (1 + math.exp(-1)), 1 / (1 + math.exp(1)), 0, 0], abs=1e-15)

    # T=4, E=4, G=2 (tokens 0,1 with experts 0,1; tokens 2,3 with experts 2,3), top-2, C = 1.
    #   round 0: e2<-t0, e3<-t1, e0<-{t2 (3.0), t3 (0.0)} keeps t2.
    #   round 1: t0->e3 full, t1->e2 full, e1<-{t2 (2.0), t3 (0.0)} keeps t2.
    #   t0: kept e2 (3.0), dropped once, local best e0 (1.0): weights e^3 : 1*e^1
    #   t1: kept e3 (2.5), dropped once, local best e1 (0.2): weights e^2.5 : e^0.2
    #   t2: both kept: e^3 : e^2 ; t3: dropped twice -> local best e2, weight 1
    a2 = np.array([[1.0, 0.5, 3.0, 2.0], [0.0, 0.2, 2.0, 2.5], [3.0, 2.0, 0.0, 0.1], [0.0, 0.0, -1.0, -2.0]], dtype=np.float32)
    t2 = orc.route(a2, 2, 2, 1.0, intra_gpu=True, fill_in=False)
    assert t2["C"] == 1
    assert t2["slot_token"].tolist() == [[2], [2], [0], [1]]
    assert t2["n_drop"].tolist() == [1, 1, 0, 2]
    assert t2["ir_expert"].tolist() == [0, 1, -1, 2]
    f32 = lambda v: float(np.float32(v))
    w = lambda kept, ir, n: [math.exp(kept) / (math.exp(kept) + n * math.exp(ir)), 0.0, 0.0,
                             n * math.exp(ir) / (math.exp(kept) + n * math.exp(ir))]
    assert t2["combine_w"][0].tolist() == pytest.approx(w(3.0, 1.0, 1), abs=1e-15)
    assert t2["combine_w"][1].tolist() == pytest.approx(w(2.5, f32(0.2), 1), abs=1e-15)
    assert t2["combine_w"][2].tolist() == pytest.approx([1 / (1 + math.exp(-1)), 1 / (1 + math.exp(1)), 0, 0], abs=1e-15)
    assert t2["combine_w"][3].tolist() == [0.0, 0.0, 0.0, 1.0]
    # A case where the factor k - |R_i| is 2 (needs k = 3: one choice kept, two dropped).
    # T = 4, E = 4, G = 1, C = ceil(0.25 * 4 / 4) = 1.  Round 0: all four tokens choose e1, which keeps
    # the best (t2 at 7.0, the lower index of the tie with t3); round 1: all four choose e2, which keeps
    # t2 (6.0); round 2: t0 -> e0 (1.0) and t1 -> e0 (0.0): e0 keeps t0.
    a3 = np.array([[1.0, 5.0, 4.0, -9.0], [0.0, 6.0, 5.0, -9.0]] + [[-9.0, 7.0, 6.0, -9.0]] * 2, dtype=np.float32)
    t3 = orc.route(a3, 3, 1, 0.25, intra_gpu=True, fill_in=False)
    assert t3["C"] == 1 and t3["slot_token"].tolist() == [[0], [2], [2], [-1]]
    assert t3["n_drop"].tolist() == [2, 3, 1, 3]
    # t0: R = {e0 (1.0)}, two drops, best expert overall e1 (5.0): weights e^1 : 2 e^5
    z = math.exp(1.0) + 2 * math.exp(5.0)
    assert t3["combine_w"][0].tolist() == pytest.approx([0, 0, math.exp(1.0) / z, 0, 2 * math.exp(5.0) / z], abs=1e-15)


# ---------------------------------------------------------------- invariants on random inputs
@pytest.mark.parametrize("seed", range(8))
def test_invariants(seed):
    rng = np.random.default_rng(300 + seed)
    E = [4, 8, 16, 6][seed % 4]
    G = [1, 2, 4, 3][seed % 4]
    T = G * [40, 33, 25, 50][seed % 4]
    k = 1 + seed % 3
    cf = [0.5, 1.0, 1.25, 2.0][(seed // 2) % 4]
    a = (rng.standard_normal((T, E)) + 1.2 * rng.standard_normal(E)).astype(np.float32)
    if seed % 2:
        a = np.round(a * 2) / 2
    policy = "arrival" if seed % 3 == 0 else "score"
    t = orc.route(a, k, G, cf, True, True, policy)
    C = t["C"]
    slot, st = t["slot"], t["slot_token"]
    assert (t["fill_total"] <= C).all() and (t["fill_topk"] <= t["fill_total"]).all()
    # kept assignments <-> occupied slots is a bijection
    n_kept = 0
    for i in range(T):
        for r in range(k + 1):
            if slot[i, r] >= 0:
                n_kept += 1
                assert st[t["rank_expert"][i, r], slot[i, r]] == i
    assert n_kept == int((st >= 0).sum()) == int(t["fill_total"].sum())
    for j in range(E):
        assert (st[j, :t["fill_total"][j]] >= 0).all() and (st[j, t["fill_total"][j]:] == -1).all()
    # fill-in only uses otherwise-empty slots, at most one per token, never a top-k expert
    for i in range(T):
        if slot[i, k] >= 0:
            j = t["rank_expert"][i, k]
            assert slot[i, k] >= t["fill_topk"][j]
            assert j not in t["rank_expert"][i, :k]
    # within a round no dropped candidate outranks a kept one; an expert that drops is full
    fill = np.zeros(E, dtype=int)
    for r in range(k + 1):
        for j in range(E):
            cand = np.flatnonzero(t["rank_expert"][:, r] == j)
            kept = [i for i in cand if slot[i, r] >= 0]
            drop = [i for i in cand if slot[i, r] < 0]
            fill[j] += len(kept)
            if drop:
                assert fill[j] == C
                for i in kept:
                    for o in drop:
                        if policy == "score" or r == k:
                            assert _beats(a, j, i, o)
                        else:
                            assert i < o
    # Intra-GPU: exactly the tokens with a top-k drop, inside their own group
    Eg, Tg = E // G, T // G
    for i in range(T):
        n = int((slot[i, :k] < 0).sum())
        assert (t["ir_expert"][i] >= 0) == (n > 0)
        if n:
            assert t["ir_expert"][i] // Eg == i // Tg
    assert t["ir_offset"][-1] == len(t["ir_token"]) == int((t["ir_expert"] >= 0).sum())
    sums = t["combine_w"].sum(axis=1)
    assert np.all((np.abs(sums - 1) < 1e-14) | (sums == 0))
    # with Intra-GPU on every token is processed
    assert np.all(np.abs(sums - 1) < 1e-14)
    # determinism
    t2 = orc.route(a, k, G, cf, True, True, policy)
    for name in t:
        assert np.array_equal(np.asarray(t[name]), np.asarray(t2[name]))


# ---------------------------------------------------------------- capacity read per GPU (quota variant)
def test_quota_hand_worked_example():
    """Four tokens, two experts, two groups of two tokens, top-1 with Fill-in, capacity factor 1:
    Cq = ceil(1 * 2 / 2) = 1 slot per (group, expert); slot g of an expert's queue belongs to group g.

    Round 0: tokens 0 and 1 (group 0) both choose expert 0; its group-0 slot takes the better one, token 1
    (2.0 > 1.0), token 0 is dropped.  Token 2 takes expert 0's group-1 slot, token 3 expert 1's group-1 slot.
    Fill-in: tokens 0, 1, 2 nominate expert 1, token 3 expert 0.  Expert 1's group-0 slot is vacant and goes to
    the better group-0 nominee, token 1 (0.5 > 0.0); its group-1 slot and both slots of expert 0 are taken.
    Intra-GPU: token 0 was dropped; group 0 hosts expert 0 only."""
    a = np.array([[1.0, 0.0],
                  [2.0, 0.5],
                  [3.0, 0.0],
                  [0.0, 1.0]], dtype=np.float32)
    q = orc.route(a, 1, 2, 1.0, intra_gpu=True, fill_in=True, quota=True)
    assert q["C"] == 2 and q["Cq"] == 1
    assert q["slot_token"].tolist() == [[1, 2], [1, 3]]
    assert q["slot"].tolist() == [[-1, -1], [0, 0], [1, -1], [1, -1]]
    assert q["fill_topk_group"].tolist() == [[1, 0], [1, 1]] and q["fill_total_group"].tolist() == [[1, 1], [1, 1]]
    assert q["fill_topk"].tolist() == [2, 1] and q["fill_total"].tolist() == [2, 2]
    assert q["ir_expert"].tolist() == [0, -1, -1, -1] and q["n_drop"].tolist() == [1, 0, 0, 0]
    # the global reading (C = 2 slots per expert for all four tokens): expert 0 keeps the two best of its three
    # candidates, tokens 1 and 2; expert 1 keeps token 3 and fills its second slot with the best nominee, token 1
    g = orc.route(a, 1, 2, 1.0, intra_gpu=True, fill_in=True, quota=False)
    assert g["slot_token"].tolist() == [[1, 2], [3, 1]]


def test_quota_with_one_group_is_the_global_reading():
    rng = np.random.default_rng(7)
    a = np.round(rng.standard_normal((48, 6)) * 2).astype(np.float32) / 2
    for k in (1, 2):
        for policy in ("score", "arrival"):
            g = orc.route(a, k, 1, 0.75, True, True, policy, quota=False)
            q = orc.route(a, k, 1, 0.75, True, True, policy, quota=True)
            for name in g:
                assert np.array_equal(np.asarray(g[name]), np.asarray(q[name])), name


@pytest.mark.parametrize("seed", range(6))
def test_quota_is_independent_routing_per_group(seed):
    """Second formulation: with quotas the slotting of group g is the global slotting of the batch made of
    group g's tokens alone, at capacity capacity(T/G, E, cf), written into the group's block of every queue."""
    rng = np.random.default_rng(500 + seed)
    E, G, Tg = [4, 8, 6][seed % 3], [2, 4, 3][seed % 3], [24, 16, 20][seed % 3]
    k = 1 + seed % 2
    cf = [0.5, 1.0, 1.5][(seed // 2) % 3]
    policy = "arrival" if seed % 3 == 0 else "score"
    T = G * Tg
    a = np.round((rng.standard_normal((T, E)) + rng.standard_normal(E)) * 2).astype(np.float32) / 2
    q = orc.route(a, k, G, cf, intra_gpu=False, fill_in=True, policy=policy, quota=True)
    Cq = orc.capacity(Tg, E, cf)
    assert q["Cq"] == Cq and q["C"] == G * Cq
    slot = np.full((T, k + 1), -1, dtype=np.int64)
    slot_token = np.full((E, G * Cq), -1, dtype=np.int64)
    for g in range(G):
        one = orc.route(a[g * Tg:(g + 1) * Tg], k, 1, cf, intra_gpu=False, fill_in=True, policy=policy, quota=False)
        assert one["C"] == Cq
        local = one["slot"].astype(np.int64)
        slot[g * Tg:(g + 1) * Tg] = np.where(local >= 0, local + g * Cq, -1)
        st = one["slot_token"].astype(np.int64)
        slot_token[:, g * Cq:(g + 1) * Cq] = np.where(st >= 0, st + g * Tg, -1)
        assert q["fill_topk_group"][g].tolist() == one["fill_topk"].tolist()
        assert q["fill_total_group"][g].tolist() == one["fill_total"].tolist()
    assert np.array_equal(slot, q["slot"]) and np.array_equal(slot_token, q["slot_token"])
    assert q["fill_total"].tolist() == q["fill_total_group"].sum(axis=0).tolist()


@pytest.mark.parametrize("seed", range(6))
def test_quota_brute_force_and_invariants(seed):
    rng = np.random.default_rng(700 + seed)
    T, E, G = 12, 4, 2
    Tg, Eg = T // G, E // G
    k = 1 + seed % 2
    cf = [0.5, 1.0, 1.5][seed % 3]
    policy = "arrival" if seed % 2 else "score"
    a = np.round(rng.standard_normal((T, E)) * 1.5).astype(np.float32) / 2
    t = orc.route(a, k, G, cf, intra_gpu=True, fill_in=True, policy=policy, quota=True)
    Cq = t["Cq"]
    rank_expert, slot, st = t["rank_expert"], t["slot"], t["slot_token"]
    # every (group, expert) pair by definition: the unique best subset of the group's own candidates
    fill = [[0] * E for _ in range(G)]
    for r in range(k + 1):
        by_score = policy == "score" or r == k
        for g in range(G):
            choice = np.where(np.arange(T) // Tg == g, rank_expert[:, r], -1)  # other groups do not compete
            kept_of = _brute_round(a, choice, fill[g], Cq, by_score=by_score)
            for j, kept in kept_of.items():
                for p, i in enumerate(kept):
                    assert slot[i, r] == g * Cq + fill[g][j] + p
                    assert st[j, slot[i, r]] == i
                for i in np.flatnonzero(choice == j):
                    if i not in kept:
                        assert slot[i, r] == -1
                fill[g][j] += len(kept)
        if r == k - 1:
            assert t["fill_topk_group"].tolist() == fill
    assert t["fill_total_group"].tolist() == fill
    # a slot of group g's block holds a token of group g or nothing; occupied slots are a prefix of the block
    for j in range(E):
        for g in range(G):
            block = st[j, g * Cq:(g + 1) * Cq]
            n = fill[g][j]
            assert (block[:n] >= 0).all() and (block[n:] == -1).all()
            assert all(i // Tg == g for i in block[:n])
    # Intra-GPU Rectification is unchanged: tokens with a top-k drop, best expert of their own group
    for i in range(T):
        n = int((slot[i, :k] < 0).sum())
        if n == 0:
            assert t["ir_expert"][i] == -1
        else:
            local = list(range((i // Tg) * Eg, (i // Tg + 1) * Eg))
            best = max(local, key=lambda j: (a[i, j], -j))
            assert t["ir_expert"][i] == best
    sums = t["combine_w"].sum(axis=1)
    assert np.all(np.abs(sums - 1) < 1e-14)


# ---------------------------------------------------------------- relabelling (metamorphic) pins
def _kept_pairs(t, k):
    """set of (token, expert, column) that hold a slot, and (token, expert) Intra-GPU assignments"""
    T = t["slot"].shape[0]
    kept = {(i, int(t["rank_expert"][i, r]), r) for i in range(T) for r in range(k + 1) if t["slot"][i, r] >= 0}
    ir = {(i, int(t["ir_expert"][i])) for i in range(T) if t["ir_expert"][i] >= 0}
    return kept, ir


@pytest.mark.parametrize("seed", range(4))
def test_relabelling_experts_relabels_the_tables(seed):
    """With distinct scores nothing depends on expert numbers except through the group an expert is in:
    a relabelling that keeps every expert in its group maps kept sets, weights and outputs onto each other."""
    rng = np.random.default_rng(900 + seed)
    T, E, G, k, d, F = 48, 8, 2, 2, 6, 10
    a = rng.standard_normal((T, E)).astype(np.float32)
    Eg = E // G
    perm = np.concatenate([g * Eg + rng.permutation(Eg) for g in range(G)])  # new label of expert j is perm[j]
    a2 = np.empty_like(a)
    a2[:, perm] = a
    t1 = orc.route(a, k, G, 0.75, True, True)
    t2 = orc.route(a2, k, G, 0.75, True, True)
    k1, ir1 = _kept_pairs(t1, k)
    k2, ir2 = _kept_pairs(t2, k)
    assert {(i, int(perm[e]), r) for (i, e, r) in k1} == k2
    assert {(i, int(perm[e])) for (i, e) in ir1} == ir2
    assert np.allclose(t1["combine_w"], t2["combine_w"], atol=1e-15)
    assert np.array_equal(t1["fill_total"], t2["fill_total"][perm])
    x = rng.standard_normal((T, d)).astype(np.float32)
    w1 = rng.standard_normal((E, F, d)).astype(np.float32)
    w3 = rng.standard_normal((E, F, d)).astype(np.float32)
    w2 = rng.standard_normal((E, d, F)).astype(np.float32)
    inv = np.argsort(perm)  # weights of new expert j are those of old expert inv[j]
    o1 = orc.moe_output(x, t1, k, w1, w3, w2, "swiglu")
    o2 = orc.moe_output(x, t2, k, w1[inv], w3[inv], w2[inv], "swiglu")
    assert np.allclose(o1, o2, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed", range(4))
def test_relabelling_tokens_relabels_the_tables(seed):
    """With distinct scores token numbers only matter through the group a token is in (and the order of
    slots inside a round): a relabelling inside the groups maps kept sets and outputs onto each other."""
    rng = np.random.default_rng(950 + seed)
    T, E, G, k, d, F = 40, 6, 2, 1, 5, 7
    a = rng.standard_normal((T, E)).astype(np.float32)
    Tg = T // G
    perm = np.concatenate([g * Tg + rng.permutation(Tg) for g in range(G)])  # new index of token i is perm[i]
    a2 = np.empty_like(a)
    a2[perm] = a
    for quota in (False, True):
        t1 = orc.route(a, k, G, 0.6, True, True, quota=quota)
        t2 = orc.route(a2, k, G, 0.6, True, True, quota=quota)
        k1, ir1 = _kept_pairs(t1, k)
        k2, ir2 = _kept_pairs(t2, k)
        assert {(int(perm[i]), e, r) for (i, e, r) in k1} == k2
        assert {(int(perm[i]), e) for (i, e) in ir1} == ir2
        assert np.allclose(t1["combine_w"], t2["combine_w"][perm], atol=1e-15)
        x = rng.standard_normal((T, d)).astype(np.float32)
        w1 = rng.standard_normal((E, F, d)).astype(np.float32)
        w2 = rng.standard_normal((E, d, F)).astype(np.float32)
        x2 = np.empty_like(x)
        x2[perm] = x
        o1 = orc.moe_output(x, t1, k, w1, None, w2, "gelu")
        o2 = orc.moe_output(x2, t2, k, w1, None, w2, "gelu")
        assert np.allclose(o1, o2[perm], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed", range(4))
def test_more_capacity_never_drops_more(seed):
    """The kept set of the top-k rounds grows with the capacity factor (Sec. 5.3 reads its tables this way):
    every assignment kept at a smaller capacity is kept at a larger one."""
    rng = np.random.default_rng(980 + seed)
    T, E, k = 64, 8, 2
    a = rng.standard_normal((T, E)).astype(np.float32) + rng.standard_normal(E).astype(np.float32)
    prev = None
    for cf in (0.25, 0.5, 0.75, 1.0, 1.5, 2.0, 4.0, float(E)):
        t = orc.route(a, k, 2, cf, False, False)
        kept = {(i, r) for i in range(T) for r in range(k) if t["slot"][i, r] >= 0}
        if prev is not None:
            assert prev <= kept
        prev = kept
    assert len(prev) == T * k  # capacity factor E: every queue holds all T tokens


# ---------------------------------------------------------------- App. A: gradient of the router scores
def _grad_case(seed, T=32, E=8, k=2, G=2, cf=1.0, d=12, F=20, ir=True, fr=True, act="swiglu", grid=None):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    wr = rng.standard_normal((E, d)) * 0.4
    w1 = rng.standard_normal((E, F, d)) * 0.3
    w3 = rng.standard_normal((E, F, d)) * 0.3 if act == "swiglu" else None
    w2 = rng.standard_normal((E, d, F)) * 0.3
    a = orc.router_scores(x, wr)
    if grid is not None:  # scores on a grid that float32 steps of `grid` stay on
        a = (np.round(a.astype(np.float64) / grid) * grid).astype(np.float32)
    t = orc.route(a, k, G, cf, intra_gpu=ir, fill_in=fr)
    dout = rng.standard_normal((T, d))
    return dict(x=x, a=a, t=t, k=k, w=(w1, w3, w2), act=act, dout=dout, T=T, E=E)


def _assignments(t, k, i):
    """(combine_w column, expert, multiplicity) of token i, read off the tables by hand."""
    P = [(r, int(t["rank_expert"][i, r]), 1.0) for r in range(k + 1) if t["slot"][i, r] >= 0]
    if t["ir_expert"][i] >= 0:
        P.append((k + 1, int(t["ir_expert"][i]), float(k - sum(t["slot"][i, r] >= 0 for r in range(k)))))
    return P


def _expert_out(c, i, e):
    w1, w3, w2 = c["w"]
    return orc.expert_ffn(c["x"][i:i + 1], w1[e], None if w3 is None else w3[e], w2[e], c["act"])[0]


GRAD_CASES = [dict(seed=1), dict(seed=2, k=1, cf=1.25), dict(seed=3, k=2, cf=0.5, ir=True, fr=False),
              dict(seed=4, k=2, cf=2.5, ir=False, fr=True), dict(seed=4, k=1, cf=1.25, ir=False, fr=True), dict(seed=5, k=3, E=8, G=4, cf=1.5, act="gelu"),
              dict(seed=6, k=2, cf=0.75, ir=False, fr=False)]


@pytest.mark.parametrize("case", GRAD_CASES)
@pytest.mark.parametrize("st", [True, False])
def test_gradient_matches_central_differences_of_the_weights(case, st):
    """dL/da against (L(a + h e_l) - L(a - h e_l)) / 2h, L = sum_p dL/dc_p c_p(a), with the
    normaliser frozen at its unperturbed value for the straight-through form (App. A, Eq. 6)."""
    c = _grad_case(**case)
    k, t = c["k"], c["t"]
    dc, da = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=st)
    h = 1e-6
    for i in range(c["T"]):
        P = _assignments(t, k, i)
        a0 = c["a"][i].astype(np.float64)

        def softmax(v):
            z = np.exp(v - v.max())
            return z / z.sum()
        S0 = sum(m * softmax(a0)[e] for _, e, m in P)

        def loss(v):
            if st:
                return sum(dc[i, col] * m * softmax(v)[e] / S0 for col, e, m in P)
            Z = sum(m * math.exp(v[e]) for _, e, m in P)
            return sum(dc[i, col] * m * math.exp(v[e]) / Z for col, e, m in P)
        for l in range(c["E"]):
            up, dn = a0.copy(), a0.copy()
            up[l] += h
            dn[l] -= h
            fd = (loss(up) - loss(dn)) / (2 * h)
            assert abs(fd - da[i, l]) <= 1e-7 * (1.0 + abs(fd)), (i, l, fd, da[i, l])


@pytest.mark.parametrize("case", GRAD_CASES)
def test_plain_gradient_matches_differences_of_the_forward_output(case):
    """Without the straight-through trick the gradient is that of the layer as the forward
    computes it: L(a) = <dL/do, o(a)> with o from moe_output and the weights from
    combine_weights at perturbed scores (decisions frozen)."""
    grid = 2.0 ** -9
    c = _grad_case(**case, grid=grid)
    k, t = c["k"], c["t"]
    _, da = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=False)

    def loss(a):
        tt = dict(t)
        tt["combine_w"] = orc.combine_weights(a, t["rank_expert"], t["slot"], k, t["n_drop"], t["ir_expert"])
        return (orc.moe_output(c["x"], tt, k, *c["w"], c["act"]) * c["dout"]).sum(axis=1)  # per token

    h = 8 * grid
    for l in range(c["E"]):
        up, dn = c["a"].copy(), c["a"].copy()
        up[:, l] += np.float32(h)
        dn[:, l] -= np.float32(h)
        fd = (loss(up) - loss(dn)) / (2 * h)
        assert np.allclose(fd, da[:, l], rtol=2e-3, atol=2e-4 * np.abs(da).max()), l


@pytest.mark.parametrize("case", GRAD_CASES)
@pytest.mark.parametrize("st", [True, False])
def test_gradient_matches_automatic_differentiation(case, st):
    torch = pytest.importorskip("torch")
    c = _grad_case(**case)
    k, t = c["k"], c["t"]
    dc, da = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=st)
    a = torch.tensor(c["a"].astype(np.float64), requires_grad=True)
    g = torch.softmax(a, dim=1)
    loss = torch.zeros((), dtype=torch.float64)
    for i in range(c["T"]):
        P = _assignments(t, k, i)
        if not P:
            continue
        terms = torch.stack([m * g[i, e] for _, e, m in P])
        S = terms.sum()
        weights = terms / (S.detach() if st else S)
        loss = loss + (weights * torch.tensor([dc[i, col] for col, _, _ in P], dtype=torch.float64)).sum()
    loss.backward()
    assert np.allclose(a.grad.numpy(), da, rtol=1e-9, atol=1e-12)


def test_weight_gradient_is_the_projection_of_the_expert_output():
    """Eq. 2 / Eq. 3 are linear in the weights: sum_p c_p dL/dc_p = <dL/do_i, o_i>, and each
    dL/dc_p is <dL/do_i, E_j(x_i)> in the combine_w column of that assignment."""
    for case in GRAD_CASES:
        c = _grad_case(**case)
        k, t = c["k"], c["t"]
        dc, _ = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"])
        o = orc.moe_output(c["x"], t, k, *c["w"], c["act"])
        assert np.allclose((t["combine_w"] * dc).sum(axis=1), (o * c["dout"]).sum(axis=1), rtol=1e-10, atol=1e-12)
        for i in range(c["T"]):
            used = {col: e for col, e, _ in _assignments(t, k, i)}
            for col in range(k + 2):
                want = float(c["dout"][i] @ _expert_out(c, i, used[col])) if col in used else 0.0
                assert abs(dc[i, col] - want) <= 1e-12 * (1 + abs(want))


def test_dense_mixture_gradient_is_the_softmax_gradient():
    """k = E and room for everybody: the weights are the softmax itself, S_i = 1, and both forms
    give dL/da_l = g_l (v_l - sum_j g_j v_j) with v_j = <dL/do_i, E_j(x_i)>."""
    c = _grad_case(seed=11, E=4, k=4, G=2, cf=4.0, ir=True, fr=False)
    k, t = c["k"], c["t"]
    assert (t["slot"][:, :k] >= 0).all()
    g = np.exp(c["a"].astype(np.float64))
    g /= g.sum(axis=1, keepdims=True)
    v = np.array([[c["dout"][i] @ _expert_out(c, i, e) for e in range(c["E"])] for i in range(c["T"])])
    want = g * (v - (g * v).sum(axis=1, keepdims=True))
    for st in (True, False):
        _, da = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=st)
        assert np.allclose(da, want, rtol=1e-10, atol=1e-13)


def test_single_available_expert_has_a_gradient_only_with_the_straight_through_form():
    """App. A, second issue: top-2, first routing kept, second dropped -> normalising over the one
    available expert gives the constant 1 and a zero gradient; with the normaliser held constant
    the gradient is v ([l = e] - g_l), v = <dL/do_i, E_e(x_i)>."""
    c = _grad_case(seed=12, T=48, k=2, cf=0.5, ir=False, fr=False)
    k, t = c["k"], c["t"]
    single = np.flatnonzero((t["slot"][:, 0] >= 0) & (t["slot"][:, 1] < 0))
    assert len(single) >= 5
    dc, da_st = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=True)
    _, da_plain = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=False)
    g = np.exp(c["a"].astype(np.float64))
    g /= g.sum(axis=1, keepdims=True)
    for i in single:
        e = t["rank_expert"][i, 0]
        assert np.abs(da_plain[i]).max() <= 1e-15 * abs(dc[i, 0])
        want = dc[i, 0] * ((np.arange(c["E"]) == e) - g[i])
        assert np.allclose(da_st[i], want, rtol=1e-12, atol=1e-15)
        assert np.abs(da_st[i]).max() > 0


@pytest.mark.parametrize("case", GRAD_CASES)
def test_inactive_experts_feel_the_gradient_only_with_the_straight_through_form(case):
    """App. A, first issue: normalised over the processed set, a score outside it gets no
    gradient; through the softmax over all experts it gets -g_l <dL/do_i, o_i>.  Both forms are
    invariant to a shift of a token's scores (rows sum to zero), and a token that no expert
    processes has no gradient."""
    c = _grad_case(**case)
    k, t = c["k"], c["t"]
    dc, da_st = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=True)
    _, da_plain = orc.router_score_gradient(c["x"], c["a"], t, k, *c["w"], c["act"], c["dout"], straight_through=False)
    o = orc.moe_output(c["x"], t, k, *c["w"], c["act"])
    g = np.exp(c["a"].astype(np.float64))
    g /= g.sum(axis=1, keepdims=True)
    for i in range(c["T"]):
        inside = {e for _, e, _ in _assignments(t, k, i)}
        outside = [l for l in range(c["E"]) if l not in inside]
        if not inside:
            assert not da_st[i].any() and not da_plain[i].any()
            continue
        assert not da_plain[i, outside].any()
        assert np.allclose(da_st[i, outside], -g[i, outside] * (c["dout"][i] @ o[i]), rtol=1e-10, atol=1e-14)
        assert abs(da_st[i].sum()) <= 1e-12 * np.abs(dc[i]).max()
        assert abs(da_plain[i].sum()) <= 1e-12 * np.abs(dc[i]).max()
