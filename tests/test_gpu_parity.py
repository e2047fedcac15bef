"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: logits rel-L2 <= 1e-5 (fp32 accumulation of a fp32 dot product against the float64 oracle
rounded to fp32); integer tables bit-exact and combine weights |err| <= 1e-6 GIVEN IDENTICAL
LOGITS - where the library computes the logits itself, the oracle's routing is run on the
library's own logits, and the number of decisions that the float64-logit routing would take
differently (near-ties flipped by rounding) is printed, not asserted; layer output rel-L2 <= 1e-5
(fp32 workload) / <= 2e-2 (bf16 workloads), plus a per-row and a per-element bound (below), so that
a wrong store mask on a ragged tile cannot hide in the norm.
"""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2402_12399_amd as rr
from oracle import rectify_router as orc
from paper_2402_12399_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

MODES = [(), ("ir",), ("fr",), ("ir", "fr")]

# Output bounds.  bf16 layers round three times on the way to an output element - h, y and the
# output itself, each by at most 2^-9 of the value - and the rounding of h enters an element as a
# random-sign sum over d_ff terms, i.e. about 2^-9 of the row's rms.  Per element:
# |got - want| <= ELEM_ATOL * rms(want row) + ELEM_RTOL * |want| (16 such roundings + 2^-7 of the
# element); per row: |got - want|_2 <= ROW_RTOL * |want|_2.  fp32 layers accumulate in fp32:
# about sqrt(d_ff) * 2^-24 of the row's rms per element.  A masked-out or misplaced store is an
# error of the order of the row's rms itself.
OUT_BOUNDS = {"bf16": dict(l2=2e-2, row=2.0 ** -6, elem_atol=2.0 ** -5, elem_rtol=2.0 ** -7),
              "f32": dict(l2=1e-5, row=3e-5, elem_atol=5e-5, elem_rtol=1e-5)}


def _assert_output_close(got, want, dtype, what=""):
    """got, want: float64 [n, d] outputs of the same tokens."""
    b = OUT_BOUNDS[dtype]
    err = gu.rel_l2(got, want)
    assert err <= b["l2"], f"{what} rel-L2 {err}"
    wn = np.linalg.norm(want, axis=1)
    row_err = np.linalg.norm(got - want, axis=1)
    bad = row_err > b["row"] * np.maximum(wn, 1e-30)
    assert not bad.any(), f"{what} {int(bad.sum())} rows off, worst {float((row_err / np.maximum(wn, 1e-30)).max())}"
    rms = wn / np.sqrt(want.shape[1])
    tol = b["elem_atol"] * rms[:, None] + b["elem_rtol"] * np.abs(want)
    off = np.abs(got - want) > tol
    assert not off.any(), (f"{what} {int(off.sum())} elements off, first at {np.argwhere(off)[0].tolist()}: "
                           f"got {got[tuple(np.argwhere(off)[0])]} want {want[tuple(np.argwhere(off)[0])]}")
    return err


def _flipped_decisions(tables, ref):
    """How many entries of the integer tables the routing from the oracle's own float64 logits takes
    differently from the routing on the library's logits (reported, not asserted)."""
    return {n: int((np.asarray(tables[n]) != np.asarray(ref[n])).sum()) if np.shape(tables[n]) == np.shape(ref[n])
            else -1 for n in ("rank_expert", "slot", "ir_expert")}


def _oracle_tables(a, cfg, mode, arrival=False, quota=False):
    return orc.route(a, cfg.k, cfg.G, cfg.capacity_factor, "ir" in mode, "fr" in mode,
                     orc.POLICY_ARRIVAL if arrival else orc.POLICY_SCORE, quota)


# ------------------------------------------------------------------ routing tables, identical logits
DISPATCH_CASES = [
    # T, E, G, k, cf, ties
    (256, 8, 2, 1, 1.0, False),
    (1000, 8, 4, 2, 1.25, False),     # ragged last token block
    (1000, 6, 2, 2, 0.5, True),       # E not a power of two, many ties, +-0
    (4099, 16, 1, 1, 1.0, True),      # prime T, one group
    (3 * 128, 64, 8, 2, 0.75, False),
    (5000, 64, 8, 4, 2.0, True),      # largest k, k+1 rounds
    (130, 4, 2, 3, 3.0, False),       # k+1 == E
    (64, 2, 2, 2, 1.0, True),         # k == E: no Fill-in possible
    (20000, 32, 8, 1, 0.5, False),
]


@pytest.mark.parametrize("T,E,G,k,cf,ties", DISPATCH_CASES)
@pytest.mark.parametrize("mode", MODES, ids=["vanilla", "ir", "fr", "ir+fr"])
def test_dispatch_tables_bit_exact(T, E, G, k, cf, ties, mode):
    if "fr" in mode and k + 1 > E:
        pytest.skip("Fill-in needs k+1 <= E")
    a = wl.synthetic_logits(T, E, seed=T + E + k, bias_std=1.0, ties=ties)
    for arrival in (False, True):
        cfg = rr.RRConfig(T, 64, 0, E, k, G, cf, rr.RR_F32, rr.RR_ACT_SWIGLU, gu.flags_of(mode, arrival))
        got = gu.run_dispatch(cfg, a)
        gu.assert_tables_equal(got, _oracle_tables(a, cfg, mode, arrival))


def test_dispatch_extreme_cases():
    # every token wants the same expert; capacity 1; capacity >= T; all scores equal
    T, E = 700, 8
    a = np.zeros((T, E), dtype=np.float32)
    a[:, 3] = 5.0
    for cf, k in [(1.0, 1), (0.001, 2), (float(E), 2)]:
        cfg = rr.RRConfig(T, 64, 0, E, k, 2, cf, rr.RR_F32, rr.RR_ACT_SWIGLU, rr.RR_INTRA_GPU | rr.RR_FILL_IN)
        gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, ("ir", "fr")))
    a[:] = 1.0
    cfg = rr.RRConfig(T, 64, 0, E, 2, 4, 1.0, rr.RR_F32, rr.RR_ACT_SWIGLU, rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, ("ir", "fr")))
    # a single token
    a1 = wl.synthetic_logits(1, 4, seed=9)
    cfg = rr.RRConfig(1, 64, 0, 4, 2, 1, 1.0, rr.RR_F32, rr.RR_ACT_SWIGLU, rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    gu.assert_tables_equal(gu.run_dispatch(cfg, a1), _oracle_tables(a1, cfg, ("ir", "fr")))


def test_dispatch_deterministic():
    a = wl.synthetic_logits(30000, 64, seed=77, ties=True)
    cfg = rr.RRConfig(30000, 64, 0, 64, 2, 8, 0.75, rr.RR_F32, rr.RR_ACT_SWIGLU, rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    first = gu.run_dispatch(cfg, a)
    for _ in range(3):
        again = gu.run_dispatch(cfg, a)
        for name in gu.INT_TABLES + ("combine_w",):
            assert np.array_equal(first[name], again[name]), name


LONG_LIST_CASES = [
    # T, E, G, k, cf, bias of expert 1, ties, arrival, quota
    (300000, 8, 2, 2, 0.5, 4.0, False, False, False),   # one expert draws ~all first choices: a list of ~290 K candidates, split
    (300032, 8, 2, 1, 1.0, 4.0, True, False, False),    # the same with scores tied en masse: the sample cannot separate them
    (200000, 4, 2, 2, 3.0, 3.0, False, False, False),   # long lists kept whole (capacity above the candidates)
    (262144, 8, 2, 2, 0.75, 4.0, False, True, False),   # long lists, arrival order
    (4 * 65536, 4, 4, 1, 0.4, 5.0, False, False, True), # per-group capacity: every group's piece of the array is long
    (500000, 64, 8, 2, 0.75, 2.0, False, False, False), # 64 experts, moderate skew: long and short lists side by side
]


@pytest.mark.parametrize("T,E,G,k,cf,hot,ties,arrival,quota", LONG_LIST_CASES)
def test_dispatch_long_lists_bit_exact(T, E, G, k, cf, hot, ties, arrival, quota):
    """Selection lists far longer than one workgroup's registers (a skewed router): tables bit-exact."""
    a = wl.synthetic_logits(T, E, seed=T % 1000 + E, bias_std=0.5, ties=ties)
    a[:, 1] += np.float32(hot)
    a[:, min(3, E - 1)] += np.float32(hot / 2)
    cfg = rr.RRConfig(T, 64, 0, E, k, G, cf, rr.RR_F32, rr.RR_ACT_SWIGLU, gu.flags_of(("ir", "fr"), arrival, quota))
    gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, ("ir", "fr"), arrival, quota))


# ------------------------------------------------------------------ router scores
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,d,E,k", [(256, 64, 8, 1), (1000, 264, 6, 2), (513, 1024, 64, 2), (2048, 2048, 16, 1)])
def test_router_scores(dtype, T, d, E, k):
    rng = np.random.default_rng(T + d)
    x = wl._store(rng.standard_normal((T, d), dtype=np.float32), dtype)
    wr = rng.standard_normal((E, d), dtype=np.float32) * np.float32(0.05)
    b = rng.standard_normal(E).astype(np.float32)
    cfg = rr.RRConfig(T, d, 0, E, k, 1, 1.0, rr.RR_F32 if dtype == "f32" else rr.RR_BF16)
    logits = torch.empty((T, E), dtype=torch.float32, device="cuda")
    probs = torch.empty((T, E), dtype=torch.float32, device="cuda")
    ranks = torch.empty((T, k + 1), dtype=torch.int32, device="cuda")
    for bias in (b, None):
        rr.rr_router_scores(cfg, gu.to_device(x, dtype), torch.from_numpy(wr).cuda(),
                            None if bias is None else torch.from_numpy(bias).cuda(), logits, probs, ranks)
        torch.cuda.synchronize()
        want = orc.router_scores(wl.values_f32(x, dtype), wr, bias)
        got = logits.cpu().numpy()
        assert gu.rel_l2(got.astype(np.float64), want.astype(np.float64)) <= 1e-5
        assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())
        # d p = p (d a - sum p d a): at most twice the logit error, plus fp32 rounding of exp and the sum
        assert np.abs(probs.cpu().numpy() - orc.softmax_probs(want)).max() <= 2e-5 * max(1.0, np.abs(want).max()) + 1e-6
        # ranking: equal to the oracle's wherever the oracle's scores are not within rounding of a tie
        want_rank = orc.rank_experts(want, k + 1)
        got_rank = ranks.cpu().numpy()
        srt = -np.sort(-want.astype(np.float64), axis=1)
        clear = (srt[:, :k + 1] - srt[:, 1:k + 2]).min(axis=1) > 1e-4 if E > k + 1 else np.ones(T, bool)
        assert np.array_equal(got_rank[clear], want_rank[clear])
        assert clear.mean() > 0.99


# ------------------------------------------------------------------ whole layer
def _forward_case(w, mode, inputs, sample=None, arrival=False, quota=False):
    cfg = gu.config_of(w, mode, arrival, T=inputs["x"].shape[0], quota=quota)
    dev = {n: (torch.from_numpy(inputs[n]).cuda() if n in ("w_router", "bias") and inputs[n] is not None
               else gu.to_device(inputs[n], w.dtype)) for n in ("x", "w_router", "bias", "w1", "w3", "w2")}
    out, tables, logits = gu.run_forward(cfg, dev)
    f32 = lambda n: None if inputs[n] is None else wl.values_f32(inputs[n], w.dtype)
    policy = orc.POLICY_ARRIVAL if arrival else orc.POLICY_SCORE
    a = orc.router_scores(f32("x"), inputs["w_router"], inputs["bias"])
    assert gu.rel_l2(logits.astype(np.float64), a.astype(np.float64)) <= 1e-5
    # identical logits: the oracle routes the library's own logits
    want_tables = orc.route(logits, w.k, w.G, w.capacity_factor, "ir" in mode, "fr" in mode, policy, quota)
    gu.assert_tables_equal(tables, want_tables, cw_atol=1e-6)
    print("[parity] %s %s: decisions flipped by logit rounding: %s" % (
        w.name, "+".join(mode) or "vanilla",
        _flipped_decisions(want_tables, orc.route(a, w.k, w.G, w.capacity_factor, "ir" in mode, "fr" in mode, policy, quota))))
    want_out = orc.moe_output(f32("x"), want_tables, w.k, f32("w1"), f32("w3"), f32("w2"), w.act, tokens=sample)
    got = gu.to_host_f64(out)
    if sample is not None:
        got = got[sample]
    err = _assert_output_close(got, want_out, w.dtype, w.name)
    unprocessed = np.flatnonzero(want_tables["combine_w"].sum(axis=1) == 0)
    assert (gu.to_host_f64(out)[unprocessed] == 0).all()
    return err


@pytest.mark.parametrize("mode", MODES, ids=["vanilla", "ir", "fr", "ir+fr"])
def test_forward_c1_fp32(mode):
    _forward_case(wl.C1, mode, wl.make_inputs(wl.C1))


def test_forward_c1_arrival_policy():
    _forward_case(wl.C1, ("ir", "fr"), wl.make_inputs(wl.C1), arrival=True)


SMALL_BF16 = [
    wl.Workload("s1", 1024, 256, 512, 8, 2, 2, 1.25, "bf16", "swiglu", "normal:0.5", 11),
    wl.Workload("s2", 1000, 136, 264, 6, 2, 1, 0.5, "bf16", "swiglu", "zipf:1.5", 12),   # ragged everything
    wl.Workload("s3", 768, 128, 256, 4, 4, 1, 1.0, "bf16", "gelu", "normal:1.0", 13),
    wl.Workload("s4", 600, 72, 200, 4, 2, 2, 1.0, "f32", "swiglu", "normal:1.0", 14),
    # the LDS-DMA GEMM at its shortest K (three chunks, both projections) with gathered rows
    wl.Workload("s5", 1536, 192, 192, 4, 2, 2, 1.0, "bf16", "swiglu", "normal:0.5", 15),
    # GELU variant of the LDS-DMA GEMM with the fused gather; d_ff not a multiple of the column tile
    wl.Workload("s6", 1024, 256, 384, 4, 2, 1, 1.0, "bf16", "gelu", "normal:1.0", 16),
    # more tiles than compute units at three chunks per tile (every workgroup streams from one tile
    # into the next); the down projection's only column tile is narrower than the tile
    wl.Workload("s7", 2048, 192, 5632, 4, 2, 1, 1.0, "bf16", "swiglu", "zipf:1.1", 17),
]


@pytest.mark.parametrize("w", SMALL_BF16, ids=[w.name for w in SMALL_BF16])
@pytest.mark.parametrize("mode", [(), ("ir", "fr")], ids=["vanilla", "ir+fr"])
def test_forward_small(w, mode):
    _forward_case(w, mode, wl.make_inputs(w))


def _full_size_case(w, mode, n_sample=1024, quota=False, report_flips=True):
    """Full-size workload in the configuration the benchmark times; oracle outputs on a token sample."""
    dev = wl.make_inputs_device(w)
    cfg = gu.config_of(w, mode, quota=quota)
    out, tables, logits = gu.run_forward(cfg, dev)
    x = wl.values_f32(gu.to_host_storage(dev["x"]), w.dtype)
    wr, b = dev["w_router"].cpu().numpy(), None if dev["bias"] is None else dev["bias"].cpu().numpy()
    a = orc.router_scores(x, wr, b)
    assert gu.rel_l2(logits.astype(np.float64), a.astype(np.float64)) <= 1e-5
    # identical logits: the oracle routes the library's own logits
    want = orc.route(logits, w.k, w.G, w.capacity_factor, "ir" in mode, "fr" in mode, quota=quota)
    gu.assert_tables_equal(tables, want, cw_atol=1e-6)
    if report_flips:
        print("[parity] %s %s: decisions flipped by logit rounding: %s" % (
            w.name, "+".join(mode) or "vanilla",
            _flipped_decisions(want, orc.route(a, w.k, w.G, w.capacity_factor, "ir" in mode, "fr" in mode, quota=quota))))
    sample = np.sort(np.random.default_rng(w.seed).choice(w.T, n_sample, replace=False))

    class PerExpert:  # expert weights are pulled to the host one expert at a time
        def __init__(self, t):
            self.t, self.shape = t, t.shape

        def __getitem__(self, j):
            return wl.values_f32(gu.to_host_storage(self.t[j]), w.dtype)

    want_out = orc.moe_output(x, want, w.k, PerExpert(dev["w1"]), PerExpert(dev["w3"]), PerExpert(dev["w2"]),
                              w.act, tokens=sample)
    got = gu.to_host_f64(out[torch.from_numpy(sample).cuda()])
    _assert_output_close(got, want_out, w.dtype, w.name)
    unprocessed = torch.from_numpy(np.flatnonzero(want["combine_w"].sum(axis=1) == 0)).cuda()
    assert (out[unprocessed] == 0).all()
    return tables


def test_forward_is_deterministic():
    """The layer has no atomics on data and a fixed reduction order: repeated calls on the same
    inputs must give the same bits (an LDS or load-ordering race in the grouped GEMM would not)."""
    w = wl.C2
    dev = wl.make_inputs_device(w)
    cfg = gu.config_of(w, ("ir", "fr"))
    first, _, _ = gu.run_forward(cfg, dev, want_tables=False)
    first = first.clone()
    for _ in range(4):
        again, _, _ = gu.run_forward(cfg, dev, want_tables=False)
        assert torch.equal(first.view(torch.int16), again.view(torch.int16))


def test_forward_with_internal_tables_and_logits():
    """tables and logits are optional outputs of rr_moe_forward: without them the call keeps both in
    its workspace and must produce the same bits."""
    w = SMALL_BF16[4]
    inputs = wl.make_inputs(w)
    cfg = gu.config_of(w, ("ir", "fr"))
    dev = {n: (torch.from_numpy(inputs[n]).cuda() if n in ("w_router", "bias") and inputs[n] is not None
               else gu.to_device(inputs[n], w.dtype)) for n in ("x", "w_router", "bias", "w1", "w3", "w2")}
    want, _, _ = gu.run_forward(cfg, dev)
    out = torch.zeros_like(want)
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], dev["w1"], dev["w3"], dev["w2"], out, None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))


def test_forward_under_graph_capture():
    """rr_moe_forward only enqueues kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a caller may capture it in a HIP graph: every replay must give the eager bits,
    also with eager calls and synchronisations in between."""
    w = SMALL_BF16[0]
    inputs = wl.make_inputs(w)
    cfg = gu.config_of(w, ("ir", "fr"))
    dev = {n: (torch.from_numpy(inputs[n]).cuda() if n in ("w_router", "bias") and inputs[n] is not None
               else gu.to_device(inputs[n], w.dtype)) for n in ("x", "w_router", "bias", "w1", "w3", "w2")}
    out = torch.empty((cfg.T, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    logits = torch.empty((cfg.T, cfg.E), dtype=torch.float32, device="cuda")
    tb, ws = rr.alloc_tables(cfg), rr.alloc_workspace(cfg)

    def step():
        rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], dev["w1"], dev["w3"], dev["w2"], out, tb, logits, ws)

    rr.rr_init()  # per-device host-side set-up happens outside the capture
    step()
    torch.cuda.synchronize()
    want = out.clone()
    want_slot = tb.slot.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        out.zero_()
        tb.slot.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16))
        assert torch.equal(tb.slot, want_slot)
        step()
        torch.cuda.synchronize()


@pytest.mark.parametrize("mode", MODES, ids=["vanilla", "ir", "fr", "ir+fr"])
def test_forward_c2_full_size(mode):
    _full_size_case(wl.C2, mode)


def test_forward_c3_full_size():
    _full_size_case(wl.C3, ("ir", "fr"), n_sample=512)


def test_forward_c5_full_size():
    t = _full_size_case(wl.C5, ("ir", "fr"), n_sample=512)
    # the workload is meant to overflow heavily and leave experts vacant
    assert (t["slot"][:, 0] < 0).mean() > 0.30
    assert (t["fill_topk"] < wl.C5.T * 0.5 / wl.C5.E).sum() >= 4


# Points of the capacity-factor sweep at the paper's layer shape (Tables 3-5): low capacity with
# Intra-GPU only, high capacity with Fill-in only, one expert per GPU.
SWEEP_POINTS = [
    ("top1_cf0.5_ir", dict(k=1, capacity_factor=0.5), ("ir",)),
    ("top2_cf3.0_fr", dict(k=2, capacity_factor=3.0), ("fr",)),
    ("top1_cf1.0_ir_one_expert_per_gpu", dict(k=1, capacity_factor=1.0, G=8), ("ir",)),
]


@pytest.mark.parametrize("name,change,mode", SWEEP_POINTS, ids=[p[0] for p in SWEEP_POINTS])
def test_forward_capacity_sweep_points_c3_shape(name, change, mode):
    _full_size_case(dataclasses.replace(wl.C3, name="c3_" + name, **change), mode, n_sample=256)


def test_c4_routing_full_size():
    """1M tokens, 64 experts, top-2: logits on sampled rows, tables bit-exact from identical logits."""
    w = wl.C4
    dev = wl.make_inputs_device(w, with_experts=False)
    cfg = gu.config_of(w)
    logits = torch.empty((w.T, w.E), dtype=torch.float32, device="cuda")
    rr.rr_router_scores(cfg, dev["x"], dev["w_router"], None, logits)
    torch.cuda.synchronize()
    sample = np.sort(np.random.default_rng(4).choice(w.T, 4096, replace=False))
    want = orc.router_scores(dev["x"][torch.from_numpy(sample).cuda()].cpu().numpy(), dev["w_router"].cpu().numpy())
    got = logits[torch.from_numpy(sample).cuda()].cpu().numpy()
    assert gu.rel_l2(got.astype(np.float64), want.astype(np.float64)) <= 1e-5
    # routing tables: the oracle and the HIP path are given the same fp32 logits (drawn on the host)
    a = wl.synthetic_logits(w.T, w.E, seed=4, bias_std=0.0)
    a *= np.float32(0.64)  # std of w.x at d_model 1024 with N(0, 0.02) router weights
    gu.assert_tables_equal(gu.run_dispatch(cfg, a), orc.route(a, w.k, w.G, w.capacity_factor, True, True))


def test_c4_forward_routing_full_size():
    """The routing-only workload through rr_moe_forward with d_ff = 0, exactly as the benchmark runs it
    (fp32, 1M tokens, d_model 1024, 64 experts: the streaming router's unpredicated path with the
    ranking fused into its epilogue, then every routing kernel).  Logits on sampled rows against Eq. 1
    in float64; then the oracle routes the library's own logits: every integer table bit-exact,
    weights within 1e-6 (Sec. 3, 4.1, 4.2, Eq. 3)."""
    w = wl.C4
    dev = wl.make_inputs_device(w, with_experts=False)
    cfg = rr.RRConfig(w.T, w.d_model, 0, w.E, w.k, w.G, w.capacity_factor, rr.RR_F32, rr.RR_ACT_SWIGLU,
                      rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    tb, logits = rr.alloc_tables(cfg), torch.empty((w.T, w.E), dtype=torch.float32, device="cuda")
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], None, None, None, None, tb, logits, ws)
    torch.cuda.synchronize()
    sample = np.sort(np.random.default_rng(44).choice(w.T, 4096, replace=False))
    sel = torch.from_numpy(sample).cuda()
    want = orc.router_scores(dev["x"][sel].cpu().numpy(), dev["w_router"].cpu().numpy())
    got = logits[sel].cpu().numpy()
    assert gu.rel_l2(got.astype(np.float64), want.astype(np.float64)) <= 1e-5
    assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())
    a = logits.cpu().numpy()
    gu.assert_tables_equal(tb.to_host(), orc.route(a, w.k, w.G, w.capacity_factor, True, True), cw_atol=1e-6)


@pytest.mark.parametrize("dtype,d,E,k,G", [("f32", 256, 64, 2, 8), ("bf16", 512, 32, 1, 8), ("bf16", 256, 32, 2, 4)])
def test_routing_only_forward_exact_path_real_inputs(dtype, d, E, k, G):
    """The streaming router (more than 16 K tokens) on whole-chunk shapes - fp32 with 64 experts, bf16
    with 32 - with N(0,1) tokens and N(0,0.02) router weights: logits against Eq. 1 in float64, tables
    from the library's own logits."""
    T = 66048 + 256 * G  # not a multiple of the router's 256-token workgroup
    T += 8 * G
    rng = np.random.default_rng(d + E)
    x = wl._store(rng.standard_normal((T, d), dtype=np.float32), dtype)
    wr = rng.standard_normal((E, d), dtype=np.float32) * np.float32(0.02)
    b = (rng.standard_normal(E) * 0.5).astype(np.float32)
    cfg = rr.RRConfig(T, d, 0, E, k, G, 0.75, rr.RR_F32 if dtype == "f32" else rr.RR_BF16, rr.RR_ACT_SWIGLU,
                      rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    tb, logits = rr.alloc_tables(cfg), torch.empty((T, E), dtype=torch.float32, device="cuda")
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, gu.to_device(x, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                      None, None, None, None, tb, logits, ws)
    torch.cuda.synchronize()
    want = orc.router_scores(wl.values_f32(x, dtype), wr, b)
    a = logits.cpu().numpy()
    assert gu.rel_l2(a.astype(np.float64), want.astype(np.float64)) <= 1e-5
    assert np.abs(a - want).max() <= 1e-5 * max(1.0, np.abs(want).max())
    gu.assert_tables_equal(tb.to_host(), orc.route(a, k, G, 0.75, True, True), cw_atol=1e-6)


@pytest.mark.parametrize("dtype,d,E,k,G", [("f32", 128, 64, 2, 8), ("f32", 384, 64, 3, 4), ("bf16", 256, 32, 1, 8),
                                           ("bf16", 768, 32, 2, 2)])
def test_routing_only_forward_exact_path_dyadic(dtype, d, E, k, G):
    """The same kernel path with small dyadic inputs: every dot product is exact, so the logits must
    equal the oracle's bit for bit, ties are frequent, and the tables must match exactly."""
    T = 65536 + 24 * G
    rng = np.random.default_rng(7 * d + E + k)
    x = rng.integers(-3, 4, size=(T, d)).astype(np.float32) / np.float32(2.0)
    wr = rng.integers(-4, 5, size=(E, d)).astype(np.float32) / np.float32(8.0)
    b = rng.integers(-8, 9, size=E).astype(np.float32) / np.float32(4.0)
    cfg = rr.RRConfig(T, d, 0, E, k, G, 0.75, rr.RR_F32 if dtype == "f32" else rr.RR_BF16, rr.RR_ACT_SWIGLU,
                      rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    xs = wl._store(x, dtype)
    tb, logits = rr.alloc_tables(cfg), torch.empty((T, E), dtype=torch.float32, device="cuda")
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, gu.to_device(xs, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                      None, None, None, None, tb, logits, ws)
    torch.cuda.synchronize()
    a = orc.router_scores(wl.values_f32(xs, dtype), wr, b)
    assert np.array_equal(logits.cpu().numpy(), a)
    gu.assert_tables_equal(tb.to_host(), orc.route(a, k, G, 0.75, True, True))


@pytest.mark.parametrize("dtype,E,k,G", [("f32", 64, 2, 8), ("bf16", 16, 1, 4), ("f32", 24, 4, 2), ("f32", 33, 2, 1),
                                         ("bf16", 17, 1, 1)])
def test_routing_only_forward_large_batch(dtype, E, k, G):
    """Large batches take the streaming router whose epilogue also ranks (d_ff = 0: routing only); here
    d_model is not a whole number of K chunks and the expert counts do not fill the staged rows.
    Inputs are small dyadic rationals, so every dot product is exact in fp32 and in bf16 parts: the logits
    must equal the oracle's bit for bit, ties are frequent, and the tables must match exactly."""
    T, d = 66112 + 16 * G, 72
    rng = np.random.default_rng(E + k)
    x = rng.integers(-3, 4, size=(T, d)).astype(np.float32) / np.float32(2.0)
    wr = rng.integers(-4, 5, size=(E, d)).astype(np.float32) / np.float32(8.0)
    b = rng.integers(-8, 9, size=E).astype(np.float32) / np.float32(4.0)
    cfg = rr.RRConfig(T, d, 0, E, k, G, 0.75, rr.RR_F32 if dtype == "f32" else rr.RR_BF16, rr.RR_ACT_SWIGLU,
                      rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    xs = wl._store(x, dtype)
    tb, logits = rr.alloc_tables(cfg), torch.empty((T, E), dtype=torch.float32, device="cuda")
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, gu.to_device(xs, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                      None, None, None, None, tb, logits, ws)
    torch.cuda.synchronize()
    a = orc.router_scores(wl.values_f32(xs, dtype), wr, b)
    assert np.array_equal(logits.cpu().numpy(), a)
    gu.assert_tables_equal(tb.to_host(), orc.route(a, k, G, 0.75, True, True))
    # the stand-alone router entry point takes the same kernel (without the ranking epilogue)
    probs = torch.empty_like(logits)
    ranks = torch.empty((T, k + 1), dtype=torch.int32, device="cuda")
    rr.rr_router_scores(cfg, gu.to_device(xs, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                        logits, probs, ranks)
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), a)
    assert np.array_equal(ranks.cpu().numpy(), orc.rank_experts(a, k + 1))
    assert np.abs(probs.cpu().numpy() - orc.softmax_probs(a)).max() <= 1e-6


@pytest.mark.parametrize("dtype,E,k,G,quota", [("bf16", 32, 1, 8, False), ("f32", 16, 2, 4, True), ("bf16", 24, 3, 2, False)])
def test_routing_only_forward_mid_batch(dtype, E, k, G, quota):
    """Just above 16 K tokens: the smallest batches of the streaming router (its grid does not fill the
    chip), a ragged last workgroup, per-group capacity.  Exact dyadic inputs: logits and tables must
    match bit for bit."""
    T, d = (20480 if quota else 20000 + 8 * G), 136
    rng = np.random.default_rng(3 * E + k)
    x = rng.integers(-3, 4, size=(T, d)).astype(np.float32) / np.float32(2.0)
    wr = rng.integers(-4, 5, size=(E, d)).astype(np.float32) / np.float32(8.0)
    b = rng.integers(-8, 9, size=E).astype(np.float32) / np.float32(4.0)
    cfg = rr.RRConfig(T, d, 0, E, k, G, 0.75, rr.RR_F32 if dtype == "f32" else rr.RR_BF16, rr.RR_ACT_SWIGLU,
                      gu.flags_of(("ir", "fr"), False, quota))
    xs = wl._store(x, dtype)
    tb, logits = rr.alloc_tables(cfg), torch.empty((T, E), dtype=torch.float32, device="cuda")
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, gu.to_device(xs, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                      None, None, None, None, tb, logits, ws)
    torch.cuda.synchronize()
    a = orc.router_scores(wl.values_f32(xs, dtype), wr, b)
    assert np.array_equal(logits.cpu().numpy(), a)
    gu.assert_tables_equal(tb.to_host(), orc.route(a, k, G, 0.75, True, True, quota=quota))
    # the stand-alone entry point takes the same kernel without the fused ranking
    probs = torch.empty_like(logits)
    ranks = torch.empty((T, k + 1), dtype=torch.int32, device="cuda")
    rr.rr_router_scores(cfg, gu.to_device(xs, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                        logits, probs, ranks)
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), a)
    assert np.array_equal(ranks.cpu().numpy(), orc.rank_experts(a, k + 1))
    assert np.abs(probs.cpu().numpy() - orc.softmax_probs(a)).max() <= 1e-6


# ------------------------------------------------------------------ capacity per group (Sec. 3 capacity read per GPU)
QUOTA_CASES = [
    # T, E, G, k, cf, ties
    (256, 8, 2, 1, 1.0, False),        # one token block per group
    (1024, 8, 1, 2, 1.25, False),      # one group: the global reading
    (1536, 6, 3, 2, 0.5, True),        # E and G not powers of two, many ties
    (8 * 128, 64, 8, 2, 0.75, False),  # per-group capacity of 2 slots
    (8 * 640, 64, 8, 4, 2.0, True),    # largest k
    (2 * 384, 4, 2, 3, 3.0, False),    # k+1 == E
    (2 * 128, 2, 2, 2, 1.0, True),     # k == E
    (5 * 4096, 30, 5, 1, 0.5, False),
    (2 * 33792, 16, 2, 2, 1.0, True),
]


@pytest.mark.parametrize("T,E,G,k,cf,ties", QUOTA_CASES)
@pytest.mark.parametrize("mode", MODES, ids=["vanilla", "ir", "fr", "ir+fr"])
def test_quota_dispatch_tables_bit_exact(T, E, G, k, cf, ties, mode):
    if "fr" in mode and k + 1 > E:
        pytest.skip("Fill-in needs k+1 <= E")
    a = wl.synthetic_logits(T, E, seed=T + E + k + 1, bias_std=1.0, ties=ties)
    for arrival in (False, True):
        cfg = rr.RRConfig(T, 64, 0, E, k, G, cf, rr.RR_F32, rr.RR_ACT_SWIGLU, gu.flags_of(mode, arrival, quota=True))
        assert rr.rr_slots_per_expert(cfg) == G * orc.capacity(T // G, E, cf)
        got = gu.run_dispatch(cfg, a)
        gu.assert_tables_equal(got, _oracle_tables(a, cfg, mode, arrival, quota=True))


def test_quota_dispatch_extreme_cases():
    # every token wants the same expert; per-group capacity 1; per-group capacity >= T/G; all scores equal
    T, E, G = 1024, 8, 4
    a = np.zeros((T, E), dtype=np.float32)
    a[:, 3] = 5.0
    flags = gu.flags_of(("ir", "fr"), quota=True)
    for cf, k in [(1.0, 1), (0.001, 2), (float(E), 2)]:
        cfg = rr.RRConfig(T, 64, 0, E, k, G, cf, rr.RR_F32, rr.RR_ACT_SWIGLU, flags)
        gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, ("ir", "fr"), quota=True))
    a[:] = 1.0
    cfg = rr.RRConfig(T, 64, 0, E, 2, G, 1.0, rr.RR_F32, rr.RR_ACT_SWIGLU, flags)
    gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, ("ir", "fr"), quota=True))
    # candidate lists of one group longer than the selection keeps in registers
    Tb = 2 * 32768
    a = wl.synthetic_logits(Tb, 4, seed=22, ties=True)
    a[:, 1] += 6.0
    cfg = rr.RRConfig(Tb, 64, 0, 4, 2, 2, 1.0, rr.RR_F32, rr.RR_ACT_SWIGLU, flags)
    gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, ("ir", "fr"), quota=True))
    a = wl.synthetic_logits(T, E, seed=21)
    # one group is starved of an expert that the other floods: the flooded group may not borrow the idle slots
    a[: T // 2, 0] += 8.0
    a[T // 2:, 0] -= 8.0
    cfg = rr.RRConfig(T, 64, 0, E, 1, 2, 1.0, rr.RR_F32, rr.RR_ACT_SWIGLU, flags)
    got = gu.run_dispatch(cfg, a)
    gu.assert_tables_equal(got, _oracle_tables(a, cfg, ("ir", "fr"), quota=True))
    Cq = orc.capacity(T // 2, E, 1.0)
    assert (got["slot_token"][0, :Cq] >= 0).all() and (got["slot_token"][0, :Cq] < T // 2).all()
    assert ((got["slot_token"][0, Cq:] >= T // 2) | (got["slot_token"][0, Cq:] < 0)).all()


def test_quota_c4_routing_full_size():
    w = wl.C4
    cfg = gu.config_of(w, quota=True)
    a = wl.synthetic_logits(w.T, w.E, seed=5, bias_std=0.3)
    gu.assert_tables_equal(gu.run_dispatch(cfg, a), orc.route(a, w.k, w.G, w.capacity_factor, True, True, quota=True))


@pytest.mark.parametrize("mode", MODES, ids=["vanilla", "ir", "fr", "ir+fr"])
def test_quota_forward_c1_fp32(mode):
    _forward_case(wl.C1, mode, wl.make_inputs(wl.C1), quota=True)


QUOTA_SMALL = [w for w in SMALL_BF16 if (w.T // w.G) * w.G == w.T and (w.T // w.G) % 128 == 0]
QUOTA_SMALL += [
    # bf16 shape that takes the register-staged GEMM and the separate gather kernel (d % 64 != 0), E not a power of two
    wl.Workload("q1", 1024, 136, 264, 6, 2, 1, 0.5, "bf16", "swiglu", "zipf:1.5", 31),
    # fp32 path (plain FMA GEMM), top-2, three groups
    wl.Workload("q2", 1152, 72, 200, 6, 3, 2, 1.0, "f32", "swiglu", "normal:1.0", 32),
]


@pytest.mark.parametrize("w", QUOTA_SMALL, ids=[w.name for w in QUOTA_SMALL])
@pytest.mark.parametrize("mode", [(), ("ir", "fr")], ids=["vanilla", "ir+fr"])
def test_quota_forward_small(w, mode):
    _forward_case(w, mode, wl.make_inputs(w), quota=True)


@pytest.mark.parametrize("mode", [(), ("ir", "fr")], ids=["vanilla", "ir+fr"])
def test_quota_forward_c2_full_size(mode):
    _full_size_case(wl.C2, mode, quota=True)


def test_quota_forward_c5_full_size():
    _full_size_case(wl.C5, ("ir", "fr"), n_sample=512, quota=True)


# ------------------------------------------------------------------ seeded random configurations
def test_dispatch_random_configurations():
    """Sixty seeded draws over the whole argument space of the routing tables (sizes on both sides of
    the small-batch path's limit, E, G, k, capacity factor, rectification modes, drop policy, capacity
    scope, tie density): tables bit-exact."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 60:
        G = int(rng.choice([1, 2, 3, 4, 8]))
        E = G * int(rng.integers(1, 64 // G + 1))
        k = int(rng.integers(1, 5))
        if k > E:
            continue
        quota = bool(rng.integers(0, 2))
        if quota:
            T = G * 128 * int(rng.integers(1, 12))
        elif rng.integers(0, 4) == 0:  # above 16 K tokens the selection lists are materialised (scan, scatter)
            T = G * int(rng.integers(16384 // G + 1, 40000 // G))
        else:
            T = G * int(rng.integers(1, 1500))
        mode = MODES[int(rng.integers(0, 4))]
        if "fr" in mode and k + 1 > E:
            continue
        cf = float(rng.choice([0.05, 0.3, 0.5, 0.75, 1.0, 1.25, 2.0, 4.0]))
        arrival = bool(rng.integers(0, 2))
        ties = bool(rng.integers(0, 2))
        a = wl.synthetic_logits(T, E, seed=1000 + done, bias_std=float(rng.choice([0.0, 1.0, 3.0])), ties=ties)
        cfg = rr.RRConfig(T, 64, 0, E, k, G, cf, rr.RR_F32, rr.RR_ACT_SWIGLU, gu.flags_of(mode, arrival, quota))
        try:
            gu.assert_tables_equal(gu.run_dispatch(cfg, a), _oracle_tables(a, cfg, mode, arrival, quota))
        except AssertionError as err:
            raise AssertionError(f"T={T} E={E} G={G} k={k} cf={cf} mode={mode} arrival={arrival} quota={quota} "
                                 f"ties={ties}: {err}") from None
        done += 1


def test_routing_only_forward_random_configurations():
    """The same through rr_moe_forward with d_ff = 0 (the router's fused ranking instead of topk_rank; every
    fourth draw is a batch for the streaming router): inputs are small dyadic rationals, so the logits are
    exact and the tables must match bit for bit."""
    rng = np.random.default_rng(77)
    done = 0
    while done < 32:
        G = int(rng.choice([1, 2, 4, 8]))
        E = G * int(rng.integers(1, 64 // G + 1))
        k = int(rng.integers(1, 4))
        if k + 1 > E:
            continue
        quota = bool(rng.integers(0, 2))
        if done % 4 == 3:  # above 16 K tokens: the streaming router and materialised selection lists
            T = G * 128 * int(rng.integers(130 // G + 1, 400 // G + 2)) if quota else G * int(rng.integers(16385 // G + 1, 70000 // G))
        else:
            T = G * 128 * int(rng.integers(1, 10)) if quota else G * int(rng.integers(10, 1200))
        d = 8 * int(rng.integers(2, 40))
        dtype = "bf16" if rng.integers(0, 2) else "f32"
        x = rng.integers(-3, 4, size=(T, d)).astype(np.float32) / np.float32(2.0)
        wr = rng.integers(-4, 5, size=(E, d)).astype(np.float32) / np.float32(8.0)
        b = rng.integers(-8, 9, size=E).astype(np.float32) / np.float32(4.0)
        cf = float(rng.choice([0.3, 0.75, 1.0, 1.5]))
        cfg = rr.RRConfig(T, d, 0, E, k, G, cf, rr.RR_F32 if dtype == "f32" else rr.RR_BF16, rr.RR_ACT_SWIGLU,
                          gu.flags_of(("ir", "fr"), False, quota))
        xs = wl._store(x, dtype)
        tb, logits = rr.alloc_tables(cfg), torch.empty((T, E), dtype=torch.float32, device="cuda")
        ws = rr.alloc_workspace(cfg)
        rr.rr_moe_forward(cfg, gu.to_device(xs, dtype), torch.from_numpy(wr).cuda(), torch.from_numpy(b).cuda(),
                          None, None, None, None, tb, logits, ws)
        torch.cuda.synchronize()
        a = orc.router_scores(wl.values_f32(xs, dtype), wr, b)
        assert np.array_equal(logits.cpu().numpy(), a), (T, d, E, dtype)
        try:
            gu.assert_tables_equal(tb.to_host(), orc.route(a, k, G, cf, True, True, quota=quota))
        except AssertionError as err:
            raise AssertionError(f"T={T} d={d} E={E} G={G} k={k} cf={cf} {dtype} quota={quota}: {err}") from None
        done += 1


def test_forward_random_grouped_gemm_shapes():
    """Twelve seeded draws of bf16 layer shapes that take the LDS-DMA grouped GEMM (d_model and d_ff
    multiples of 64 from 192 up: ragged row tiles, column tiles narrower than the tile, few or many
    chunks per tile), over expert counts, k, modes, capacity scope and both activations.  Router
    inputs are small dyadic rationals, so logits and tables must match bit for bit."""
    rng = np.random.default_rng(5)
    done = 0
    while done < 12:
        G = int(rng.choice([1, 2, 4]))
        E = G * int(rng.integers(1, 16 // G + 1))
        k = int(rng.integers(1, 4))
        if k + 1 > E:
            continue
        quota = bool(rng.integers(0, 2))
        T = G * 128 * int(rng.integers(1, 17)) if quota else G * int(rng.integers(50, 2500))
        d = 64 * int(rng.integers(3, 17))
        F = 64 * int(rng.integers(3, 33))
        act = "swiglu" if rng.integers(0, 2) else "gelu"
        mode = MODES[int(rng.integers(0, 4))]
        cf = float(rng.choice([0.3, 0.75, 1.0, 1.5, 3.0]))
        x = rng.integers(-3, 4, size=(T, d)).astype(np.float32) / np.float32(2.0)
        wr = rng.integers(-4, 5, size=(E, d)).astype(np.float32) / np.float32(8.0)
        b = rng.integers(-8, 9, size=E).astype(np.float32) / np.float32(4.0)
        w1 = wl._store(rng.standard_normal((E, F, d), dtype=np.float32) * np.float32(0.05), "bf16")
        w3 = wl._store(rng.standard_normal((E, F, d), dtype=np.float32) * np.float32(0.05), "bf16") if act == "swiglu" else None
        w2 = wl._store(rng.standard_normal((E, d, F), dtype=np.float32) * np.float32(0.05), "bf16")
        xs = wl._store(x, "bf16")
        what = f"T={T} d={d} F={F} E={E} G={G} k={k} cf={cf} {act} mode={mode} quota={quota}"
        cfg = rr.RRConfig(T, d, F, E, k, G, cf, rr.RR_BF16, rr.RR_ACT_GELU if act == "gelu" else rr.RR_ACT_SWIGLU,
                          gu.flags_of(mode, False, quota))
        dev = {"x": gu.to_device(xs, "bf16"), "w_router": torch.from_numpy(wr).cuda(), "bias": torch.from_numpy(b).cuda(),
               "w1": gu.to_device(w1, "bf16"), "w3": gu.to_device(w3, "bf16"), "w2": gu.to_device(w2, "bf16")}
        out, tables, logits = gu.run_forward(cfg, dev)
        f32 = lambda s: None if s is None else wl.values_f32(s, "bf16")
        a = orc.router_scores(f32(xs), wr, b)
        assert np.array_equal(logits, a), what
        want = orc.route(a, k, G, cf, "ir" in mode, "fr" in mode, quota=quota)
        try:
            gu.assert_tables_equal(tables, want, cw_atol=1e-6)
            _assert_output_close(gu.to_host_f64(out), orc.moe_output(f32(xs), want, k, f32(w1), f32(w3), f32(w2), act),
                                 "bf16")
        except AssertionError as err:
            raise AssertionError(f"{what}: {err}") from None
        done += 1
