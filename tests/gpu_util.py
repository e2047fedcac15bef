"""Helpers for the GPU parity tests: host <-> device marshalling and table comparison."""
import numpy as np
import torch

import paper_2402_12399_amd as rr
from paper_2402_12399_amd import workloads as wl

INT_TABLES = ("rank_expert", "slot", "slot_token", "fill_topk", "fill_total",
              "ir_expert", "ir_row", "ir_offset", "ir_token")


def flags_of(mode, arrival=False, quota=False):
    f = 0
    if "ir" in mode:
        f |= rr.RR_INTRA_GPU
    if "fr" in mode:
        f |= rr.RR_FILL_IN
    if arrival:
        f |= rr.RR_POLICY_ARRIVAL
    if quota:
        f |= rr.RR_QUOTA_PER_GROUP
    return f


def config_of(w: wl.Workload, mode=("ir", "fr"), arrival=False, T=None, quota=False) -> rr.RRConfig:
    return rr.RRConfig(T or w.T, w.d_model, w.d_ff, w.E, w.k, w.G, w.capacity_factor,
                       rr.RR_F32 if w.dtype == "f32" else rr.RR_BF16,
                       rr.RR_ACT_GELU if w.act == "gelu" else rr.RR_ACT_SWIGLU, flags_of(mode, arrival, quota))


def to_device(a, dtype):
    """storage array (float32 / uint16 bf16 bits) -> device tensor"""
    if a is None:
        return None
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


def to_host_storage(t):
    """device tensor -> storage array (float32 / uint16 bf16 bits)"""
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def to_host_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def assert_tables_equal(got: dict, want: dict, cw_atol=1e-6):
    for name in INT_TABLES:
        g, w_ = np.asarray(got[name]), np.asarray(want[name])
        assert g.shape == w_.shape, (name, g.shape, w_.shape)
        if not np.array_equal(g, w_):
            bad = np.argwhere(g != w_)
            raise AssertionError(f"table {name}: {len(bad)} mismatches, first at {bad[0].tolist()}: "
                                 f"got {g[tuple(bad[0])]} want {w_[tuple(bad[0])]}")
    err = np.abs(got["combine_w"].astype(np.float64) - want["combine_w"]).max()
    assert err <= cw_atol, f"combine_w max abs err {err}"


def rel_l2(got, want):
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def run_dispatch(cfg: rr.RRConfig, logits_np: np.ndarray) -> dict:
    logits = torch.from_numpy(logits_np).cuda()
    tb = rr.alloc_tables(cfg)
    ws = rr.alloc_workspace(cfg)
    rr.rr_rectified_dispatch(cfg, logits, tb, ws)
    torch.cuda.synchronize()
    return tb.to_host()


def run_forward(cfg: rr.RRConfig, dev: dict, want_tables=True):
    """dev: device tensors x, w_router, bias, w1, w3, w2.  Returns (out tensor, tables dict, logits np)."""
    tdt = torch.float32 if cfg.dtype == rr.RR_F32 else torch.bfloat16
    out = torch.empty((cfg.T, cfg.d_model), dtype=tdt, device="cuda")
    logits = torch.empty((cfg.T, cfg.E), dtype=torch.float32, device="cuda")
    tb = rr.alloc_tables(cfg) if want_tables else None
    ws = rr.alloc_workspace(cfg)
    rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], dev["w1"], dev["w3"], dev["w2"], out, tb, logits, ws)
    torch.cuda.synchronize()
    return out, (tb.to_host() if tb is not None else None), logits.cpu().numpy()
