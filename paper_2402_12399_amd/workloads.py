"""Seeded synthetic inputs shaped like the paper's MoE layers.

This module only draws random numbers and rounds them to the storage type.
It holds none of the method's arithmetic, so both the HIP path and the CPU
oracle can be fed from it without sharing anything else.

The paper measures a LLaMA2-7B-derived MoE (d_model 4096, d_ff 11008, SwiGLU,
8 or 32 experts, 1-4 experts per GPU, 8 x 2048 = 16384 tokens per GPU
micro-batch; Sec. 5.1) on OpenOrca activations that are not available here;
these workloads stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    d_model: int
    d_ff: int            # 0: routing-only workload, no expert FFN
    E: int
    G: int
    k: int
    capacity_factor: float
    dtype: str           # "f32" | "bf16" (x, expert weights, out); router is fp32
    act: str             # "gelu" | "swiglu"
    bias: str            # "normal:<std>" | "zipf:<s>" | "none"
    seed: int
    modes: tuple = field(default=(("ir", "fr"),))


# The five configurations of the build's baseline description.
C1 = Workload("c1_tiny_top1_f32", 256, 64, 128, 8, 2, 1, 1.0, "f32", "gelu", "normal:1.0", 1)
C2 = Workload("c2_top1_bf16_zipf1.1", 8192, 2048, 5632, 16, 4, 1, 1.0, "bf16", "swiglu", "zipf:1.1", 2,
              modes=((), ("ir",), ("fr",), ("ir", "fr")))
C3 = Workload("c3_top2_bf16", 16384, 4096, 11008, 8, 2, 2, 1.25, "bf16", "swiglu", "normal:0.5", 3)
C4 = Workload("c4_routing_stress_f32", 1 << 20, 1024, 0, 64, 8, 2, 0.75, "f32", "swiglu", "none", 4)
C5 = Workload("c5_heavy_imbalance_bf16", 32768, 4096, 14336, 32, 8, 1, 0.5, "bf16", "swiglu", "zipf:1.5", 5)
ALL = {w.name.split("_")[0]: w for w in (C1, C2, C3, C4, C5)}


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the storage type: float32 as is, bf16 as uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a if dtype == "f32" else to_bf16_bits(a)


def router_bias(w: Workload, rng: np.random.Generator):
    kind, _, arg = w.bias.partition(":")
    if kind == "none":
        return None
    if kind == "normal":
        return (rng.standard_normal(w.E) * float(arg)).astype(np.float32)
    if kind == "zipf":
        # popularity p_j proportional to rank_j^-s, ranks a seeded permutation of the experts
        ranks = rng.permutation(w.E).astype(np.float64) + 1.0
        p = ranks ** (-float(arg))
        return np.log(p / p.sum()).astype(np.float32)
    raise ValueError(w.bias)


def values_f32(stored: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float32 values of a storage array (float32, or uint16 bf16 bit patterns)."""
    return stored if dtype == "f32" else bf16_bits_to_f32(stored)


def make_inputs(w: Workload, with_experts: bool = True, T: int | None = None):
    """Host arrays for one workload, drawn with numpy (small and medium workloads).

    x and the expert weights are returned in storage form: float32, or uint16 bf16 bit patterns
    (see values_f32).  Router weights and bias are fp32.
    """
    T = w.T if T is None else T
    rng = np.random.default_rng(w.seed)
    out = {}
    out["w_router"] = (rng.standard_normal((w.E, w.d_model), dtype=np.float32) * np.float32(0.02))
    out["bias"] = router_bias(w, rng)
    out["x"] = _store(rng.standard_normal((T, w.d_model), dtype=np.float32), w.dtype)
    out["w1"] = out["w3"] = out["w2"] = None
    if with_experts and w.d_ff > 0:
        shapes = {"w1": (w.E, w.d_ff, w.d_model), "w3": (w.E, w.d_ff, w.d_model), "w2": (w.E, w.d_model, w.d_ff)}
        for name, shp in shapes.items():
            if name == "w3" and w.act != "swiglu":
                continue
            out[name] = _store(rng.standard_normal(shp, dtype=np.float32) * np.float32(0.02), w.dtype)
    return out


def make_inputs_device(w: Workload, device="cuda", with_experts: bool = True):
    """Device tensors for one workload, drawn by torch's seeded generator on the GPU.

    Used for the large workloads, where drawing billions of normals on the host would take
    minutes.  The bits are reproducible for a given torch build and GPU; the CPU oracle is fed by
    copying the very same bits to the host.  Router weights and bias come from the numpy recipe.
    """
    import torch
    rng = np.random.default_rng(w.seed)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    out = {}
    out["w_router"] = torch.from_numpy(rng.standard_normal((w.E, w.d_model), dtype=np.float32) * np.float32(0.02)).to(device)
    b = router_bias(w, rng)
    out["bias"] = None if b is None else torch.from_numpy(b).to(device)
    out["x"] = torch.randn((w.T, w.d_model), generator=gen, device=device, dtype=torch.float32).to(tdt)
    out["w1"] = out["w3"] = out["w2"] = None
    if with_experts and w.d_ff > 0:
        shapes = {"w1": (w.E, w.d_ff, w.d_model), "w3": (w.E, w.d_ff, w.d_model), "w2": (w.E, w.d_model, w.d_ff)}
        for name, shp in shapes.items():
            if name == "w3" and w.act != "swiglu":
                continue
            m = torch.empty(shp, device=device, dtype=tdt)
            for e in range(w.E):  # per expert, to bound the fp32 temporary
                m[e] = (torch.randn(shp[1:], generator=gen, device=device, dtype=torch.float32) * 0.02).to(tdt)
            out[name] = m
    return out


def make_output_gradient(w: Workload, T: int | None = None) -> np.ndarray:
    """dL/d out for the backward pass of a workload: N(0,1) in storage form, from its own seed."""
    rng = np.random.default_rng(w.seed + 7919)
    return _store(rng.standard_normal((w.T if T is None else T, w.d_model), dtype=np.float32), w.dtype)


def make_output_gradient_device(w: Workload, device="cuda"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed + 7919)
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    return torch.randn((w.T, w.d_model), generator=gen, device=device, dtype=torch.float32).to(tdt)


def synthetic_logits(T: int, E: int, seed: int, bias_std: float = 1.0, ties: bool = False) -> np.ndarray:
    """fp32 router logits drawn directly (for routing-table parity with identical logits).

    `ties=True` quantises them coarsely so that equal scores (and +-0.0) occur often.
    """
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((T, E), dtype=np.float32)
    a += (rng.standard_normal(E) * bias_std).astype(np.float32)[None, :]
    if ties:
        a = np.round(a * 2.0) / 2.0
        a[a == 0.0] = np.where(rng.random(int((a == 0.0).sum())) < 0.5, np.float32(-0.0), np.float32(0.0))
    return np.ascontiguousarray(a, dtype=np.float32)
