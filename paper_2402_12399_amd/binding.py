"""ctypes binding of librr.so: argument marshalling only, every step runs in the HIP kernels.

Function names and argument order follow include/rr.h.  Tensors are torch CUDA tensors (torch is
used for device memory and streams only); calls are enqueued on torch's current stream.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

RR_F32, RR_BF16 = 0, 1
RR_ACT_GELU, RR_ACT_SWIGLU = 0, 1
RR_INTRA_GPU, RR_FILL_IN, RR_POLICY_ARRIVAL, RR_QUOTA_PER_GROUP = 1, 2, 4, 8
RR_GRAD_STRAIGHT_THROUGH = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class RRError(RuntimeError):
    pass


class _Config(C.Structure):
    _fields_ = [("T", C.c_int32), ("d_model", C.c_int32), ("d_ff", C.c_int32), ("E", C.c_int32),
                ("k", C.c_int32), ("G", C.c_int32), ("capacity_factor", C.c_float),
                ("dtype", C.c_int32), ("act", C.c_int32), ("flags", C.c_uint32)]


_TABLE_FIELDS = ("rank_expert", "slot", "slot_token", "fill_topk", "fill_total",
                 "ir_expert", "ir_row", "ir_offset", "ir_token", "combine_w")


class _Tables(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _TABLE_FIELDS]


class _KernelTime(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int32), ("total_ms", C.c_float)]


@dataclass
class RRConfig:
    T: int
    d_model: int
    d_ff: int
    E: int
    k: int
    G: int
    capacity_factor: float
    dtype: int = RR_BF16
    act: int = RR_ACT_SWIGLU
    flags: int = RR_INTRA_GPU | RR_FILL_IN

    def c(self) -> _Config:
        return _Config(self.T, self.d_model, self.d_ff, self.E, self.k, self.G, self.capacity_factor,
                       self.dtype, self.act, self.flags)


def library_path() -> str:
    return os.path.join(_HERE, "librr.so")


def load_library():
    """Loads librr.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RRError(f"{path} is missing: build it with `python -m paper_2402_12399_amd.build`")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.rr_capacity.restype = i32
    lib.rr_capacity.argtypes = [i32, i32, C.c_float]
    lib.rr_slots_per_expert.restype = i32
    lib.rr_slots_per_expert.argtypes = [C.POINTER(_Config)]
    lib.rr_workspace_bytes.restype = C.c_int
    lib.rr_workspace_bytes.argtypes = [C.POINTER(_Config), C.POINTER(sz)]
    lib.rr_router_scores.restype = C.c_int
    lib.rr_router_scores.argtypes = [C.POINTER(_Config), vp, vp, vp, vp, vp, vp, vp]
    lib.rr_rectified_dispatch.restype = C.c_int
    lib.rr_rectified_dispatch.argtypes = [C.POINTER(_Config), vp, C.POINTER(_Tables), vp, sz, vp]
    lib.rr_rectified_dispatch_static.restype = C.c_int
    lib.rr_rectified_dispatch_static.argtypes = [C.POINTER(_Config), vp, C.POINTER(_Tables), vp]
    lib.rr_moe_forward.restype = C.c_int
    lib.rr_moe_forward.argtypes = [C.POINTER(_Config), vp, vp, vp, vp, vp, vp, vp, C.POINTER(_Tables), vp, vp, sz, vp]
    lib.rr_router_backward.restype = C.c_int
    lib.rr_router_backward.argtypes = [C.POINTER(_Config), vp, vp, C.POINTER(_Tables), vp, sz, C.c_uint32, vp, vp, vp]
    lib.rr_init.restype = C.c_int
    lib.rr_init.argtypes = []
    lib.rr_profile_enable.restype = C.c_int
    lib.rr_profile_enable.argtypes = [C.c_int]
    lib.rr_profile_read.restype = C.c_int
    lib.rr_profile_read.argtypes = [C.POINTER(_KernelTime), i32, C.POINTER(i32)]
    lib.rr_strerror.restype = C.c_char_p
    lib.rr_strerror.argtypes = [C.c_int]
    _LIB = lib
    return lib


def rr_strerror(code: int) -> str:
    return load_library().rr_strerror(code).decode()


def _check(code: int, what: str):
    if code != 0:
        raise RRError(f"{what} failed: {rr_strerror(code)} ({code})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def rr_init():
    _check(load_library().rr_init(), "rr_init")


def rr_capacity(T: int, E: int, capacity_factor: float) -> int:
    return int(load_library().rr_capacity(T, E, capacity_factor))


def rr_slots_per_expert(cfg: RRConfig) -> int:
    cc = cfg.c()
    n = int(load_library().rr_slots_per_expert(C.byref(cc)))
    if n < 0:
        raise RRError("rr_slots_per_expert: invalid or unsupported configuration")
    return n


def rr_workspace_bytes(cfg: RRConfig) -> int:
    n = C.c_size_t(0)
    cc = cfg.c()
    _check(load_library().rr_workspace_bytes(C.byref(cc), C.byref(n)), "rr_workspace_bytes")
    return int(n.value)


def alloc_workspace(cfg: RRConfig, device="cuda"):
    import torch
    return torch.empty(rr_workspace_bytes(cfg), dtype=torch.uint8, device=device)


class Tables:
    """Device tensors of rr_tables plus the C struct that points at them."""

    def __init__(self, cfg: RRConfig, device="cuda"):
        import torch
        C_ = rr_slots_per_expert(cfg)
        i32 = dict(dtype=torch.int32, device=device)
        self.capacity = C_
        self.rank_expert = torch.empty((cfg.T, cfg.k + 1), **i32)
        self.slot = torch.empty((cfg.T, cfg.k + 1), **i32)
        self.slot_token = torch.empty((cfg.E, C_), **i32)
        self.fill_topk = torch.empty(cfg.E, **i32)
        self.fill_total = torch.empty(cfg.E, **i32)
        self.ir_expert = torch.empty(cfg.T, **i32)
        self.ir_row = torch.empty(cfg.T, **i32)
        self.ir_offset = torch.empty(cfg.E + 1, **i32)
        self.ir_token = torch.empty(cfg.T, **i32)
        self.combine_w = torch.empty((cfg.T, cfg.k + 2), dtype=torch.float32, device=device)

    def c(self) -> _Tables:
        return _Tables(*[getattr(self, n).data_ptr() for n in _TABLE_FIELDS])

    def to_host(self) -> dict:
        out = {n: getattr(self, n).cpu().numpy() for n in _TABLE_FIELDS}
        out["ir_token"] = out["ir_token"][:int(out["ir_offset"][-1])]
        return out


def alloc_tables(cfg: RRConfig, device="cuda") -> Tables:
    return Tables(cfg, device)


def rr_router_scores(cfg: RRConfig, x, w_router, bias, logits, probs=None, rank_expert=None):
    cc = cfg.c()
    _check(load_library().rr_router_scores(C.byref(cc), _ptr(x), _ptr(w_router), _ptr(bias), _ptr(logits),
                                           _ptr(probs), _ptr(rank_expert), _stream()), "rr_router_scores")


def rr_rectified_dispatch(cfg: RRConfig, logits, tables: Tables, workspace):
    cc, tc = cfg.c(), tables.c()
    _check(load_library().rr_rectified_dispatch(C.byref(cc), _ptr(logits), C.byref(tc), _ptr(workspace),
                                                workspace.numel(), _stream()), "rr_rectified_dispatch")


def rr_rectified_dispatch_static(cfg: RRConfig, logits, tables: Tables):
    """rr_rectified_dispatch with the library's own static scratch buffer (allocates nothing)."""
    cc, tc = cfg.c(), tables.c()
    _check(load_library().rr_rectified_dispatch_static(C.byref(cc), _ptr(logits), C.byref(tc), _stream()),
           "rr_rectified_dispatch_static")


def rr_moe_forward(cfg: RRConfig, x, w_router, bias, w1, w3, w2, out, tables: Tables | None, logits, workspace):
    cc = cfg.c()
    tc = tables.c() if tables is not None else None
    _check(load_library().rr_moe_forward(C.byref(cc), _ptr(x), _ptr(w_router), _ptr(bias), _ptr(w1), _ptr(w3),
                                         _ptr(w2), _ptr(out), C.byref(tc) if tc is not None else None,
                                         _ptr(logits), _ptr(workspace), workspace.numel(), _stream()),
           "rr_moe_forward")


def rr_router_backward(cfg: RRConfig, dout, logits, tables: Tables | None, workspace, dlogits, dcombine_w=None,
                       straight_through: bool = True):
    cc = cfg.c()
    tc = tables.c() if tables is not None else None
    _check(load_library().rr_router_backward(C.byref(cc), _ptr(dout), _ptr(logits),
                                             C.byref(tc) if tc is not None else None, _ptr(workspace),
                                             workspace.numel(), RR_GRAD_STRAIGHT_THROUGH if straight_through else 0,
                                             _ptr(dcombine_w), _ptr(dlogits), _stream()), "rr_router_backward")


def rr_profile_enable(on: bool):
    _check(load_library().rr_profile_enable(1 if on else 0), "rr_profile_enable")


def rr_profile_read() -> dict:
    arr = (_KernelTime * 32)()
    n = C.c_int32(0)
    _check(load_library().rr_profile_read(arr, 32, C.byref(n)), "rr_profile_read")
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms)) for i in range(n.value)}
