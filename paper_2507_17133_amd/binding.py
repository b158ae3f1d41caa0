"""Thin ctypes binding of libbrownout_moe.so (see include/brownout_moe.h).

Argument marshalling only: every step of the layer runs in the library's HIP
kernels.  PyTorch is used to own device memory and to name the HIP stream.
There is no CPU or PyTorch fallback: if the library is missing or a call fails,
an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbrownout_moe.so")

MOE_OK = 0
STAGES = ("prep", "gate", "count", "scan", "scatter", "tiles", "gemm1", "gemm2", "combine")
EXPORTS = ("moe_status_string", "moe_last_hip_error", "moe_init", "moe_workspace_size", "moe_gate_packed_size",
           "moe_pack_gate", "moe_build_united", "moe_route", "moe_route_static", "moe_forward",
           "moe_distill_workspace_size", "moe_distill_united", "moe_profile_enable", "moe_profile_collect",
           "moe_latency_p90", "moe_salc_update", "moe_probe_mfma", "moe_probe_hbm_read")
MOE_GATE_FP32, MOE_GATE_PACKED = 0, 1


class MoeError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


class moe_salc_params(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("slo", "warning_factor", "increment", "shrink_ratio")]


class moe_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d_model", "d_ff", "n_experts", "top_k", "way", "n_shared", "d_ff_shared",
                                         "score_fn", "add_residual", "gate_format")]


class moe_ffn_weights(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("w3", C.c_void_p), ("w2", C.c_void_p)]


moe_ffn_weights_out = moe_ffn_weights        # same layout; the C header's type for tensors a call writes


class moe_route_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("topk_idx", "topk_w", "expert_cnt", "expert_unit", "expert_in_s1",
                                          "unit_cnt", "unit_off", "row_token", "row_weight", "token_rows",
                                          "n_rows", "near_tie")]


_lib = None


def lib():
    """Loads the HIP library; fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2507_17133_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        L.moe_status_string.restype = C.c_char_p
        L.moe_status_string.argtypes = [C.c_int32]
        L.moe_last_hip_error.restype = C.c_char_p
        L.moe_init.restype = C.c_int32
        L.moe_init.argtypes = []
        L.moe_workspace_size.restype = C.c_int32
        L.moe_workspace_size.argtypes = [C.POINTER(moe_config), C.c_int32, C.POINTER(C.c_size_t)]
        L.moe_gate_packed_size.restype = C.c_int32
        L.moe_gate_packed_size.argtypes = [C.POINTER(moe_config), C.POINTER(C.c_size_t)]
        L.moe_pack_gate.restype = C.c_int32
        L.moe_pack_gate.argtypes = [C.POINTER(moe_config), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.moe_route_static.restype = C.c_int32
        L.moe_route_static.argtypes = [C.POINTER(moe_config), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_double,
                                       C.c_int32, C.POINTER(moe_route_out), C.c_void_p]
        L.moe_build_united.restype = C.c_int32
        L.moe_build_united.argtypes = [C.POINTER(moe_config), C.POINTER(moe_ffn_weights), C.POINTER(moe_ffn_weights),
                                       C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.moe_distill_workspace_size.restype = C.c_int32
        L.moe_distill_workspace_size.argtypes = [C.POINTER(moe_config), C.c_int32, C.POINTER(C.c_size_t)]
        L.moe_distill_united.restype = C.c_int32
        L.moe_distill_united.argtypes = [C.POINTER(moe_config), C.POINTER(moe_ffn_weights), C.POINTER(moe_ffn_weights),
                                         C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                         C.c_void_p]
        L.moe_route.restype = C.c_int32
        L.moe_route.argtypes = [C.POINTER(moe_config), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_double,
                                C.c_int32, C.POINTER(moe_route_out), C.c_void_p, C.c_size_t, C.c_void_p]
        L.moe_forward.restype = C.c_int32
        L.moe_forward.argtypes = [C.POINTER(moe_config), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                  C.POINTER(moe_ffn_weights), C.POINTER(moe_ffn_weights), C.POINTER(moe_ffn_weights),
                                  C.c_double, C.c_int32, C.POINTER(moe_route_out), C.c_void_p, C.c_void_p, C.c_size_t,
                                  C.c_void_p]
        L.moe_latency_p90.restype = C.c_double
        L.moe_latency_p90.argtypes = [C.POINTER(C.c_double), C.c_size_t]
        L.moe_salc_update.restype = C.c_double
        L.moe_salc_update.argtypes = [C.c_double, C.c_double, C.POINTER(moe_salc_params)]
        L.moe_probe_mfma.restype = C.c_int32
        L.moe_probe_mfma.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double)]
        L.moe_probe_hbm_read.restype = C.c_int32
        L.moe_probe_hbm_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double)]
        L.moe_profile_enable.restype = C.c_int32
        L.moe_profile_enable.argtypes = [C.c_int32]
        L.moe_profile_collect.restype = C.c_int32
        L.moe_profile_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != MOE_OK:
        L = lib()
        detail = L.moe_status_string(status).decode()
        hip = L.moe_last_hip_error().decode()
        raise MoeError(status, where, detail + (": " + hip if hip else ""))


def make_config(d_model, d_ff, n_experts, top_k, way, n_shared=0, d_ff_shared=0, score_fn=0, add_residual=0,
                gate_format=MOE_GATE_FP32):
    return moe_config(d_model, d_ff, n_experts, top_k, way, n_shared, d_ff_shared, score_fn, add_residual, gate_format)


def with_packed_gate(cfg: moe_config) -> moe_config:
    """A copy of cfg that says gate_w is the buffer pack_gate() returned."""
    c = moe_config.from_buffer_copy(cfg)
    c.gate_format = MOE_GATE_PACKED
    return c


def init():
    """Per-device set-up of the library on the current device (needed only before a FIRST call under capture)."""
    _check(lib().moe_init(), "moe_init")


def pack_gate(cfg: moe_config, gate_w: torch.Tensor, stream=None) -> torch.Tensor:
    """One-time repack of the fp32 gate matrix [m][d]; pass the result as gate_w with with_packed_gate(cfg)."""
    assert gate_w.is_cuda and gate_w.dtype == torch.float32 and gate_w.is_contiguous()
    assert tuple(gate_w.shape) == (cfg.n_experts, cfg.d_model)
    n = C.c_size_t(0)
    _check(lib().moe_gate_packed_size(C.byref(cfg), C.byref(n)), "moe_gate_packed_size")
    packed = torch.empty(n.value, dtype=torch.uint8, device=gate_w.device)
    _check(lib().moe_pack_gate(C.byref(cfg), _ptr(gate_w), _ptr(packed), packed.numel(), _stream(stream)),
           "moe_pack_gate")
    return packed


def config_of(cfg) -> moe_config:
    """From a workloads.LayerConfig."""
    return make_config(cfg.d, cfg.F, cfg.m, cfg.K, cfg.way, cfg.n_shared, cfg.F_s, cfg.score_fn, 0)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _weights(w: Optional[Sequence[torch.Tensor]]):
    if w is None:
        return None
    for t in w:
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()
    return moe_ffn_weights(w[0].data_ptr(), w[1].data_ptr(), w[2].data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def workspace_size(cfg: moe_config, T_max: int) -> int:
    n = C.c_size_t(0)
    _check(lib().moe_workspace_size(C.byref(cfg), T_max, C.byref(n)), "moe_workspace_size")
    return int(n.value)


def alloc_workspace(cfg: moe_config, T_max: int, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_size(cfg, T_max), dtype=torch.uint8, device=device)


@dataclass
class RouteOut:
    topk_idx: torch.Tensor
    topk_w: torch.Tensor
    expert_cnt: torch.Tensor
    expert_unit: torch.Tensor
    expert_in_s1: torch.Tensor
    unit_cnt: torch.Tensor
    unit_off: torch.Tensor
    row_token: torch.Tensor
    row_weight: torch.Tensor
    token_rows: torch.Tensor
    n_rows: torch.Tensor
    near_tie: torch.Tensor

    def as_struct(self) -> moe_route_out:
        return moe_route_out(*(getattr(self, n).data_ptr() for n, _ in moe_route_out._fields_))


def alloc_route_out(cfg: moe_config, T: int, device="cuda") -> RouteOut:
    m, K, Ns = cfg.n_experts, cfg.top_k, cfg.n_shared
    G = (m + cfg.way - 1) // cfg.way
    U = m + G + Ns
    i32 = dict(dtype=torch.int32, device=device)
    return RouteOut(
        topk_idx=torch.empty((T, K), **i32), topk_w=torch.empty((T, K), dtype=torch.float32, device=device),
        expert_cnt=torch.empty((m,), **i32), expert_unit=torch.empty((m,), **i32),
        expert_in_s1=torch.empty((m,), dtype=torch.uint8, device=device),
        unit_cnt=torch.empty((U,), **i32), unit_off=torch.empty((U + 1,), **i32),
        row_token=torch.empty((T * (K + Ns),), **i32),
        row_weight=torch.empty((T * (K + Ns),), dtype=torch.float32, device=device),
        token_rows=torch.empty((T, K + Ns), **i32), n_rows=torch.empty((1,), **i32),
        near_tie=torch.empty((T,), dtype=torch.uint8, device=device))


def moe_route(cfg: moe_config, x, gate_w, gate_bias, threshold: float, use_full_brownout: bool = False,
              out: Optional[RouteOut] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> RouteOut:
    T = x.shape[0]
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[1] == cfg.d_model
    _check_gate(cfg, gate_w)
    if out is None:
        out = alloc_route_out(cfg, T, x.device)
    if workspace is None:
        workspace = alloc_workspace(cfg, T, x.device)
    st = out.as_struct()
    _check(lib().moe_route(C.byref(cfg), _ptr(x), T, _ptr(gate_w), _ptr(gate_bias), float(threshold),
                           1 if use_full_brownout else 0, C.byref(st), _ptr(workspace), workspace.numel(),
                           _stream(stream)), "moe_route")
    return out


def _check_gate(cfg: moe_config, gate_w):
    assert gate_w.is_cuda and gate_w.is_contiguous()
    if cfg.gate_format == MOE_GATE_PACKED:
        assert gate_w.dtype == torch.uint8
    else:
        assert gate_w.dtype == torch.float32 and tuple(gate_w.shape) == (cfg.n_experts, cfg.d_model)


def moe_route_static(cfg: moe_config, x, gate_w, gate_bias, threshold: float, use_full_brownout: bool,
                     out: RouteOut, stream=None) -> RouteOut:
    """moe_route on the library's own fixed scratch: no workspace argument; `out` is the caller's (allocate it
    beforehand: this call allocates nothing)."""
    T = x.shape[0]
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[1] == cfg.d_model
    _check_gate(cfg, gate_w)
    st = out.as_struct()
    _check(lib().moe_route_static(C.byref(cfg), _ptr(x), T, _ptr(gate_w), _ptr(gate_bias), float(threshold),
                                  1 if use_full_brownout else 0, C.byref(st), _stream(stream)), "moe_route_static")
    return out


def moe_forward(cfg: moe_config, x, gate_w, gate_bias, experts, united=None, shared=None, threshold: float = 1.0,
                use_full_brownout: bool = False, route: Optional[RouteOut] = None, out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    T = x.shape[0]
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[1] == cfg.d_model
    if out is None:
        out = torch.empty((T, cfg.d_model), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = alloc_workspace(cfg, T, x.device)
    we, wu, ws = _weights(experts), _weights(united), _weights(shared)
    rs = route.as_struct() if route is not None else None
    _check(lib().moe_forward(C.byref(cfg), _ptr(x), T, _ptr(gate_w), _ptr(gate_bias),
                             C.byref(we) if we is not None else None, C.byref(wu) if wu is not None else None,
                             C.byref(ws) if ws is not None else None, float(threshold),
                             1 if use_full_brownout else 0, C.byref(rs) if rs is not None else None, _ptr(out),
                             _ptr(workspace), workspace.numel(), _stream(stream)), "moe_forward")
    return out


def moe_build_united(cfg: moe_config, experts, calib_x: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None
                     ) -> Tuple[Tuple[torch.Tensor, torch.Tensor, torch.Tensor], Optional[torch.Tensor]]:
    m, d, F = cfg.n_experts, cfg.d_model, cfg.d_ff
    G = (m + cfg.way - 1) // cfg.way
    dev = experts[0].device
    united = (torch.empty((G, F, d), dtype=torch.bfloat16, device=dev),
              torch.empty((G, F, d), dtype=torch.bfloat16, device=dev),
              torch.empty((G, d, F), dtype=torch.bfloat16, device=dev))
    loss = None
    n_calib = 0
    if calib_x is not None:
        assert calib_x.is_cuda and calib_x.dtype == torch.bfloat16 and calib_x.is_contiguous()
        n_calib = calib_x.shape[0]
        loss = torch.empty((G,), dtype=torch.float32, device=dev)
        if workspace is None:
            workspace = alloc_workspace(cfg, n_calib, dev)
    we, wu = _weights(experts), _weights(united)
    _check(lib().moe_build_united(C.byref(cfg), C.byref(we), C.byref(wu), _ptr(calib_x), n_calib, _ptr(loss),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)),
           "moe_build_united")
    return united, loss


def moe_distill_united(cfg: moe_config, experts, united, calib_x: torch.Tensor, steps: int, lr: float,
                       workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Trains `united` in place; returns the loss history [G][steps+1] (fp32, device)."""
    assert calib_x.is_cuda and calib_x.dtype == torch.bfloat16 and calib_x.is_contiguous()
    n_calib = calib_x.shape[0]
    G = (cfg.n_experts + cfg.way - 1) // cfg.way
    if workspace is None:
        nbytes = C.c_size_t(0)
        _check(lib().moe_distill_workspace_size(C.byref(cfg), n_calib, C.byref(nbytes)), "moe_distill_workspace_size")
        workspace = torch.empty((nbytes.value + 255) // 256 * 256, dtype=torch.uint8, device=calib_x.device)
    hist = torch.empty((G, steps + 1), dtype=torch.float32, device=calib_x.device)
    we, wu = _weights(experts), _weights(united)
    _check(lib().moe_distill_united(C.byref(cfg), C.byref(we), C.byref(wu), _ptr(calib_x), n_calib, steps, lr,
                                    _ptr(hist), _ptr(workspace), workspace.numel(), _stream(stream)),
           "moe_distill_united")
    return hist


def probe_mfma(operands: torch.Tensor, stream=None) -> float:
    """TFLOP/s of a pure bf16 MFMA loop whose operand bits are the first 64 KiB of `operands` (waits)."""
    assert operands.is_cuda and operands.is_contiguous()
    sink = torch.empty(2 << 20, dtype=torch.uint8, device=operands.device)
    r = C.c_double(0.0)
    _check(lib().moe_probe_mfma(_ptr(operands), operands.numel() * operands.element_size(), _ptr(sink), sink.numel(),
                                _stream(stream), C.byref(r)), "moe_probe_mfma")
    return r.value


def probe_hbm_read(buf: torch.Tensor, stream=None) -> float:
    """GB/s of a read-only sweep over `buf` (waits)."""
    assert buf.is_cuda and buf.is_contiguous()
    sink = torch.zeros(4, dtype=torch.uint8, device=buf.device)
    r = C.c_double(0.0)
    _check(lib().moe_probe_hbm_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), sink.numel(),
                                    _stream(stream), C.byref(r)), "moe_probe_hbm_read")
    return r.value


def profile_enable(stages: Sequence[str] = STAGES):
    mask = 0
    for s in stages:
        mask |= 1 << STAGES.index(s)
    _check(lib().moe_profile_enable(mask), "moe_profile_enable")


def profile_disable():
    _check(lib().moe_profile_enable(0), "moe_profile_enable")


def profile_collect():
    """Returns {stage: (total_ms, launches)} and clears the record (synchronises)."""
    ms = (C.c_double * len(STAGES))()
    n = (C.c_int64 * len(STAGES))()
    _check(lib().moe_profile_collect(ms, n), "moe_profile_collect")
    return {s: (float(ms[i]), int(n[i])) for i, s in enumerate(STAGES)}


def latency_p90(latencies) -> float:
    """P90 (nearest rank) of a sequence of host latencies, through the C ABI."""
    n = len(latencies)
    arr = (C.c_double * max(n, 1))(*[float(v) for v in latencies])
    return float(lib().moe_latency_p90(arr if n else None, n))


def salc_update(threshold: float, latency: float, slo: float, warning_factor: float = 0.8, increment: float = 0.1,
                shrink_ratio: float = 0.8) -> float:
    """One step of the SLO-aware latency controller (Algorithm 2), through the C ABI."""
    p = moe_salc_params(slo, warning_factor, increment, shrink_ratio)
    return float(lib().moe_salc_update(threshold, latency, C.byref(p)))

