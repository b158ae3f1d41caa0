"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2507_17133_amd as P
from paper_2507_17133_amd import binding as B

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "brownout_moe.h")

if not os.path.exists(B.LIB_PATH):
    from paper_2507_17133_amd import build as _build
    _build.build()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_function_is_exported():
    names = _declared()
    assert {"moe_build_united", "moe_route", "moe_forward", "moe_workspace_size"} <= set(names)
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in brownout_moe.h but not exported"
    assert set(B.EXPORTS) == set(names)


def test_status_strings():
    L = P.lib()
    for code in range(0, -7, -1):
        assert L.moe_status_string(code)
    assert L.moe_status_string(0) == b"ok"


def test_workspace_size_grows_with_tokens_and_rejects_bad_shapes():
    good = P.make_config(4096, 14336, 8, 2, 8)
    a, b = P.workspace_size(good, 256), P.workspace_size(good, 4096)
    assert 0 < a < b and a % 256 == 0
    for bad, status in [
        (P.make_config(4096, 14336, 8, 9, 8), -1),        # top_k > n_experts
        (P.make_config(4096, 14336, 8, 2, 0), -1),        # way < 1
        (P.make_config(4096, 14336, 0, 1, 1), -1),        # no experts
        (P.make_config(4100, 14336, 8, 2, 8), -2),        # d not a multiple of 64
        (P.make_config(4096, 100, 8, 2, 8), -2),          # F not a multiple of 64
        (P.make_config(4096, 14336, 300, 2, 8), -2),      # too many experts
        (P.make_config(4096, 14336, 8, 2, 8, 1, 0), -2),  # shared expert without a width
        (P.make_config(4096, 14336, 8, 2, 8, score_fn=7), -1),
    ]:
        with pytest.raises(P.MoeError) as ei:
            P.workspace_size(bad, 128)
        assert ei.value.status == status, bad
    with pytest.raises(P.MoeError) as ei:
        P.workspace_size(good, 0)
    assert ei.value.status == -1


def test_a_workspace_sized_for_t_max_serves_every_smaller_batch():
    """moe_route / moe_forward / moe_build_united / moe_distill_united take the bytes moe_workspace_size
    gives for THEIR T (the same carving code), so a workspace sized for T_max serves every T <= T_max iff
    the size never shrinks as T grows.  Checked for every T on small shapes and on a dense grid of T on the
    benchmark shapes (where the number of K planes of Y, which falls as T grows, used to make it shrink)."""
    shapes = [
        P.make_config(4096, 14336, 8, 2, 8),                       # Mixtral
        P.make_config(2048, 768, 128, 8, 8),                       # Qwen3-30B-A3B
        P.make_config(7168, 2048, 256, 8, 8, 1, 2048, 1),          # DeepSeek-V3 shape
        P.make_config(2048, 1408, 60, 4, 8, 1, 5632),              # Qwen1.5-MoE shape (shared expert of its own width)
        P.make_config(256, 512, 8, 2, 8),
        P.make_config(64, 64, 4, 2, 2, 2, 128),
        B.with_packed_gate(P.make_config(4096, 14336, 8, 2, 8)),
    ]
    for cfg in shapes:
        dense = cfg.d_model <= 256
        ts = list(range(1, 2200)) if dense else sorted(set(list(range(1, 4200, 7)) + list(range(370, 400)) +
                                                        list(range(1500, 1560)) + [4096, 8192, 16384, 20000]))
        prev = 0
        for T in ts:
            n = P.workspace_size(cfg, T)
            assert n >= prev, f"workspace shrinks from {prev} to {n} at T={T} (d={cfg.d_model}, m={cfg.n_experts})"
            assert n % 256 == 0
            prev = n
    # the trainer's workspace contains the forward workspace for the same number of tokens
    cfg = P.make_config(4096, 14336, 8, 2, 8)
    n = C.c_size_t(0)
    for n_calib in (64, 384, 512, 1024):
        assert P.lib().moe_distill_workspace_size(C.byref(cfg), n_calib, C.byref(n)) == 0
        assert n.value >= P.workspace_size(cfg, n_calib)


def test_packed_gate_size_and_validation():
    L = P.lib()
    cfg = P.make_config(256, 512, 8, 2, 8)
    n = C.c_size_t(0)
    assert L.moe_gate_packed_size(C.byref(cfg), C.byref(n)) == 0
    assert n.value == 3 * 16 * 256 * 2                       # three bf16 pieces of the 16-row padded matrix
    assert L.moe_gate_packed_size(C.byref(cfg), None) == -1
    assert L.moe_pack_gate(C.byref(cfg), None, _fake(), n.value, None) == -1
    assert L.moe_pack_gate(C.byref(cfg), _fake(), None, n.value, None) == -1
    assert L.moe_pack_gate(C.byref(cfg), _fake(), _fake(0x20000), n.value - 1, None) == -4
    assert L.moe_pack_gate(C.byref(cfg), _fake(0x10004), _fake(0x20000), n.value, None) == -3
    bad = P.make_config(256, 512, 8, 2, 8, gate_format=5)
    with pytest.raises(P.MoeError) as ei:
        P.workspace_size(bad, 64)
    assert ei.value.status == -1
    # a packed gate needs no room for the pieces in the workspace (nor does an fp32 gate of at most 16 experts,
    # which is read as it is)
    cfg32 = P.make_config(256, 512, 32, 2, 8)
    assert P.workspace_size(B.with_packed_gate(cfg32), 64) < P.workspace_size(cfg32, 64)
    assert P.workspace_size(B.with_packed_gate(cfg), 64) == P.workspace_size(cfg, 64)
    assert P.workspace_size(B.with_packed_gate(cfg), 4096) == P.workspace_size(cfg, 4096)


def test_activations_beyond_32_bit_offsets_are_refused():
    cfg = P.make_config(4096, 14336, 8, 2, 8)
    with pytest.raises(P.MoeError) as ei:
        P.workspace_size(cfg, 600000)                        # T*d*2 bytes >= 4 GiB
    assert ei.value.status == -5


def test_route_static_validates_and_rejects_batches_beyond_its_scratch():
    L = P.lib()
    cfg = P.make_config(256, 512, 8, 2, 8)
    ro = B.moe_route_out()

    def rs(x=_fake(), T=64, gw=_fake(0x20000), thr=1.0, out=C.byref(ro), c=cfg):
        return L.moe_route_static(C.byref(c), x, T, gw, None, thr, 0, out, None)

    assert rs(thr=1.5) == -1
    assert rs(T=0) == -1
    assert rs(x=None) == -1
    assert rs(out=None) == -1
    assert rs(x=_fake(0x10004)) == -3
    big = P.make_config(7168, 2048, 256, 8, 8, 1, 2048, 1)     # unpacked gate alone is 11 MB: beyond the 8 MiB
    assert rs(c=big, T=64) == -4
    assert rs(T=200000) == -4                                 # row lists beyond the 8 MiB


def _fake(addr=0x10000):
    return C.c_void_p(addr)


def test_route_and_forward_validate_before_launching():
    """Dummy non-null pointers: every one of these calls must fail in host-side validation,
    i.e. return an error without dereferencing anything."""
    L = P.lib()
    cfg = P.make_config(256, 512, 8, 2, 8)
    ro = B.moe_route_out()
    ws_bytes = P.workspace_size(cfg, 64)

    def route(x=_fake(), T=64, gw=_fake(0x20000), thr=1.0, out=C.byref(ro), ws=_fake(0x100000), nbytes=None):
        return L.moe_route(C.byref(cfg), x, T, gw, None, thr, 0, out, ws, ws_bytes if nbytes is None else nbytes, None)

    assert route(thr=1.5) == -1
    assert route(thr=-0.1) == -1
    assert route(thr=float("nan")) == -1
    assert route(T=0) == -1
    assert route(x=None) == -1
    assert route(gw=None) == -1
    assert route(out=None) == -1
    assert route(x=_fake(0x10004)) == -3
    assert route(ws=None) == -4
    assert route(nbytes=ws_bytes - 1) == -4

    w = B.moe_ffn_weights(0x30000, 0x40000, 0x50000)

    def fwd(thr=1.0, united=None, shared=None, experts=C.byref(w), out=_fake(0x60000), full=0, nbytes=ws_bytes):
        return L.moe_forward(C.byref(cfg), _fake(), 64, _fake(0x20000), None, experts, united, shared, thr, full,
                             None, out, _fake(0x100000), nbytes, None)

    assert fwd(thr=0.5) == -1                 # partial brownout needs united experts
    assert fwd(experts=None) == -1
    assert fwd(out=None) == -1
    assert fwd(shared=C.byref(w)) == -1       # shared weights given but n_shared == 0
    assert fwd(thr=2.0) == -1
    assert fwd(nbytes=16) == -4
    half = B.moe_ffn_weights(0x30000, None, 0x50000)
    assert fwd(experts=C.byref(half)) == -1
    cfg_s = P.make_config(256, 512, 8, 2, 8, 1, 512)
    assert L.moe_forward(C.byref(cfg_s), _fake(), 64, _fake(0x20000), None, C.byref(w), None, None, 1.0, 0, None,
                         _fake(0x60000), _fake(0x100000), 1 << 40, None) == -1      # shared expert weights missing


def test_build_united_validates():
    L = P.lib()
    cfg = P.make_config(256, 512, 8, 2, 4)
    w = B.moe_ffn_weights(0x30000, 0x40000, 0x50000)
    assert L.moe_build_united(C.byref(cfg), None, C.byref(w), None, 0, None, None, 0, None) == -1
    assert L.moe_build_united(C.byref(cfg), C.byref(w), None, None, 0, None, None, 0, None) == -1
    assert L.moe_build_united(C.byref(cfg), C.byref(w), C.byref(w), None, -1, None, None, 0, None) == -1
    # calibration requested but no workspace
    assert L.moe_build_united(C.byref(cfg), C.byref(w), C.byref(w), _fake(), 16, _fake(0x70000), None, 0, None) == -4


def test_distill_workspace_and_validation_on_the_host():
    """The distillation entry points reject bad arguments before any device work (dummy pointers)."""
    L = P.lib()
    cfg = P.make_config(256, 512, 8, 2, 4)
    n = C.c_size_t(0)
    assert L.moe_distill_workspace_size(C.byref(cfg), 128, C.byref(n)) == 0
    assert n.value > P.workspace_size(cfg, 128) and n.value % 256 == 0
    assert L.moe_distill_workspace_size(C.byref(cfg), 96, C.byref(n)) == -2       # not a multiple of 64
    assert L.moe_distill_workspace_size(C.byref(cfg), 0, C.byref(n)) == -2
    assert L.moe_distill_workspace_size(C.byref(cfg), 128, None) == -1
    w = B.moe_ffn_weights(_fake(0x10000), _fake(0x20000), _fake(0x30000))

    def distill(n_calib=128, steps=1, lr=1e-3, x=_fake(0x40000), ws=_fake(0x100000), nbytes=1 << 40, ex=C.byref(w)):
        return L.moe_distill_united(C.byref(cfg), ex, C.byref(w), x, n_calib, steps, lr, None, ws, nbytes, None)

    assert distill(n_calib=100) == -2
    assert distill(steps=-1) == -1
    assert distill(lr=-1.0) == -1
    assert distill(lr=float("nan")) == -1
    assert distill(x=None) == -1
    assert distill(ex=None) == -1
    assert distill(ws=None) == -4
    assert distill(nbytes=1024) == -4
    assert distill(ws=_fake(0x100010)) == -3                                      # workspace not 256-byte aligned


def test_probes_validate_on_the_host():
    L = P.lib()
    r = C.c_double(0.0)
    assert L.moe_probe_mfma(None, 65536, _fake(), 2 << 20, None, C.byref(r)) == -1
    assert L.moe_probe_mfma(_fake(), 65536, _fake(0x200000), 2 << 20, None, None) == -1
    assert L.moe_probe_mfma(_fake(), 1024, _fake(0x200000), 2 << 20, None, C.byref(r)) == -4
    assert L.moe_probe_mfma(_fake(), 65536, _fake(0x200000), 1024, None, C.byref(r)) == -4
    assert L.moe_probe_mfma(_fake(0x10004), 65536, _fake(0x200000), 2 << 20, None, C.byref(r)) == -3
    assert L.moe_probe_hbm_read(None, 1 << 30, _fake(), 4, None, C.byref(r)) == -1
    assert L.moe_probe_hbm_read(_fake(), 1024, _fake(0x200000), 4, None, C.byref(r)) == -4
    assert L.moe_probe_hbm_read(_fake(), 1 << 30, _fake(0x200000), 0, None, C.byref(r)) == -4
