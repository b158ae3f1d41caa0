"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on seeded inputs small enough for the oracle to finish in seconds but spanning several tiles,
ragged tails and the degenerate cases of the method."""
import numpy as np
import pytest
import torch

import paper_2507_17133_amd as P
from oracle import oracle as O
from paper_2507_17133_amd import workloads as WL
from tests._util import OUT_TOL, check_route, npf, oracle_route, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _layer(cfg, seed=0):
    torch.cuda.set_device(0)
    L = WL.make_layer(cfg, seed, "cpu")
    to = lambda t: None if t is None else t.to(DEV)
    Lg = WL.Layer(cfg, to(L.x), to(L.gate_w), to(L.gate_b), tuple(to(a) for a in L.experts),
                  None if L.shared is None else tuple(to(a) for a in L.shared), L.popularity)
    return L, Lg


SMALL = {
    # name: (config, thresholds)
    "tiny": (WL.CONFIGS["tiny"], [1.0, 0.75, 0.0]),
    "tiny_way2": (WL.CONFIGS["tiny"].with_(way=2), [0.6, 0.3]),
    "tiny_way3": (WL.CONFIGS["tiny"].with_(way=3), [0.5]),
    "ragged_T": (WL.LayerConfig("ragged_T", T=333, d=128, F=192, m=12, K=3, way=4, zipf_s=1.0), [1.0, 0.5, 0.0]),
    "one_token": (WL.LayerConfig("one_token", T=1, d=64, F=64, m=4, K=2, way=2), [1.0, 0.0]),
    "one_expert": (WL.LayerConfig("one_expert", T=70, d=128, F=256, m=1, K=1, way=1), [1.0]),
    "k_equals_m": (WL.LayerConfig("k_equals_m", T=50, d=64, F=128, m=4, K=4, way=2), [1.0, 0.4]),
    "many_experts": (WL.LayerConfig("many_experts", T=700, d=256, F=128, m=128, K=8, way=8, zipf_s=1.0),
                     [1.0, 0.5, 0.0]),
    "max_experts_sigmoid_shared": (WL.LayerConfig("max_experts", T=300, d=192, F=128, m=256, K=8, way=8, n_shared=1,
                                                  F_s=128, score_fn=1, zipf_s=1.1), [1.0, 0.6]),
    "shared_other_width": (WL.LayerConfig("shared_other_width", T=130, d=128, F=256, m=6, K=2, way=4, n_shared=2,
                                          F_s=64), [1.0, 0.5]),
    "sixty_experts_way8": (WL.LayerConfig("sixty", T=260, d=128, F=64, m=60, K=4, way=8, zipf_s=1.0), [0.4]),
    "way_above_m": (WL.LayerConfig("way_above_m", T=90, d=64, F=64, m=5, K=2, way=16), [0.5]),
    "tiled_gate_2groups": (WL.LayerConfig("tiled_gate_2groups", T=6200, d=128, F=64, m=96, K=4, way=8, zipf_s=1.0),
                           [0.5]),
    "tiled_gate_4groups": (WL.LayerConfig("tiled_gate_4groups", T=12500, d=64, F=64, m=60, K=3, way=8, score_fn=1),
                           [1.0, 0.3]),
    # more than 128 experts in blocks of 32 tokens (wave layout: two token tiles x two expert tiles, 8 groups)
    "tiled_gate_200_experts": (WL.LayerConfig("tiled_gate_200_experts", T=6200, d=64, F=64, m=200, K=8, way=8,
                                              zipf_s=1.0), [0.5]),
    # 128 experts in blocks of 64 tokens (narrow k stages, 8 expert groups of one tile)
    "tiled_gate_128_experts": (WL.LayerConfig("tiled_gate_128_experts", T=12400, d=64, F=64, m=128, K=6, way=8,
                                              score_fn=1), [0.4]),
    "mid_tile": (WL.LayerConfig("mid_tile", T=600, d=128, F=256, m=8, K=2, way=4), [1.0, 0.5]),
    "multi_tile": (WL.LayerConfig("multi_tile", T=1500, d=256, F=384, m=4, K=2, way=4, zipf_s=1.2), [1.0, 0.7]),
    # 256-row tiles with long K: the persistent GEMM cuts the tiles left over after its last full round of one
    # tile per block along K.  Fewer tiles than blocks, ragged last tile: GEMM2 cut four ways ...
    "k_split_tail_gemm2": (WL.LayerConfig("k_split_tail_gemm2", T=500, d=1024, F=4096, m=2, K=2, way=2), [0.0, 1.0]),
    # ... GEMM1 cut three ways (SwiGLU applied to the summed slices) ...
    "k_split_tail_gemm1": (WL.LayerConfig("k_split_tail_gemm1", T=500, d=4096, F=512, m=2, K=2, way=2), [0.0]),
    # ... and more tiles than blocks in GEMM1: one round of whole tiles, then the remainder cut eight ways
    "k_split_tail_after_full_round": (WL.LayerConfig("k_split_tail_full", T=2200, d=4096, F=4096, m=2, K=2, way=2),
                                      [0.0]),
    # 384 expected rows per expert and more: the persistent 256-row kernel on strongly skewed loads (hot experts
    # of many tiles beside cold ones of a few rows), with and without a shared expert in the same launch
    "skewed_256_row_tiles": (WL.LayerConfig("skewed_256_row_tiles", T=2600, d=256, F=384, m=6, K=1, way=3, zipf_s=2.0),
                             [1.0, 0.6]),
    "skewed_with_shared": (WL.LayerConfig("skewed_with_shared", T=1700, d=128, F=256, m=4, K=2, way=2, n_shared=1,
                                            F_s=256, zipf_s=1.5), [1.0, 0.5]),
    # shared experts of their own width in a batch whose routed rows are few enough for K planes of Y: the
    # persistent 256-row kernel runs the shared rows with the K split over the planes ...
    "shared_own_width_k_planes": (WL.LayerConfig("shared_own_width_k_planes", T=600, d=128, F=2048, m=16, K=2, way=4,
                                                 n_shared=1, F_s=1024), [1.0, 0.5]),
    # ... also when the shared experts have fewer k tiles than there are planes (empty slices: zeros)
    "shared_narrower_than_planes": (WL.LayerConfig("shared_narrower_than_planes", T=600, d=128, F=2048, m=16, K=2,
                                                   way=4, n_shared=1, F_s=64), [1.0]),
    # at most 16 experts: the plain fp64 gate up to 2048 tokens, the MFMA gate (pieces cut from the fp32 rows on the
    # way, whichever format the caller passes) from 2049 on
    "few_experts_2048_tokens": (WL.LayerConfig("few_experts_2048_tokens", T=2048, d=64, F=64, m=16, K=3, way=4,
                                               zipf_s=1.0), [0.5]),
    "few_experts_2049_tokens": (WL.LayerConfig("few_experts_2049_tokens", T=2049, d=64, F=64, m=16, K=3, way=4,
                                               zipf_s=1.0), [0.5]),
    # the largest K and number of shared experts the library accepts
    "max_topk_max_shared": (WL.LayerConfig("max_topk_max_shared", T=48, d=64, F=64, m=64, K=32, way=8, n_shared=8,
                                           F_s=64), [1.0, 0.5]),
}


def _cases():
    for name, (cfg, thrs) in SMALL.items():
        for thr in thrs:
            for full in ((False, True) if 0.0 < thr < 1.0 and name in ("tiny", "ragged_T", "many_experts") else (False,)):
                yield pytest.param(cfg, thr, full, id=f"{name}-thr{thr}-{'full' if full else 'partial'}")


@pytest.mark.parametrize("cfg,thr,full", list(_cases()))
def test_route_and_forward(cfg, thr, full):
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    ref = oracle_route(L, cfg, thr, full)
    R = P.moe_route(c, Lg.x, Lg.gate_w, Lg.gate_b, thr, full)
    torch.cuda.synchronize()
    idx, w, unit = check_route(R, ref, cfg, thr, full)

    united_cpu = WL.make_random_united(cfg, 0, "cpu")
    united = tuple(a.to(DEV) for a in united_cpu)
    out = P.moe_forward(c, Lg.x, Lg.gate_w, Lg.gate_b, Lg.experts, united, Lg.shared, thr, full)
    out_r = P.moe_forward(c, Lg.x, None, None, Lg.experts, united, Lg.shared, route=R)
    # the gate matrix repacked once instead of on every call: same bits everywhere
    cp, gp = P.with_packed_gate(c), P.pack_gate(c, Lg.gate_w)
    Rp = P.moe_route(cp, Lg.x, gp, Lg.gate_b, thr, full)
    out_p = P.moe_forward(cp, Lg.x, gp, Lg.gate_b, Lg.experts, united, Lg.shared, thr, full)
    torch.cuda.synchronize()
    for f in ("topk_idx", "topk_w", "expert_cnt", "expert_unit", "unit_cnt", "unit_off", "token_rows", "n_rows"):
        assert torch.equal(getattr(R, f), getattr(Rp, f)), f
    assert torch.equal(out, out_p)
    want = O.forward_tokens(npf(L.x), idx, w, unit, cfg.way, npf(L.experts), npf(united_cpu), npf(L.shared))
    got = npf(out)
    assert np.isfinite(got).all()
    e = rel_err(got, want)
    assert e <= OUT_TOL, f"max relative error {e}"
    assert torch.equal(out, out_r), "forward with a precomputed route must equal routing internally"


def test_workspace_reuse_and_side_stream():
    """One workspace, sized for the larger batch, serves calls of different sizes on a caller's stream: what an
    earlier call left in it (row lists, tile tables, partial tiles of the K-split tail) must not show."""
    big, _ = SMALL["k_split_tail_gemm2"]
    small = big.with_(T=300)
    c_big, c_small = P.config_of(big), P.config_of(small)
    Lb, Lgb = _layer(big, seed=1)
    Ls, Lgs = _layer(small, seed=2)
    united = tuple(a.to(DEV) for a in WL.make_random_united(big, 0, "cpu"))
    fresh_big = P.moe_forward(c_big, Lgb.x, Lgb.gate_w, Lgb.gate_b, Lgb.experts, united, None, 0.0)
    fresh_small = P.moe_forward(c_small, Lgs.x, Lgs.gate_w, Lgs.gate_b, Lgb.experts, united, None, 0.5)
    torch.cuda.synchronize()
    ws = P.alloc_workspace(c_big, big.T, DEV)
    ws.fill_(0xA5)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        a = P.moe_forward(c_big, Lgb.x, Lgb.gate_w, Lgb.gate_b, Lgb.experts, united, None, 0.0, workspace=ws, stream=side)
        b = P.moe_forward(c_small, Lgs.x, Lgs.gate_w, Lgs.gate_b, Lgb.experts, united, None, 0.5, workspace=ws, stream=side)
        a2 = P.moe_forward(c_big, Lgb.x, Lgb.gate_w, Lgb.gate_b, Lgb.experts, united, None, 0.0, workspace=ws, stream=side)
    side.synchronize()
    assert torch.equal(a, fresh_big) and torch.equal(a2, fresh_big)
    assert torch.equal(b, fresh_small)


def test_hand_made_rows_hot_and_cold_units_side_by_side():
    """Row lists brought by the caller (moe_forward with route != NULL; the tile table is then built by the
    stand-alone kernel): units of 3000, 1, 129, 64, 65, 0, 257 and 128 rows in one batch, so one grouped launch
    holds a unit of many whole tiles, ragged last tiles of every fill, a one-row unit and an empty one."""
    torch.cuda.set_device(0)
    counts = [3000, 1, 129, 64, 65, 0, 257, 128]
    m, K = len(counts), 1
    T = sum(counts)
    cfg = WL.LayerConfig("hand_made", T=T, d=256, F=320, m=m, K=K, way=4)
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    rng = np.random.default_rng(7)
    idx = np.repeat(np.arange(m, dtype=np.int32), counts)
    rng.shuffle(idx)
    idx = idx.reshape(T, 1)
    w = rng.uniform(0.25, 1.0, size=(T, 1)).astype(np.float32)
    unit = np.arange(m, dtype=np.int32)
    rows = O.build_rows(idx, w, m, cfg.way, 0, unit)
    assert rows.unit_cnt[:m].tolist() == counts
    R = P.alloc_route_out(c, T, DEV)
    put = lambda dst, a: dst[:len(a)].copy_(torch.from_numpy(np.ascontiguousarray(a)).to(DEV))
    put(R.expert_unit, unit); put(R.unit_cnt, rows.unit_cnt); put(R.unit_off, rows.unit_off)
    put(R.row_token, rows.row_token); put(R.row_weight, rows.row_weight)
    R.token_rows.copy_(torch.from_numpy(rows.token_rows).to(DEV))
    out = P.moe_forward(c, Lg.x, None, None, Lg.experts, None, None, route=R)
    torch.cuda.synchronize()
    want = O.forward_tokens(npf(L.x), idx, w, unit, cfg.way, npf(L.experts))
    got = npf(out)
    assert np.isfinite(got).all()
    per_unit = {u: rel_err(got[idx[:, 0] == u], want[idx[:, 0] == u]) for u in range(m) if counts[u]}
    assert max(per_unit.values()) <= OUT_TOL, per_unit


def test_first_call_of_a_process_can_be_the_captured_one():
    """A fresh process sizes its workspace (which performs the library's per-device set-up) and then makes its
    very FIRST moe_forward under stream capture; the replayed graph must give the eager result."""
    import subprocess
    import sys
    code = r'''
import sys, torch
sys.path.insert(0, %r)
import paper_2507_17133_amd as P
from paper_2507_17133_amd import workloads as WL
torch.cuda.set_device(0)
for name, cfg in (("small", WL.LayerConfig("g", T=600, d=128, F=256, m=8, K=2, way=4)),
                  ("tiled_gate_and_256_row_tiles", WL.LayerConfig("g2", T=6200, d=128, F=64, m=96, K=4, way=8, zipf_s=1.0, n_shared=1, F_s=64))):
    L = WL.make_layer(cfg, 3, "cuda")
    united = WL.make_random_united(cfg, 0, "cuda")
    c = P.config_of(cfg)
    ws = P.alloc_workspace(c, cfg.T)                       # moe_workspace_size: per-device set-up happens here
    out = torch.empty_like(L.x)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        P.moe_forward(c, L.x, L.gate_w, L.gate_b, L.experts, united, L.shared, 0.5, out=out, workspace=ws)
    g.replay(); torch.cuda.synchronize()
    first = out.clone()
    eager = P.moe_forward(c, L.x, L.gate_w, L.gate_b, L.experts, united, L.shared, 0.5)
    g.replay(); torch.cuda.synchronize()
    assert torch.equal(first, eager) and torch.equal(out, eager), name
print("captured-first ok")
''' % (str(__import__("pathlib").Path(__file__).resolve().parents[1]),)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "captured-first ok" in r.stdout, r.stdout + r.stderr


@pytest.mark.parametrize("name", ["mid_tile", "k_split_tail_gemm2"])
def test_forward_replays_from_a_hip_graph(name):
    """moe_forward launches kernels only, so a caller can capture it; every replay, with eager work on other
    inputs in between, must give the eager result for whatever the input buffer holds at that moment."""
    cfg, _ = SMALL[name]
    thr = 0.5
    c = P.config_of(cfg)
    L, Lg = _layer(cfg, seed=3)
    _, Lg2 = _layer(cfg, seed=4)
    united = tuple(a.to(DEV) for a in WL.make_random_united(cfg, 0, "cpu"))
    x_buf = Lg.x.clone()
    out_buf = torch.empty_like(x_buf)
    ws = P.alloc_workspace(c, cfg.T, DEV)

    def eager(x):
        return P.moe_forward(c, x, Lg.gate_w, Lg.gate_b, Lg.experts, united, Lg.shared, thr)

    want1, want2 = eager(Lg.x), eager(Lg2.x)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        P.moe_forward(c, x_buf, Lg.gate_w, Lg.gate_b, Lg.experts, united, Lg.shared, thr, out=out_buf, workspace=ws)
    for x_new, want in ((Lg.x, want1), (Lg2.x, want2), (Lg.x, want1)):
        x_buf.copy_(x_new)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_buf, want)
        assert torch.equal(eager(Lg2.x), want2)        # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["tiny", "few_experts_2049_tokens", "sixty_experts_way8", "many_experts",
                                  "tiled_gate_2groups", "tiled_gate_200_experts", "max_topk_max_shared"])
def test_exact_ties_go_to_the_lower_expert_id(name):
    """All-zero activations: every affinity is exactly equal, so TopK must list experts 0..K-1 for every token
    (lower id wins: in the fp64 gate, the MFMA gate for few experts, the LDS-staged gate with 4, 8 and 16
    candidate registers per lane and with one token per wavefront), every token is flagged as a near tie, the weights are
    1/K, and the layer output is zero (FFN(0) = 0)."""
    cfg, _ = SMALL[name]
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    x0 = torch.zeros_like(Lg.x)
    R = P.moe_route(c, x0, Lg.gate_w, None, 1.0)
    out = P.moe_forward(c, x0, Lg.gate_w, None, Lg.experts, None, Lg.shared, 1.0)
    torch.cuda.synchronize()
    idx = npf(R.topk_idx)
    assert (idx == np.arange(cfg.K)[None, :]).all()
    assert np.allclose(npf(R.topk_w), 1.0 / cfg.K, rtol=1e-6)
    assert (npf(R.near_tie) == 1).all() or cfg.K == cfg.m
    cnt = npf(R.expert_cnt)
    assert (cnt[:cfg.K] == cfg.T).all() and (cnt[cfg.K:] == 0).all()
    assert (npf(out) == 0).all()


def test_ceiling_probes_give_plausible_rates():
    """The two measurement aids: a pure MFMA loop cannot beat the chip's nominal 2.5 PFLOP/s and constant
    operand bits are never slower than random ones; a read-only sweep cannot beat 8 TB/s."""
    torch.cuda.set_device(0)
    rnd = torch.randn(1 << 16, device=DEV).to(torch.bfloat16)
    t_rnd = P.probe_mfma(rnd)
    t_one = P.probe_mfma(torch.ones(1 << 16, dtype=torch.bfloat16, device=DEV))
    assert 200.0 < t_rnd <= 2600.0 and 200.0 < t_one <= 2600.0
    assert t_one >= 0.95 * t_rnd
    gbs = P.probe_hbm_read(torch.ones(1 << 30, dtype=torch.uint8, device=DEV))
    assert 1000.0 < gbs <= 8200.0


def test_empty_batch_is_rejected():
    cfg = WL.CONFIGS["tiny"]
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    x0 = Lg.x[:0].contiguous()
    with pytest.raises(P.MoeError) as ei:
        P.moe_forward(c, x0, Lg.gate_w, Lg.gate_b, Lg.experts, None, None, 1.0,
                      out=torch.empty((0, cfg.d), dtype=torch.bfloat16, device=DEV),
                      workspace=P.alloc_workspace(c, 1, DEV))
    assert ei.value.status == -1


def test_residual():
    cfg = WL.CONFIGS["tiny"]
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    c.add_residual = 1
    ref = oracle_route(L, cfg, 1.0)
    out = P.moe_forward(c, Lg.x, Lg.gate_w, Lg.gate_b, Lg.experts, None, None, 1.0)
    want = O.forward_tokens(npf(L.x), ref.topk_idx, ref.topk_w, ref.expert_unit, cfg.way, npf(L.experts),
                            add_residual=True)
    assert rel_err(npf(out), want) <= OUT_TOL


def test_full_brownout_threshold_zero_outputs_zero():
    cfg = WL.CONFIGS["tiny"]
    L, Lg = _layer(cfg)
    out = P.moe_forward(P.config_of(cfg), Lg.x, Lg.gate_w, Lg.gate_b, Lg.experts, None, None, 0.0, True)
    assert (npf(out) == 0).all()


def test_threshold_sweep_is_monotone_in_united_rows():
    cfg = SMALL["many_experts"][0]
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    prev = None
    for thr in [0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]:
        R = P.moe_route(c, Lg.x, Lg.gate_w, Lg.gate_b, thr)
        ref = oracle_route(L, cfg, thr)
        check_route(R, ref, cfg, thr, False)
        s1 = set(np.nonzero(npf(R.expert_in_s1))[0].tolist())
        if prev is not None:
            assert prev <= s1
        prev = s1


def test_build_united_mean_and_loss():
    cfg = WL.LayerConfig("united", T=96, d=128, F=192, m=7, K=2, way=3)
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    calib_cpu = WL.make_activations(cfg, 0, "cpu", name="calib", n=96)
    united, loss = P.moe_build_united(c, Lg.experts, calib_cpu.to(DEV))
    torch.cuda.synchronize()
    for k in range(3):
        mean = O.united_mean(npf(L.experts[k]), cfg.way)                      # double
        # round to bf16 (8 significant bits), nearest-even, straight from the double
        mant, ex = np.frexp(mean)
        want = np.ldexp(np.rint(mant * 256.0), ex - 8).astype(np.float32)
        assert (npf(united[k]) == want).all()
    ref_loss = O.united_loss(npf(calib_cpu), cfg.way, npf(L.experts), npf(united))
    got = npf(loss)
    assert np.allclose(got, ref_loss, rtol=3e-2, atol=1e-6), (got, ref_loss)
    assert abs(got[2]) < 1e-6                                                   # single-member group
    # way = 1: every united expert is its expert, loss 0
    c1 = P.config_of(cfg.with_(way=1))
    u1, l1 = P.moe_build_united(c1, Lg.experts, calib_cpu.to(DEV))
    for k in range(3):
        assert torch.equal(u1[k], Lg.experts[k])
    assert (npf(l1) == 0).all()


def test_build_united_loss_with_a_large_calibration_batch():
    """512 calibration tokens: the FFNs behind the loss run in 256-row tiles, and the workspace the binding
    allocates (moe_workspace_size for 512 tokens) must be enough."""
    cfg = WL.LayerConfig("united512", T=512, d=128, F=256, m=4, K=2, way=2)
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    calib_cpu = WL.make_activations(cfg, 0, "cpu", name="calib", n=512)
    united, loss = P.moe_build_united(c, Lg.experts, calib_cpu.to(DEV))
    torch.cuda.synchronize()
    ref_loss = O.united_loss(npf(calib_cpu), cfg.way, npf(L.experts), npf(united))
    assert np.allclose(npf(loss), ref_loss, rtol=3e-2, atol=1e-6), (npf(loss), ref_loss)


def test_identical_group_members_hide_brownout():
    cfg = WL.LayerConfig("ident", T=200, d=128, F=128, m=6, K=2, way=3)
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    ex = tuple(a[::3].repeat_interleave(3, dim=0).contiguous() for a in Lg.experts)
    un = tuple(a[::3].contiguous() for a in Lg.experts)
    base = P.moe_forward(c, Lg.x, Lg.gate_w, Lg.gate_b, ex, un, None, 1.0)
    for thr in (0.6, 0.0):
        out = P.moe_forward(c, Lg.x, Lg.gate_w, Lg.gate_b, ex, un, None, thr)
        assert rel_err(npf(out), npf(base)) <= 1e-2      # same FFNs, rows merged: only bf16 rounding differs


def test_errors_are_reported_before_any_launch():
    cfg = WL.CONFIGS["tiny"]
    L, Lg = _layer(cfg)
    c = P.config_of(cfg)
    with pytest.raises(P.MoeError) as ei:
        P.moe_route(c, Lg.x, Lg.gate_w, None, 1.5)
    assert ei.value.status == -1
    with pytest.raises(P.MoeError) as ei:
        P.moe_forward(c, Lg.x, Lg.gate_w, None, Lg.experts, None, None, 0.5)      # united missing
    assert ei.value.status == -1
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(P.MoeError) as ei:
        P.moe_route(c, Lg.x, Lg.gate_w, None, 1.0, workspace=small)
    assert ei.value.status == -4
