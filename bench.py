#!/usr/bin/env python3
"""Benchmark of the BrownoutMoE layer forward on one MI355X.

A step = one moe_forward call (gate, TopK, Algorithm 1, row scatter, both grouped GEMMs, combine)
on a batch of synthetic tokens resident in HBM.  Default workload: the Mixtral-8x7B-shaped prefill
layer (T=4096, d=4096, F=14336, 8 experts, top-2, Zipf(1.2) expert load, brownout fraction 0.3,
one 8-way united expert).  Prints ONE JSON line on stdout; everything else goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mixtral_prefill")
    ap.add_argument("--fraction", type=float, default=None, help="brownout fraction f (threshold = 1-f)")
    ap.add_argument("--way", type=int, default=None)
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true",
                    help="default workload only: skip the decode-sized sub-record (mixtral_decode at f = 0 and f = 1)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=None)
    ap.add_argument("--stages", action="store_true", help="also print a per-kernel time breakdown to stderr")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the layer at thresholds 1.0 .. 0.0, partial and full brownout (to stderr)")
    ap.add_argument("--salc", action="store_true",
                    help="also run the SLO-aware latency controller over a synthetic burst trace (to stderr)")
    ap.add_argument("--salc-layers", type=int, default=24, help="MoE layers per serving iteration in --salc")
    ap.add_argument("--no-probes", action="store_true",
                    help="skip the two ceiling probes (pure MFMA loop on this workload's weight bits, read-only sweep)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured HIP graph (to stderr)")
    ap.add_argument("--distill", action="store_true",
                    help="also train the united experts by distillation on synthetic calibration tokens and compare "
                         "the full-brownout layer output before and after (to stderr)")
    ap.add_argument("--distill-steps", type=int, default=100)
    ap.add_argument("--distill-tokens", type=int, default=2048)
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy three times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2507_17133_amd as P
    from paper_2507_17133_amd import workloads as WL

    torch.cuda.set_device(0)
    dev = "cuda"
    if args.copy_probe:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("copy probe: 3 device copies of 1 GiB (each reads 1 GiB and writes 1 GiB)")
        return
    cfg = WL.CONFIGS[args.workload]
    if args.way is not None:
        cfg = cfg.with_(way=args.way)
    if args.tokens is not None:
        cfg = cfg.with_(T=args.tokens)
    f = cfg.brownout_fractions[0] if args.fraction is None else args.fraction
    m = measure(cfg, f, args.steps, args.warmup, dev, default_shape=args.fraction is None and args.way is None
                and args.tokens is None)
    L, united, c, gate, ws, out, threshold = m["L"], m["united"], m["c"], m["gate"], m["ws"], m["out"], m["threshold"]
    line_cfg = m["line_cfg"]
    roofline, ms_per_step, tokens_per_s = m["roofline"], m["ms_per_step"], m["tokens_per_s"]

    def step():
        P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, threshold, False, None, out, ws)

    if args.stages:
        P.profile_enable()
        for _ in range(10):
            step()
        pr = P.profile_collect()
        P.profile_disable()
        log("  per-kernel ms (mean of 10): " + ", ".join(f"{k}={v[0]/max(1,v[1]):.4f}" for k, v in pr.items()))

    if args.graph:
        # the same step captured once and replayed: what a serving loop that cannot afford launch latency would do
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        log(f"  replayed from a HIP graph: {(time.perf_counter() - tg) * 1e3 / args.steps:.3f} ms per step "
            f"(eager launches: {ms_per_step:.3f})")

    if args.sweep:
        # latency against the brownout threshold, 1.0 -> 0.0 in steps of 0.1, partial and full brownout
        # (the grid of the paper's accuracy study, Results / Accuracy; here only the time side of it)
        log(f"  threshold sweep ({cfg.name}, way {cfg.way}): threshold, ms/step partial (rows, active units), ms/step full")
        for i in range(10, -1, -1):
            thr = i / 10.0
            res = []
            for full in (False, True):
                Rs = P.moe_route(c, L.x, gate, L.gate_b, thr, full, workspace=ws)
                torch.cuda.synchronize()
                rows_s, act_s = int(Rs.n_rows.item()), int((Rs.unit_cnt > 0).sum().item())
                for _ in range(3):
                    P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, thr, full, None, out, ws)
                torch.cuda.synchronize()
                ts = time.perf_counter()
                for _ in range(10):
                    P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, thr, full, None, out, ws)
                torch.cuda.synchronize()
                res.append(((time.perf_counter() - ts) * 100.0, rows_s, act_s))
            log(f"    {thr:.1f}   {res[0][0]:8.3f} ({res[0][1]} rows, {res[0][2]} units)   {res[1][0]:8.3f} ({res[1][1]} rows, {res[1][2]} units)")

    if args.salc:
        # Algorithm 2 in a serving loop: the iteration time as a function of the threshold is measured here
        # (args.salc_layers MoE layers per iteration), the request trace is synthetic (Poisson, rate doubling
        # at 75 s of 250 s as in the paper's burst experiment, sized so that threshold 1 is at 45 % load before
        # the burst and at 90 % after it), SLO = 3 x the iteration time without brownout.
        from paper_2507_17133_amd import salc
        thr_grid = [i / 10.0 for i in range(11)]
        t_of = []
        for thr in thr_grid:
            for _ in range(3):
                P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, thr, False, None, out, ws)
            torch.cuda.synchronize()
            ts = time.perf_counter()
            for _ in range(10):
                P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, thr, False, None, out, ws)
            torch.cuda.synchronize()
            t_of.append((time.perf_counter() - ts) / 10.0 * args.salc_layers)
        tau = lambda thr: float(np.interp(thr, thr_grid, t_of))
        tau1 = t_of[-1]
        slo = 3.0 * tau1
        lam = 0.45 / tau1
        arr = salc.poisson_arrivals([(0.0, lam), (75.0, 2.0 * lam)], 250.0, seed=0)
        fixed = salc.serve(arr, tau)
        ctl = salc.serve(arr, tau, slo=slo)
        log(f"  SALC trace ({cfg.name}, way {cfg.way}, {args.salc_layers} layers per iteration): iteration time "
            f"{t_of[0]*1e3:.2f} ms at threshold 0 .. {tau1*1e3:.2f} ms at threshold 1; SLO {slo*1e3:.1f} ms; "
            f"{len(arr)} requests, {lam:.1f}/s doubling at 75 s")
        for nm, tr in (("threshold fixed at 1", fixed), ("SALC", ctl)):
            lat = tr.latency[tr.arrival >= 75.0]
            log(f"    {nm:22s}: SLO violations after the burst {salc.violation_rate(tr, slo, 75.0)*100:6.2f} %  "
                f"(before {(tr.latency[tr.arrival < 75.0] > slo).mean()*100:5.2f} %), P90 latency after the burst "
                f"{np.quantile(lat, 0.9)*1e3:8.1f} ms, mean threshold before / after "
                f"{tr.threshold[tr.arrival < 75.0].mean():.3f} / {tr.threshold[tr.arrival >= 75.0].mean():.3f}")

    if args.distill:
        # United Expert Model section: the student of every group is trained on calibration tokens (a seeded
        # draw of the same distribution as x, other tokens) from the parameter mean; the layer output at
        # threshold 0 (every multi-member group served by its united expert) is compared with the exact
        # layer output before and after the training.
        calib = WL.make_activations(cfg, 1, dev, name="calib", n=args.distill_tokens)
        lr = 0.02 / float(np.sqrt(cfg.d))                # 2 % of the weights' standard deviation per step
        exact = P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, 1.0).float()
        before = P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, 0.0).float()
        trained = tuple(u.clone() for u in united)
        torch.cuda.synchronize()
        ts = time.perf_counter()
        hist = P.moe_distill_united(m["c_plain"], L.experts, trained, calib, args.distill_steps, lr)
        torch.cuda.synchronize()
        dt = time.perf_counter() - ts
        after = P.moe_forward(c, L.x, gate, L.gate_b, L.experts, trained, L.shared, 0.0).float()
        rel = lambda a: float(((a - exact).norm() / exact.norm()).item())
        h = hist.cpu().numpy()
        multi = [g for g in range(cfg.G) if min(cfg.m, (g + 1) * cfg.way) - g * cfg.way > 1]
        log(f"  distillation ({cfg.name}, way {cfg.way}, {len(multi)} groups, {args.distill_tokens} calibration tokens, "
            f"{args.distill_steps} Adam steps, lr {lr:.2e}): {dt:.2f} s = {dt/max(1,len(multi)*max(1,args.distill_steps))*1e3:.2f} ms per "
            f"group step; mean loss {h[multi,0].mean():.4g} -> {h[multi,-1].mean():.4g}; layer output error against "
            f"threshold 1 at threshold 0: parameter mean {rel(before):.4f}, distilled {rel(after):.4f}")

    if not args.no_probes:
        # What this machine sustains on the resource the dominant kernel is priced against, measured after the timed
        # region: a pure MFMA loop whose operand bits are this workload's expert weights (random data draws
        # more power than constants, and the chip clocks down under it), or a read-only sweep of the weights.
        w1 = L.experts[0]
        mfma_data = P.probe_mfma(w1)
        mfma_const = P.probe_mfma(torch.ones(65536, dtype=torch.bfloat16, device=dev))
        hbm_read = P.probe_hbm_read(w1)
        measured = hbm_read if roofline["bound"] == "hbm" else mfma_data
        roofline["measured_ceiling"] = measured
        roofline["frac_of_measured_ceiling"] = roofline["achieved"] / measured
        roofline["ceilings"] = {"mfma_loop_weight_bits_tflops": mfma_data, "mfma_loop_constant_bits_tflops": mfma_const,
                                "hbm_read_gbs": hbm_read}
        log(f"  measured ceilings on this box: pure MFMA loop {mfma_data:.0f} TFLOP/s on the weights' bits "
            f"({mfma_const:.0f} on constants; nominal {PEAK_BF16_TFLOPS:.0f}), read-only sweep {hbm_read:.0f} GB/s "
            f"(nominal {PEAK_HBM_GBS:.0f}); GEMM1 at {roofline['frac_of_measured_ceiling']:.3f} of its measured ceiling")

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, L, united, threshold, args.cpu_sample_tokens)

    # The other half of the metric: the decode-sized batch of the same layer shape (HBM-bound weight streaming),
    # at zero brownout and with every expert delegated to the one united expert (an eighth of the weight bytes).
    decode = None
    if cfg.name == "mixtral_prefill" and not args.no_decode and m["default_shape"]:
        dcfg = WL.CONFIGS["mixtral_decode"]
        d0 = measure(dcfg, 0.0, max(args.steps, 30), args.warmup, dev, default_shape=True)
        d1 = measure(dcfg, 1.0, max(args.steps, 30), args.warmup, dev, default_shape=False, reuse=d0)
        decode = {"workload": dcfg.name, "T": dcfg.T, "brownout_fraction": 0.0, "ms_per_step": d0["ms_per_step"],
                  "tokens_per_s": d0["tokens_per_s"], "route_ms": d0["route_ms"],
                  "layer_roofline_frac": d0["layer_frac"], "bytes_min": d0["bytes_min"],
                  "bytes_two_gemm": d0["bytes_two_gemm"], "roofline": d0["roofline"],
                  "brownout_fraction_1": {"ms_per_step": d1["ms_per_step"], "tokens_per_s": d1["tokens_per_s"],
                                               "bytes_min": d1["bytes_min"], "layer_roofline_frac": d1["layer_frac"],
                                               "gemm1_gbs": d1["roofline"]["achieved"]}}
    line = {
        "metric": "MoE-layer tokens/s at 1 MI355X", "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": line_cfg, "roofline": roofline, "cpu_baseline": cpu, "decode": decode,
    }
    print(json.dumps(line), flush=True)


def measure(cfg, f, steps, warmup, dev, default_shape, reuse=None):
    """Times `steps` moe_forward calls of one workload at brownout fraction f (inputs resident in HBM, the gate
    matrix packed once beforehand) and prices the step and its dominant kernel against the rooflines."""
    import numpy as np
    import torch

    import paper_2507_17133_amd as P
    from paper_2507_17133_amd import workloads as WL

    threshold = 1.0 - f
    c_plain = P.config_of(cfg)
    t0 = time.time()
    if reuse is None:
        L = WL.make_layer(cfg, 0, dev)
        united, _ = P.moe_build_united(c_plain, L.experts)
        gate = P.pack_gate(c_plain, L.gate_w)          # one-time repack of the gate matrix, outside the timed region
    else:
        L, united, gate = reuse["L"], reuse["united"], reuse["gate"]
    c = P.with_packed_gate(c_plain)
    ws = P.alloc_workspace(c, cfg.T, dev)
    out = torch.empty((cfg.T, cfg.d), dtype=torch.bfloat16, device=dev)
    R = P.moe_route(c, L.x, gate, L.gate_b, threshold, workspace=ws)
    torch.cuda.synchronize()
    n_rows = int(R.n_rows.item())
    unit_cnt = R.unit_cnt.cpu().numpy()
    expert_cnt = R.expert_cnt.cpu().numpy()
    n_shared_rows = cfg.T * cfg.n_shared
    n_routed_rows = n_rows - n_shared_rows
    active_units = int((unit_cnt > 0).sum())
    united_rows_before_merge = int(expert_cnt[(R.expert_unit.cpu().numpy() >= cfg.m)].sum())
    log(f"[setup {time.time()-t0:.1f}s] {cfg.name}: T={cfg.T} d={cfg.d} F={cfg.F} m={cfg.m} K={cfg.K} way={cfg.way} "
        f"threshold={threshold:.2f} rows={n_rows} active_units={active_units}/{len(unit_cnt)}")
    log(f"  expert load (tokens): max={expert_cnt.max()} mean={expert_cnt.mean():.1f} min={expert_cnt.min()} "
        f"units with <16 rows: {int(((unit_cnt > 0) & (unit_cnt < 16)).sum())}; realised brownout fraction "
        f"{united_rows_before_merge / float(cfg.T * cfg.K):.3f} (asked {f:.2f})")

    def step():
        P.moe_forward(c, L.x, gate, L.gate_b, L.experts, united, L.shared, threshold, False, None, out, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    P.profile_enable(["gemm1"])          # two HIP events per step around the dominant kernel, on its stream
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    prof = P.profile_collect()
    P.profile_disable()
    ms_per_step = (t2 - t1) * 1e3 / steps
    tokens_per_s = cfg.T * steps / (t2 - t1)
    # routing alone (gate, TopK, Algorithm 1, row lists), same inputs
    for _ in range(3):
        P.moe_route(c, L.x, gate, L.gate_b, threshold, False, R, ws)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for _ in range(20):
        P.moe_route(c, L.x, gate, L.gate_b, threshold, False, R, ws)
    torch.cuda.synchronize()
    route_ms = (time.perf_counter() - t3) * 1e3 / 20

    # GEMM1 time per step (a layer whose shared experts have their own width runs GEMM1 twice per step)
    gemm1_ms = prof["gemm1"][0] / steps
    # algorithmic flops of GEMM1 per launch: rows x (W1 and W3) : 2*2*d*F per row (shared rows with their own F)
    flops_gemm1 = 4.0 * cfg.d * (cfg.F * n_routed_rows + cfg.F_s * n_shared_rows)
    flops_step = 6.0 * cfg.d * (cfg.F * n_routed_rows + cfg.F_s * n_shared_rows) + 2.0 * cfg.T * cfg.d * cfg.m
    # algorithmic bytes per step: x in, out, gate, weights of the ACTIVE units only; and what the two-GEMM
    # design moves on top of that: gathered x rows, H written and read, Y written and read
    unit_bytes = np.where(np.arange(len(unit_cnt)) < cfg.m + cfg.G, 3 * cfg.d * cfg.F * 2, 3 * cfg.d * cfg.F_s * 2)
    bytes_min = 2 * cfg.T * cfg.d * 2 + cfg.d * cfg.m * 4 + int(unit_bytes[unit_cnt > 0].sum())
    h_bytes = 2 * (n_routed_rows * cfg.F + n_shared_rows * cfg.F_s)
    bytes_two_gemm = bytes_min + n_rows * cfg.d * 2 + 2 * h_bytes + 2 * n_rows * cfg.d * 2
    t_mfma = flops_step / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = bytes_min / (PEAK_HBM_GBS * 1e9)
    hbm_bound = t_hbm > t_mfma
    if hbm_bound:
        # weight streaming dominates: price GEMM1 by the bytes it must read (W1, W3 of active units + gathered x)
        g1_bytes = int((unit_bytes[unit_cnt > 0] * 2 // 3).sum()) + n_rows * cfg.d * 2 + h_bytes
        achieved = g1_bytes / (gemm1_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    else:
        achieved = flops_gemm1 / (gemm1_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None}
    # with 256-row tiles GEMM1 is two launches (the GEMM kernel, whose extra blocks take the pieces of the tiles
    # left over after its last full round, and the sum of their K slices): both are inside the timed interval
    roofline["kernel"] = "GEMM1 (ffn_gemm_*_kernel<SWIGLU> and, with 256-row tiles, gemm_tail_sum_kernel)"
    roofline["kernel_ms"] = gemm1_ms
    # HBM-side bytes of one GEMM1 launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by a copy
    # probe) in a separate counter run of this workload: read from the committed summary, not measured here
    tpath = os.path.join(ROOT, "profiles", f"moe_forward_{cfg.name}.txt")
    roofline["traffic_source"] = None
    if os.path.exists(tpath) and default_shape:
        for ln in open(tpath):
            if ln.startswith("gemm1_hbm_bytes_per_launch"):
                roofline["traffic"] = float(ln.split("=")[1].split()[0])
                roofline["traffic_source"] = f"profiles/moe_forward_{cfg.name}.txt (rocprofv3 counter runs, not this run)"
    layer_frac = max(t_mfma, t_hbm) * 1e3 / ms_per_step
    log(f"  step {ms_per_step:.3f} ms  -> {tokens_per_s/1e6:.3f} M tok/s; layer roofline time "
        f"{max(t_mfma, t_hbm)*1e3:.3f} ms ({'HBM' if hbm_bound else 'MFMA'}-bound) -> whole-step fraction "
        f"{layer_frac:.3f}; GEMM1 {gemm1_ms:.3f} ms ({roofline['frac']:.3f} of nominal); routing alone {route_ms:.3f} ms")
    return {"L": L, "united": united, "c": c, "c_plain": c_plain, "gate": gate, "ws": ws, "out": out,
            "threshold": threshold, "roofline": roofline, "ms_per_step": ms_per_step, "tokens_per_s": tokens_per_s,
            "route_ms": route_ms, "layer_frac": layer_frac, "bytes_min": bytes_min, "bytes_two_gemm": bytes_two_gemm,
            "default_shape": default_shape,
            "line_cfg": {"workload": cfg.name, "T": cfg.T, "d_model": cfg.d, "d_ff": cfg.F, "n_experts": cfg.m,
                         "top_k": cfg.K, "way": cfg.way, "n_shared": cfg.n_shared, "brownout_fraction": f,
                         "threshold": threshold, "rows": n_rows, "active_units": active_units,
                         "layer_roofline_frac": layer_frac, "route_ms": route_ms, "bytes_min": bytes_min,
                         "bytes_two_gemm": bytes_two_gemm, "flops": flops_step}}


def cpu_baseline(cfg, L, united, threshold, n_sample):
    """The oracle as it stands, on the host cores: routing on every token, the layer equation on a
    bounded sample of tokens (sized for roughly 10-30 s), throughput extrapolated linearly."""
    import numpy as np
    from oracle import oracle as O

    f32 = lambda t: None if t is None else t.float().cpu().numpy()
    x, gw, gb = f32(L.x), f32(L.gate_w), f32(L.gate_b)
    t0 = time.perf_counter()
    r = O.route(x, gw, gb, cfg.K, cfg.way, threshold, False, cfg.score_fn, cfg.n_shared)
    t_route = time.perf_counter() - t0
    per_token_flops = 6.0 * cfg.d * (cfg.F * cfg.K + cfg.F_s * cfg.n_shared)
    whole = cfg.m * cfg.d * cfg.F <= 6e8        # all experts fit as float arrays: tokens run in parallel
    cores = O.num_threads()
    if whole:
        if n_sample is None:
            n_sample = int(max(8, min(cfg.T, 1e12 / per_token_flops)))     # about 1 TFLOP of plain loops
        tokens = np.linspace(0, cfg.T - 1, n_sample).astype(np.int32)
        how = f"{n_sample} evenly spaced tokens"
        ex, un, sh = tuple(f32(a) for a in L.experts), tuple(f32(a) for a in united), \
            None if L.shared is None else tuple(f32(a) for a in L.shared)
        t0 = time.perf_counter()
        O.forward_tokens(x, r.topk_idx, r.topk_w, r.expert_unit, cfg.way, ex, un, sh, tokens=tokens)
        t_ffn = time.perf_counter() - t0
    else:
        # Too large to hold as float arrays: a stratified sample (a token from every execution unit that holds
        # rows, then evenly spaced ones, at least 256, about 0.2 TFLOP of plain loops), one FFN at a time with
        # its sampled rows spread over the cores; the weights are fetched before the clock starts.
        if n_sample is None:
            n_sample = int(max(256, min(cfg.T, 2e11 / per_token_flops)))
        rows = r.rows
        chosen = [int(rows.row_token[int(rows.unit_off[u]) + int(rows.unit_cnt[u]) // 2])
                  for u in np.nonzero(rows.unit_cnt > 0)[0]]
        chosen = list(dict.fromkeys(chosen))[:n_sample]
        have = set(chosen)
        for t in np.linspace(0, cfg.T - 1, n_sample).astype(int):
            if len(chosen) >= n_sample:
                break
            if int(t) not in have:
                chosen.append(int(t))
                have.add(int(t))
        tokens = np.array(sorted(chosen), np.int64)
        n_sample = len(tokens)
        how = f"{n_sample} tokens (one from every active execution unit, the rest evenly spaced)"
        src = {"expert": L.experts, "united": united, "shared": L.shared}
        need = set(("shared", s) for s in range(cfg.n_shared))
        for t in tokens:
            for j in range(cfg.K):
                u = int(r.expert_unit[r.topk_idx[t, j]])
                if u >= 0:
                    need.add(("expert", u) if u < cfg.m else ("united", u - cfg.m))
        t_fetch, t_ffn, out_rows = 0.0, 0.0, None
        # the helper asks for each FFN once: time the fetches apart from the arithmetic
        def get(kind, i):
            nonlocal t_fetch
            tf = time.perf_counter()
            w = tuple(f32(a[i]) for a in src[kind])
            t_fetch += time.perf_counter() - tf
            return w
        t0 = time.perf_counter()
        O.forward_tokens_lazy(x[tokens], r.topk_idx[tokens], r.topk_w[tokens], r.expert_unit, cfg.m, get, cfg.n_shared)
        t_ffn = time.perf_counter() - t0 - t_fetch
        log(f"  oracle: {len(need)} FFNs fetched from the GPU in {t_fetch:.2f} s (not counted)")
    per_token = t_route / cfg.T + t_ffn / n_sample
    log(f"  oracle: routing {t_route:.2f} s for {cfg.T} tokens, layer equation {t_ffn:.2f} s for {n_sample} tokens, "
        f"{cores} threads")
    return {"value": 1.0 / per_token, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"routing on all {cfg.T} tokens ({t_route:.2f} s) + layer equation on {how} "
                      f"({t_ffn:.2f} s), extrapolated linearly"}


if __name__ == "__main__":
    main()
