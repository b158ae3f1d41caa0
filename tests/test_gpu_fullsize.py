"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Routing is checked on ALL tokens against the oracle run from x and the gate weights (TopK with the
near-tie rule of tests/_util.check_topk, everything downstream bit-exact).  The oracle cannot evaluate
the FFNs of these layers whole in reasonable time, so layer outputs are compared on a stratified sample
of tokens the oracle computes one by one: for every execution unit that holds rows, the token of a row in
its first GEMM tile and of a row in its last (ragged) tile, then evenly spaced tokens up to the stated
number; the decode-sized batches and the T = 1024 batches are compared in full.
Inputs are drawn on the GPU by torch's seeded generator (never by the library under test); united
experts are random tensors, the forward pass accepting any.
"""
import numpy as np
import pytest
import torch

import paper_2507_17133_amd as P
from oracle import oracle as O
from paper_2507_17133_amd import workloads as WL
from tests._util import OUT_TOL, check_route, npf, rel_err

pytestmark = pytest.mark.gpu

ALL = -1
# (workload, overrides, brownout fraction f = 1 - threshold, tokens whose output is compared)
CASES = [
    ("mixtral_prefill", {}, 0.3, 256), ("mixtral_prefill", {}, 0.0, 256),
    ("mixtral_prefill", {"way": 4}, 0.3, 256),                       # two united experts of four
    ("mixtral_decode", {}, 0.0, ALL), ("mixtral_decode", {}, 0.25, ALL), ("mixtral_decode", {}, 0.5, ALL),
    ("mixtral_decode", {}, 0.75, ALL), ("mixtral_decode", {}, 1.0, ALL),
    ("qwen3_30b_a3b", {}, 0.5, 256), ("qwen3_30b_a3b", {}, 0.0, 320),
    # a batch of 1024 tokens over 128 skewed experts: many units with fewer than 16 rows
    ("qwen3_30b_a3b", {"T": 1024}, 0.0, ALL), ("qwen3_30b_a3b", {"T": 1024}, 0.5, ALL),
    # 4096 tokens over 128 experts: the LDS-staged gate with 16-token blocks on every CU
    ("qwen3_30b_a3b", {"T": 4096}, 0.25, 256),
    # 16 384 tokens over 8 experts: the K-splitting gate for few experts, 256 routing segments
    ("mixtral_prefill", {"T": 16384}, 0.3, 256),
    ("deepseek_v3", {}, 0.4, 256), ("deepseek_v3", {}, 0.0, 560),
    # the paper's 60-expert layer shape at the three (way, threshold) settings of its throughput experiment
    # (Results): (8, 0.4), (4, 0.2), (2, 0), and with every multi-member group on its united expert
    ("qwen15_moe_a27b", {}, 0.6, 256), ("qwen15_moe_a27b", {"way": 4}, 0.8, 256),
    ("qwen15_moe_a27b", {"way": 2}, 1.0, 256), ("qwen15_moe_a27b", {}, 1.0, 256),
]


def _case_id(c):
    extra = "".join(f"-{k}{v}" for k, v in c[1].items())
    return f"{c[0]}{extra}-f{c[2]}"


def _pick_tokens(rows, n, T):
    """Tokens of a first-tile row and of a last-tile row of every unit that holds rows, then evenly
    spaced tokens until there are n."""
    chosen = []
    for u in np.nonzero(rows.unit_cnt > 0)[0]:
        o, c = int(rows.unit_off[u]), int(rows.unit_cnt[u])
        chosen.append(int(rows.row_token[o + min(c - 1, 5)]))
        chosen.append(int(rows.row_token[o + c - 1]))
    chosen = list(dict.fromkeys(chosen))
    have = set(chosen)
    for t in np.linspace(0, T - 1, max(n, 2)).astype(int):
        if len(chosen) >= n:
            break
        if int(t) not in have:
            chosen.append(int(t))
            have.add(int(t))
    return np.array(sorted(chosen), np.int64)


@pytest.mark.parametrize("name,over,frac,n_tok", CASES, ids=[_case_id(c) for c in CASES])
def test_fullsize(name, over, frac, n_tok):
    torch.cuda.set_device(0)
    cfg = WL.CONFIGS[name].with_(**over)
    thr = 1.0 - frac
    c = P.config_of(cfg)
    L = WL.make_layer(cfg, 0, "cuda")
    united = WL.make_random_united(cfg, 0, "cuda")
    ws = P.alloc_workspace(c, cfg.T)
    R = P.moe_route(c, L.x, L.gate_w, L.gate_b, thr, workspace=ws)
    # the layer as bench.py runs it: packed gate, routing inside moe_forward, one workspace
    cp = P.with_packed_gate(c)
    out = P.moe_forward(cp, L.x, P.pack_gate(c, L.gate_w), L.gate_b, L.experts, united, L.shared, thr,
                        workspace=P.alloc_workspace(cp, cfg.T))
    torch.cuda.synchronize()
    T, m = cfg.T, cfg.m

    # ---- routing on all tokens: TopK (near ties: either neighbour, but a valid one), then counts,
    # Algorithm 1 and the row lists bit-exact against the oracle fed with the agreed TopK
    x_cpu = npf(L.x)
    ref = O.route(x_cpu, npf(L.gate_w), npf(L.gate_b), cfg.K, cfg.way, thr, False, cfg.score_fn, cfg.n_shared)
    idx, w, unit = check_route(R, ref, cfg, thr, False)
    assert np.allclose(npf(R.topk_w).astype(np.float64).sum(1), 1.0, atol=1e-5)
    if frac == 0.0:
        assert (unit == np.arange(m)).all()
    rows = O.build_rows(idx, w, m, cfg.way, cfg.n_shared, unit)
    if frac == 1.0 and cfg.way >= m:
        assert rows.n_rows == T + T * cfg.n_shared

    # ---- layer output
    toks = np.arange(T, dtype=np.int64) if n_tok == ALL else _pick_tokens(rows, n_tok, T)
    src = {"expert": L.experts, "united": united, "shared": L.shared}
    want = O.forward_tokens_lazy(x_cpu[toks], idx[toks], w[toks], unit, m,
                                 lambda kind, i: tuple(npf(a[i]) for a in src[kind]), cfg.n_shared)
    got_all = npf(out)
    assert np.isfinite(got_all).all()
    e = rel_err(got_all[toks], want)
    assert e <= OUT_TOL, f"{_case_id((name, over, frac))}: max relative error {e} over {len(toks)} tokens"
