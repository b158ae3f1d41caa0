"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import oracle as O

NEAR_TIE = 1e-6        # margin below which a TopK decision may legitimately differ (fp32 summation order)
OUT_TOL = 2e-2         # max relative error of layer outputs: bf16 compute, fp32 accumulate, vs the oracle


def npf(t):
    """torch tensor (any device, bf16/fp32/int) -> numpy (bf16 widened to float32)."""
    if t is None:
        return None
    if isinstance(t, (tuple, list)):
        return tuple(npf(a) for a in t)
    t = t.detach()
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.cpu().numpy()


def rel_err(got, ref):
    """max_{t,c} |got-ref| / max(|ref_tc|, rms(ref_t)): relative error that does not blow up on
    the entries of a row that happen to be near zero."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    den = np.maximum(np.abs(ref), np.maximum(rms, 1e-30))
    return float((np.abs(got - ref) / den).max())


def oracle_route(layer, cfg, threshold, full=False):
    x, gw = npf(layer.x), npf(layer.gate_w)
    gb = npf(layer.gate_b)
    return O.route(x, gw, gb, cfg.K, cfg.way, threshold, full, cfg.score_fn, cfg.n_shared)


def check_topk(gpu_idx, gpu_w, ref, K):
    """TopK parity.  Tokens whose fp64 margin is >= NEAR_TIE must match exactly.  On the others the
    GPU may have taken either neighbour: its choice must be valid (every chosen expert within
    NEAR_TIE of qualifying, order descending up to NEAR_TIE).  Returns the flagged token ids at
    which the GPU differs."""
    flagged = ref.margin < NEAR_TIE
    same = (gpu_idx == ref.topk_idx).all(axis=1)
    assert same[~flagged].all(), f"TopK differs on {int((~same & ~flagged).sum())} unflagged tokens"
    diff = np.nonzero(~same)[0]
    for t in diff:
        s = ref.s64[t]
        kth = np.sort(s)[::-1][K - 1]
        chosen = s[gpu_idx[t]]
        assert len(set(gpu_idx[t].tolist())) == K
        assert (chosen >= kth - NEAR_TIE).all()
        assert (np.diff(chosen) <= NEAR_TIE).all()
    ok = same
    assert np.allclose(gpu_w[ok], ref.topk_w[ok], rtol=2e-5, atol=1e-7)
    return diff


def downstream_reference(gpu_idx, gpu_w, ref, diff, m, way, n_shared, threshold, full):
    """Counts, Algorithm 1 and row lists from the oracle, fed with the oracle's TopK except on the
    flagged tokens where the GPU legitimately chose the other neighbour."""
    idx, w = ref.topk_idx.copy(), ref.topk_w.copy()
    idx[diff], w[diff] = gpu_idx[diff], gpu_w[diff]
    cnt = O.expert_counts(idx, m)
    unit, in_s1 = O.brownout_decide(cnt, way, threshold, full)
    rows = O.build_rows(idx, w, m, way, n_shared, unit)
    return idx, w, cnt, unit, in_s1, rows


def check_route(R, ref, cfg, threshold, full):
    """Full routing parity of a binding.RouteOut against the oracle's Route.  Integer artefacts
    bit-exact; weights to fp32 rounding.  Returns (idx, w, unit) the downstream reference used."""
    m, K = cfg.m, cfg.K
    g_idx, g_w = npf(R.topk_idx), npf(R.topk_w)
    diff = check_topk(g_idx, g_w, ref, K)
    idx, w, cnt, unit, in_s1, rows = downstream_reference(g_idx, g_w, ref, diff, m, cfg.way, cfg.n_shared,
                                                          threshold, full)
    # feed the GPU's own weights into the row reference so that row_weight compares bit-exactly
    rows_g = O.build_rows(idx, g_w, m, cfg.way, cfg.n_shared, unit)
    assert (npf(R.expert_cnt) == cnt).all()
    assert (npf(R.expert_unit) == unit).all()
    assert (npf(R.expert_in_s1) == in_s1).all()
    assert (npf(R.unit_cnt) == rows.unit_cnt).all()
    assert (npf(R.unit_off) == rows.unit_off).all()
    n = rows.n_rows
    assert int(npf(R.n_rows)[0]) == n
    assert (npf(R.row_token)[:n] == rows.row_token).all()
    assert (npf(R.token_rows) == rows.token_rows).all()
    assert (npf(R.row_weight)[:n] == rows_g.row_weight).all()
    assert np.allclose(npf(R.row_weight)[:n], rows.row_weight, rtol=2e-5, atol=1e-7)
    return idx, w, unit
