"""Pins for the oracle's FFN, layer equation and united-expert construction.

The references used here are library routines (torch fp64 matmul / silu) and an
independently written plain top-K MoE, plus the special cases the method
reduces to: no brownout == ordinary MoE, one expert == dense SwiGLU FFN,
united == copy of identical members, threshold 0 under full brownout == only
the shared experts, linearity in the down projection.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O


def _layer(T=24, d=32, F=40, m=6, K=2, seed=0, n_shared=0, Fs=24):
    rng = np.random.default_rng(seed)
    f = lambda *s: (rng.standard_normal(s) / np.sqrt(s[-1])).astype(np.float32)
    L = dict(x=rng.standard_normal((T, d)).astype(np.float32), gw=f(m, d),
             experts=(f(m, F, d), f(m, F, d), f(m, d, F)))
    L["shared"] = (f(n_shared, Fs, d), f(n_shared, Fs, d), f(n_shared, d, Fs)) if n_shared else None
    return L


def _dense_swiglu(x, w1, w3, w2):
    xt = torch.from_numpy(x).double()
    a = xt @ torch.from_numpy(w1).double().T
    b = xt @ torch.from_numpy(w3).double().T
    return ((torch.nn.functional.silu(a) * b) @ torch.from_numpy(w2).double().T).numpy()


def test_ffn_is_dense_swiglu():
    L = _layer()
    w1, w3, w2 = (a[2] for a in L["experts"])
    y = O.ffn(L["x"], w1, w3, w2)
    assert np.allclose(y, _dense_swiglu(L["x"], w1, w3, w2), rtol=1e-10, atol=1e-12)
    # swapping the gate and up projections must be visible
    assert not np.allclose(y, _dense_swiglu(L["x"], w3, w1, w2), atol=1e-3)


def test_one_expert_top1_equals_dense_ffn():
    L = _layer(m=1, K=1)
    r = O.route(L["x"], L["gw"], None, K=1, way=1, threshold=1.0)
    assert np.allclose(r.topk_w, 1.0)
    out = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 1, L["experts"])
    ref = _dense_swiglu(L["x"], *(a[0] for a in L["experts"]))
    assert np.allclose(out, ref, rtol=1e-6, atol=1e-6)


def _plain_topk_moe(x, gw, experts, K, shared=None, residual=False):
    """An ordinary top-K MoE layer, written token by token with numpy, no routing tables."""
    T, d = x.shape
    w1, w3, w2 = (a.astype(np.float64) for a in experts)
    out = np.zeros((T, d))
    for t in range(T):
        xt = x[t].astype(np.float64)
        s = (gw.astype(np.float64) @ xt).astype(np.float32)
        top = sorted(range(len(s)), key=lambda i: (-s[i], i))[:K]
        e = np.exp(s[top].astype(np.float64) - float(s[top[0]]))
        g = e / e.sum()
        acc = xt.copy() if residual else np.zeros(d)
        if shared is not None:
            for si in range(shared[0].shape[0]):
                a, b = shared[0][si].astype(np.float64) @ xt, shared[1][si].astype(np.float64) @ xt
                acc += shared[2][si].astype(np.float64) @ (a / (1 + np.exp(-a)) * b)
        for gi, i in zip(g, top):
            a, b = w1[i] @ xt, w3[i] @ xt
            acc += gi * (w2[i] @ (a / (1 + np.exp(-a)) * b))
        out[t] = acc
    return out


@pytest.mark.parametrize("residual", [False, True])
def test_zero_brownout_equals_plain_topk_moe(residual):
    L = _layer(n_shared=1)
    r = O.route(L["x"], L["gw"], None, K=2, way=3, threshold=1.0, n_shared=1)
    assert (r.expert_unit == np.arange(6)).all()
    out = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 3, L["experts"], None, L["shared"],
                           add_residual=residual)
    ref = _plain_topk_moe(L["x"], L["gw"], L["experts"], 2, L["shared"], residual)
    assert np.allclose(out, ref, rtol=1e-5, atol=1e-6)


def test_rows_then_ffn_then_combine_equals_the_equation():
    """Permute rows by unit, run each unit's FFN once per row, weighted un-permute: same h_t."""
    L = _layer(T=40, m=8, K=3, seed=2, n_shared=1)
    rng = np.random.default_rng(11)
    way = 4
    united = tuple((rng.standard_normal((2,) + a.shape[1:]) / 6).astype(np.float32) for a in L["experts"])
    for thr, full in [(0.4, False), (0.0, False), (0.4, True)]:
        r = O.route(L["x"], L["gw"], None, K=3, way=way, threshold=thr, use_full_brownout=full, n_shared=1)
        direct = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, way, L["experts"], united,
                                  L["shared"])
        R = r.rows
        out = np.zeros_like(direct, dtype=np.float64)
        m, G = 8, 2
        for u in range(m + G + 1):
            lo, hi = R.unit_off[u], R.unit_off[u + 1]
            if hi == lo:
                continue
            src = L["experts"] if u < m else (united if u < m + G else L["shared"])
            k = u if u < m else (u - m if u < m + G else u - m - G)
            y = O.ffn(L["x"][R.row_token[lo:hi]], src[0][k], src[1][k], src[2][k])
            np.add.at(out, R.row_token[lo:hi], R.row_weight[lo:hi, None].astype(np.float64) * y)
        assert np.allclose(out, direct, rtol=1e-5, atol=1e-6)


def test_identical_members_make_brownout_invisible():
    """If every expert of a group is the same FFN and the united expert is that FFN too,
    delegating tokens to the united expert cannot change the output."""
    L = _layer(m=6, K=2, seed=5)
    way = 3
    ex = tuple(np.repeat(a[::way], way, axis=0) for a in L["experts"])      # members of a group identical
    un = tuple(np.ascontiguousarray(a[::way]) for a in L["experts"])
    base = None
    for thr in (1.0, 0.7, 0.3, 0.0):
        r = O.route(L["x"], L["gw"], None, K=2, way=way, threshold=thr)
        out = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, way, ex, un)
        base = out if base is None else base
        assert np.allclose(out, base, rtol=1e-5, atol=1e-6)
    assert (r.expert_unit >= 6).any()


def test_full_brownout_threshold_zero_leaves_only_shared_and_residual():
    L = _layer(n_shared=2)
    r = O.route(L["x"], L["gw"], None, K=2, way=2, threshold=0.0, use_full_brownout=True, n_shared=2)
    assert (r.expert_unit[r.expert_cnt > 0] == -1).all()
    out = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 2, L["experts"], None, L["shared"],
                           add_residual=True)
    ref = L["x"].astype(np.float64).copy()
    for s in range(2):
        ref += _dense_swiglu(L["x"], *(a[s] for a in L["shared"]))
    assert np.allclose(out, ref, rtol=1e-5, atol=1e-6)


def test_dropped_experts_are_not_renormalised():
    L = _layer(m=4, K=2, seed=8)
    r = O.route(L["x"], L["gw"], None, K=2, way=2, threshold=0.5, use_full_brownout=True)
    out = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 2, L["experts"])
    ref = np.zeros_like(out, dtype=np.float64)
    for t in range(out.shape[0]):
        for j in range(2):
            i = r.topk_idx[t, j]
            if r.expert_unit[i] >= 0:
                ref[t] += float(r.topk_w[t, j]) * _dense_swiglu(L["x"][t:t + 1], *(a[i] for a in L["experts"]))[0]
    assert (r.expert_unit == -1).any()
    assert np.allclose(out, ref, rtol=1e-5, atol=1e-6)


def test_linear_in_down_projection():
    L = _layer(seed=3)
    r = O.route(L["x"], L["gw"], None, K=2, way=2, threshold=1.0)
    a = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 2, L["experts"])
    ex = (L["experts"][0], L["experts"][1], L["experts"][2] * np.float32(-2.0))
    b = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 2, ex)
    assert np.allclose(b, -2.0 * a, rtol=1e-5, atol=1e-6)


def test_token_subset():
    L = _layer()
    r = O.route(L["x"], L["gw"], None, K=2, way=2, threshold=1.0)
    full = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 2, L["experts"])
    sub = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, r.expert_unit, 2, L["experts"], tokens=[5, 0, 17])
    assert (sub == full[[5, 0, 17]]).all()


# --------------------------------------------------------------------- united experts
def test_united_mean_special_cases():
    rng = np.random.default_rng(0)
    w = rng.standard_normal((7, 5, 3)).astype(np.float32)
    assert (O.united_mean(w, 1) == w.astype(np.float64)).all()            # way 1: the expert itself
    u = O.united_mean(w, 3)                                               # groups {0,1,2} {3,4,5} {6}
    assert u.shape == (3, 5, 3)
    assert np.allclose(u[0], w[:3].astype(np.float64).mean(0), atol=1e-15)
    assert np.allclose(u[1], w[3:6].astype(np.float64).mean(0), atol=1e-15)
    assert (u[2] == w[6]).all()                                           # ragged last group: its one member
    same = np.repeat(w[:1], 4, axis=0)
    assert (O.united_mean(same, 4)[0] == w[0]).all()


def test_united_loss_decomposition():
    """(1/k) sum_i |H_u - H_i|^2 = |H_u - mean H|^2 + (1/k) sum_i |H_i - mean H|^2, so the loss
    is never below the teachers' spread, and it is 0 when way = 1 and the student is the teacher."""
    L = _layer(T=16, m=5, seed=6)
    way = 2
    calib = L["x"]
    un = tuple(O.united_mean(a, way).astype(np.float32) for a in L["experts"])
    loss = O.united_loss(calib, way, L["experts"], un)
    assert loss.shape == (3,)
    for g in range(3):
        mem = list(range(g * way, min(5, g * way + way)))
        H = np.stack([_dense_swiglu(calib, *(a[i] for a in L["experts"])) for i in mem])
        Hu = _dense_swiglu(calib, *(a[g] for a in un))
        mean = H.mean(0)
        want = ((Hu - mean) ** 2).sum() / 16 + ((H - mean) ** 2).sum() / len(mem) / 16
        assert np.isclose(loss[g], want, rtol=1e-9)
        assert loss[g] >= ((H - mean) ** 2).sum() / len(mem) / 16 - 1e-12
    assert abs(loss[2]) < 1e-20                                           # single-member group: student == teacher
    ident = O.united_loss(calib, 1, L["experts"], L["experts"])
    assert (ident == 0).all()


def _explicit_layer(x, idx, w, unit, m, experts, united, shared, add_residual):
    """The layer equation written out with torch fp64 matmuls, token by token (independent of the C file)."""
    def f(xr, W, i):
        return _dense_swiglu(xr[None, :], W[0][i], W[1][i], W[2][i])[0]
    out = np.zeros(x.shape, np.float64)
    for t in range(x.shape[0]):
        if add_residual:
            out[t] += x[t]
        for s in range(0 if shared is None else shared[0].shape[0]):
            out[t] += f(x[t], shared, s)
        for j in range(idx.shape[1]):
            u = unit[idx[t, j]]
            if u < 0:
                continue
            out[t] += float(w[t, j]) * (f(x[t], experts, u) if u < m else f(x[t], united, u - m))
    return out


@pytest.mark.parametrize("full,residual", [(False, False), (False, True), (True, False)])
def test_forward_tokens_lazy_equals_forward_tokens(full, residual):
    """The helper that evaluates the layer equation for sampled tokens of layers too large to hold as float
    arrays (weights fetched per FFN) against the plain evaluation, on a layer where every kind of term
    occurs: experts served by themselves, several TopK entries of a token delegated to the SAME united
    expert, dropped experts (full brownout), two shared experts, the residual."""
    m, K, way, ns = 8, 4, 4, 2
    L = _layer(T=40, d=32, F=40, m=m, K=K, seed=11, n_shared=ns, Fs=24)
    rng = np.random.default_rng(5)
    un = tuple((rng.standard_normal(a[:2].shape) / 6).astype(np.float32) for a in L["experts"])
    r = O.route(L["x"], L["gw"], None, K, way, 0.35, full, 0, ns)
    unit = r.expert_unit
    if full:
        assert (unit < 0).any()
    else:
        assert (unit >= m).any() and (unit < m).any()
        # some token has two of its TopK experts delegated to one united expert
        assert any(len(set(u for u in unit[r.topk_idx[t]] if u >= m)) < sum(unit[r.topk_idx[t]] >= m)
                   for t in range(40))
    want = O.forward_tokens(L["x"], r.topk_idx, r.topk_w, unit, way, L["experts"], un, L["shared"],
                            add_residual=residual)
    src = {"expert": L["experts"], "united": un, "shared": L["shared"]}
    calls = []

    def get(kind, i):
        calls.append((kind, i))
        return tuple(a[i] for a in src[kind])
    toks = np.array([0, 3, 4, 17, 18, 39, 25], np.int64)
    got = O.forward_tokens_lazy(L["x"][toks], r.topk_idx[toks], r.topk_w[toks], unit, m, get, ns, residual)
    assert np.allclose(got, want[toks], rtol=1e-6, atol=1e-7)            # forward_tokens returns float
    exact = _explicit_layer(L["x"], r.topk_idx, r.topk_w, unit, m, L["experts"], un, L["shared"], residual)
    assert np.allclose(got, exact[toks], rtol=1e-9, atol=1e-11)
    assert len(calls) == len(set(calls))                                  # one fetch per distinct FFN
    # a wrong unit -> weights lookup must be visible: shift the united index by one
    def get_wrong(kind, i):
        return tuple(a[(i + 1) % a.shape[0]] if kind == "united" else a[i] for a in src[kind])
    if not full:
        bad = O.forward_tokens_lazy(L["x"][toks], r.topk_idx[toks], r.topk_w[toks], unit, m, get_wrong, ns, residual)
        assert not np.allclose(bad, exact[toks], rtol=1e-3, atol=1e-4)
