"""Pins for the oracle's gating: affinities, TopK, renormalised weights, counts."""
import numpy as np
import pytest
import scipy.special

from oracle import oracle as O


def _inputs(T=37, d=48, m=10, seed=0, bias=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(np.float32)
    gw = (rng.standard_normal((m, d)) / np.sqrt(d)).astype(np.float32)
    b = rng.standard_normal(m).astype(np.float32) if bias else None
    return x, gw, b


def test_logits_match_library_matmul():
    x, gw, b = _inputs()
    s64, s32 = O.gate_logits(x, gw, b)
    ref = x.astype(np.float64) @ gw.astype(np.float64).T + b.astype(np.float64)
    assert np.allclose(s64, ref, rtol=0, atol=1e-12)
    assert (s32 == ref.astype(np.float32)).mean() > 0.99    # same value up to the last double bit
    assert np.allclose(s32, ref, atol=1e-6)
    # a transposed gate matrix must NOT pass
    s64_t, _ = O.gate_logits(x[:, :10], np.ascontiguousarray(gw[:, :10]), None)
    assert np.allclose(s64_t, x[:, :10].astype(np.float64) @ gw[:, :10].astype(np.float64).T, atol=1e-12)


@pytest.mark.parametrize("K", [1, 2, 3, 10])
@pytest.mark.parametrize("score_fn", [0, 1])
def test_topk_against_full_sort(K, score_fn):
    x, gw, b = _inputs(T=200, m=10, seed=K)
    s64, s32 = O.gate_logits(x, gw, b)
    idx, w, margin = O.topk(s64, s32, K, score_fn)
    order = np.argsort(-s32, axis=1, kind="stable")[:, :K]         # descending score, ties: lower index
    assert (idx == order).all()
    sel = np.take_along_axis(s32.astype(np.float64), idx.astype(np.int64), axis=1)
    if score_fn == 0:
        ref = scipy.special.softmax(sel, axis=1)
    else:
        sg = scipy.special.expit(sel)
        ref = sg / sg.sum(1, keepdims=True)
    assert np.allclose(w, ref, rtol=1e-6, atol=1e-7)
    assert np.allclose(w.astype(np.float64).sum(1), 1.0, atol=1e-6)
    assert (np.diff(w, axis=1) <= 1e-7).all()                      # weights follow the score order
    assert (margin >= -1e-6).all()


def test_k_equals_m_is_the_full_softmax():
    x, gw, b = _inputs(T=50, m=6, seed=9, bias=False)
    s64, s32 = O.gate_logits(x, gw, b)
    idx, w, _ = O.topk(s64, s32, 6, 0)
    full = scipy.special.softmax(s32.astype(np.float64), axis=1)
    got = np.zeros_like(full)
    np.put_along_axis(got, idx.astype(np.int64), w.astype(np.float64), axis=1)
    assert np.allclose(got, full, atol=1e-7)


def test_ties_take_the_lower_index_and_margin_is_zero():
    s = np.array([[0.5, 2.0, 2.0, -1.0, 2.0]], np.float32)
    idx, w, margin = O.topk(s.astype(np.float64), s, 2, 0)
    assert idx.tolist() == [[1, 2]]
    assert margin[0] == 0.0
    assert np.allclose(w, 0.5)
    # a well separated token reports its true gap (K-th winner minus best loser is the smallest here)
    s = np.array([[3.0, 1.0, 0.0, -2.0]], np.float32)
    idx, w, margin = O.topk(s.astype(np.float64), s, 2, 0)
    assert idx.tolist() == [[0, 1]] and margin[0] == 1.0


def test_counts():
    x, gw, b = _inputs(T=300, m=16, seed=4)
    s64, s32 = O.gate_logits(x, gw, b)
    idx, _, _ = O.topk(s64, s32, 4, 0)
    cnt = O.expert_counts(idx, 16)
    assert cnt.sum() == 300 * 4
    assert (cnt == np.bincount(idx.ravel(), minlength=16)).all()
    assert all(len(set(r)) == 4 for r in idx.tolist())
