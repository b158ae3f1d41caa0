"""Pins for the oracle's Algorithm 1 (brownout decision) and row bookkeeping.

Nothing here re-types the oracle's loop: the pins are the paper's printed worked
examples, the limiting cases the paper states (threshold 1 = zero-brownout,
threshold 0 = everything delegated), a brute-force set definition on tiny
inputs, and order/monotonicity properties.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_worked_examples.txt")


def _parse_golden():
    cases = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, counts, thr, way, full, s1, units, acc = [p.strip() for p in line.split(";")]
            cases.append(dict(name=name, counts=[int(v) for v in counts.split()], thr=float(thr), way=int(way),
                              full=bool(int(full)), s1=[int(v) for v in s1.split()], units=units.split(),
                              accesses=int(acc)))
    return cases


@pytest.mark.parametrize("case", _parse_golden(), ids=lambda c: c["name"])
def test_paper_worked_examples(case):
    cnt = np.array(case["counts"], np.int32)
    m = len(cnt)
    unit, in_s1 = O.brownout_decide(cnt, case["way"], case["thr"], case["full"])
    assert sorted(np.nonzero(in_s1)[0].tolist()) == case["s1"]
    want = []
    for i, tag in enumerate(case["units"]):
        want.append(i if tag[0] == "E" else (-1 if tag == "X" else m + int(tag[1:])))
    assert unit.tolist() == want
    used = {u for u, c in zip(unit.tolist(), cnt.tolist()) if u >= 0 and c > 0}
    assert len(used) == case["accesses"]


def test_paper_example_token_totals():
    """Partial-brownout example: UE0 gets 3 tokens, UE1 gets 5; full-brownout keeps 12 of 20."""
    cnt = np.array([2, 4, 1, 5, 2, 1, 2, 3], np.int32)
    unit, in_s1 = O.brownout_decide(cnt, 4, 0.6, False)
    assert cnt[unit == 8].sum() == 3 and cnt[unit == 9].sum() == 5
    unit, in_s1 = O.brownout_decide(cnt, 4, 0.6, True)
    assert cnt[unit >= 0].sum() == 12 and (unit >= 0).sum() == 3


@pytest.mark.parametrize("way", [1, 2, 3, 8])
@pytest.mark.parametrize("full", [False, True])
def test_threshold_one_is_zero_brownout(way, full):
    rng = np.random.default_rng(1)
    for _ in range(20):
        cnt = rng.integers(0, 50, size=8).astype(np.int32)
        unit, in_s1 = O.brownout_decide(cnt, way, 1.0, full)
        assert unit.tolist() == list(range(8))
        assert (in_s1[cnt > 0] == 1).all()


def test_threshold_zero_empties_s1():
    cnt = np.array([5, 0, 3, 3, 1, 0, 7, 2], np.int32)
    unit, in_s1 = O.brownout_decide(cnt, 2, 0.0, False)
    assert in_s1.sum() == 0
    # groups {0,1} {2,3} {4,5} {6,7}: group 0 and 2 have one member with tokens -> served by itself
    assert unit.tolist() == [0, 1, 8 + 1, 8 + 1, 4, 5, 8 + 3, 8 + 3]
    unit, in_s1 = O.brownout_decide(cnt, 2, 0.0, True)
    assert unit.tolist() == [-1, 1, -1, -1, -1, 5, -1, -1]


def test_equal_counts_lower_id_first():
    cnt = np.array([3, 3, 3, 3], np.int32)
    # 12 tokens, threshold 0.5 -> 6 tokens needed -> two experts -> ids 0 and 1
    unit, in_s1 = O.brownout_decide(cnt, 4, 0.5, False)
    assert in_s1.tolist() == [1, 1, 0, 0]
    assert unit.tolist() == [0, 1, 4, 4]


def _brute_s1(cnt, thr):
    """S1 by definition: the fewest most-loaded experts whose tokens total at least S*threshold."""
    m = len(cnt)
    order = sorted(range(m), key=lambda i: (-cnt[i], i))
    S = sum(cnt)
    need = float(S) * float(thr)
    for n in range(m + 1):
        if sum(cnt[i] for i in order[:n]) >= need:
            return set(order[:n])
    return set(order)


def _brute_units(cnt, in_s1, way, full):
    m = len(cnt)
    unit = list(range(m))
    G = -(-m // way)
    for g in range(G):
        mem = [i for i in range(g * way, min(m, g * way + way)) if i not in in_s1 and cnt[i] > 0]
        for i in mem:
            unit[i] = -1 if full else (m + g if len(mem) >= 2 else i)
    return unit


def test_brute_force_small_m():
    thresholds = [0.0, 0.1, 0.25, 1.0 / 3.0, 0.5, 0.6, 0.75, 0.9, 1.0]
    n = 0
    for m in (1, 2, 3, 4, 5):
        for cnt in itertools.product(range(4), repeat=m):
            for thr in thresholds:
                for way in (1, 2, 3, m):
                    for full in (False, True):
                        unit, in_s1 = O.brownout_decide(np.array(cnt, np.int32), way, thr, full)
                        got_s1 = {i for i in range(m) if in_s1[i] and cnt[i] > 0}
                        want_s1 = {i for i in _brute_s1(list(cnt), thr) if cnt[i] > 0}
                        assert got_s1 == want_s1, (cnt, thr)
                        s1_all = {i for i in range(m) if in_s1[i]}
                        assert unit.tolist() == _brute_units(list(cnt), s1_all, way, full), (cnt, thr, way, full)
                        n += 1
    assert n > 10000


def test_minimal_and_monotone():
    rng = np.random.default_rng(7)
    for _ in range(200):
        m = int(rng.integers(2, 64))
        cnt = rng.zipf(1.5, size=m).clip(max=500).astype(np.int32) * (rng.random(m) > 0.2)
        cnt = cnt.astype(np.int32)
        S = int(cnt.sum())
        prev = None
        for thr in np.linspace(0, 1, 11):
            thr = float(thr)
            _, in_s1 = O.brownout_decide(cnt, 4, thr, False)
            s1 = set(np.nonzero(in_s1 & (cnt > 0))[0].tolist())
            covered = int(cnt[list(s1)].sum()) if s1 else 0
            assert covered >= S * thr - 1e-9
            if s1:
                smallest = min(cnt[list(s1)])
                assert covered - smallest < S * thr     # dropping the least-loaded member breaks it
            if prev is not None:
                assert prev <= s1
            prev = s1


def test_rows_bookkeeping_and_dedup():
    rng = np.random.default_rng(3)
    T, K, m, way = 97, 4, 12, 4
    idx = np.stack([rng.permutation(m)[:K] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, K)).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    cnt = O.expert_counts(idx, m)
    assert cnt.sum() == T * K
    for thr, full in [(1.0, False), (0.5, False), (0.0, False), (0.5, True)]:
        unit, _ = O.brownout_decide(cnt, way, thr, full)
        rows = O.build_rows(idx, w, m, way, 1, unit)
        G = 3
        assert rows.unit_off[0] == 0 and (np.diff(rows.unit_off) == rows.unit_cnt).all()
        assert rows.n_rows == rows.unit_off[-1]
        assert rows.unit_cnt[m + G] == T                      # the shared unit takes every token
        # rows ascend in token inside every unit, and a token appears at most once per unit
        for u in range(m + G + 1):
            seg = rows.row_token[rows.unit_off[u]:rows.unit_off[u + 1]]
            assert (np.diff(seg) > 0).all()
        # per token: the weights of its rows add up to the g of its non-dropped experts
        for t in range(T):
            kept = sum(float(w[t, j]) for j in range(K) if unit[idx[t, j]] >= 0)
            r = [int(v) for v in rows.token_rows[t, :K] if v >= 0]
            assert abs(sum(float(rows.row_weight[i]) for i in r) - kept) < 1e-5
            assert all(rows.row_token[i] == t for i in r)
            assert rows.row_weight[rows.token_rows[t, K]] == 1.0
            # the set of units the rows sit in == the set of units of the non-dropped experts
            units_rows = {int(np.searchsorted(rows.unit_off, i, side="right") - 1) for i in r}
            assert units_rows == {int(unit[idx[t, j]]) for j in range(K) if unit[idx[t, j]] >= 0}
        if thr == 1.0:
            assert rows.n_rows == T * K + T
            assert (rows.unit_cnt[:m] == cnt).all()


def test_everything_on_one_united_expert():
    """threshold 0 and way = m: one dense united-expert pass, one row per token, weight 1."""
    rng = np.random.default_rng(5)
    T, K, m = 50, 3, 8
    idx = np.stack([rng.permutation(m)[:K] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, K)).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    cnt = O.expert_counts(idx, m)
    unit, _ = O.brownout_decide(cnt, m, 0.0, False)
    rows = O.build_rows(idx, w, m, m, 0, unit)
    assert rows.n_rows == T and rows.unit_cnt[m] == T
    assert np.allclose(rows.row_weight, 1.0, atol=1e-6)
    assert (rows.row_token == np.arange(T)).all()
