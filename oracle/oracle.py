"""ctypes front end of the CPU oracle (oracle/brownout_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  Nothing in the product package may import it.

Every function takes and returns numpy arrays; all arithmetic happens in the C
file, this module only marshals arguments and composes the steps in the order
Algorithm 1 / the layer equation give them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "brownout_oracle.c")
_LIB = os.path.join(_HERE, "libbrownout_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over the outermost loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_build_rows.restype = C.c_int32
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def gate_logits(x, gate_w, gate_bias=None):
    """s[t,i] = x_t . e_i (+ bias_i).  Returns (s64 [T,m] double, s32 [T,m] float)."""
    x, gate_w, gate_bias = _f32(x), _f32(gate_w), _f32(gate_bias)
    T, d = x.shape
    m = gate_w.shape[0]
    assert gate_w.shape == (m, d)
    s64 = np.empty((T, m), np.float64)
    s32 = np.empty((T, m), np.float32)
    _load().oracle_gate_logits(_p(x), C.c_int(T), C.c_int(d), _p(gate_w), _p(gate_bias), C.c_int(m),
                               _p(s64), _p(s32))
    return s64, s32


def topk(s64, s32, K, score_fn=0):
    """Returns (topk_idx [T,K] i32, topk_w [T,K] f32, margin [T] f64)."""
    s64 = np.ascontiguousarray(s64, np.float64)
    s32 = _f32(s32)
    T, m = s32.shape
    assert 1 <= K <= m
    idx = np.empty((T, K), np.int32)
    w = np.empty((T, K), np.float32)
    margin = np.empty((T,), np.float64)
    _load().oracle_topk(_p(s64), _p(s32), C.c_int(T), C.c_int(m), C.c_int(K), C.c_int(score_fn),
                        _p(idx), _p(w), _p(margin))
    return idx, w, margin


def expert_counts(topk_idx, m):
    topk_idx = _i32(topk_idx)
    T, K = topk_idx.shape
    cnt = np.empty((m,), np.int32)
    _load().oracle_expert_counts(_p(topk_idx), C.c_int(T), C.c_int(K), C.c_int(m), _p(cnt))
    return cnt


def brownout_decide(cnt, way, threshold, use_full_brownout=False):
    """Algorithm 1's split.  Returns (unit [m] i32, in_s1 [m] u8)."""
    cnt = _i32(cnt)
    m = cnt.shape[0]
    unit = np.empty((m,), np.int32)
    in_s1 = np.empty((m,), np.uint8)
    _load().oracle_brownout_decide(_p(cnt), C.c_int(m), C.c_int(way), C.c_double(threshold),
                                   C.c_int(1 if use_full_brownout else 0), _p(unit), _p(in_s1))
    return unit, in_s1


@dataclass
class Rows:
    unit_cnt: np.ndarray
    unit_off: np.ndarray
    row_token: np.ndarray
    row_weight: np.ndarray
    token_rows: np.ndarray
    n_rows: int


def build_rows(topk_idx, topk_w, m, way, n_shared, unit) -> Rows:
    topk_idx, topk_w, unit = _i32(topk_idx), _f32(topk_w), _i32(unit)
    T, K = topk_idx.shape
    G = (m + way - 1) // way
    U = m + G + n_shared
    cap = T * (K + n_shared)
    unit_cnt = np.empty((U,), np.int32)
    unit_off = np.empty((U + 1,), np.int32)
    row_token = np.full((cap,), -1, np.int32)
    row_weight = np.zeros((cap,), np.float32)
    token_rows = np.empty((T, K + n_shared), np.int32)
    n = _load().oracle_build_rows(_p(topk_idx), _p(topk_w), C.c_int(T), C.c_int(K), C.c_int(m),
                                  C.c_int(way), C.c_int(n_shared), _p(unit), _p(unit_cnt), _p(unit_off),
                                  _p(row_token), _p(row_weight), _p(token_rows))
    return Rows(unit_cnt, unit_off, row_token[:n].copy(), row_weight[:n].copy(), token_rows, int(n))


def ffn(x, w1, w3, w2):
    """SwiGLU FFN of ONE expert on rows x [n,d]; w1,w3 [F,d], w2 [d,F].  Returns [n,d] double."""
    x, w1, w3, w2 = _f32(x), _f32(w1), _f32(w3), _f32(w2)
    n, d = x.shape
    F = w1.shape[0]
    assert w1.shape == (F, d) and w3.shape == (F, d) and w2.shape == (d, F)
    y = np.empty((n, d), np.float64)
    _load().oracle_ffn(_p(x), C.c_int(n), C.c_int(d), C.c_int(F), _p(w1), _p(w3), _p(w2), _p(y))
    return y


def forward_tokens(x, topk_idx, topk_w, unit, way, experts, united=None, shared=None,
                   add_residual=False, tokens=None):
    """The layer equation for the listed tokens (all if None).  experts/united/shared are
    (w1 [n,F,d], w3 [n,F,d], w2 [n,d,F]) triples or None.  Returns [n_tok,d] float."""
    x, topk_idx, topk_w, unit = _f32(x), _i32(topk_idx), _f32(topk_w), _i32(unit)
    T, d = x.shape
    K = topk_idx.shape[1]
    ew1, ew3, ew2 = (_f32(a) for a in experts)
    m, F = ew1.shape[0], ew1.shape[1]
    uw1 = uw3 = uw2 = None
    if united is not None:
        uw1, uw3, uw2 = (_f32(a) for a in united)
    elif (unit >= m).any():
        raise ValueError("a united unit is used but no united weights were given")
    ns, Fs, sw1, sw3, sw2 = 0, 0, None, None, None
    if shared is not None:
        sw1, sw3, sw2 = (_f32(a) for a in shared)
        ns, Fs = sw1.shape[0], sw1.shape[1]
    tl = None if tokens is None else _i32(tokens)
    n_tok = T if tl is None else tl.shape[0]
    out = np.empty((n_tok, d), np.float32)
    _load().oracle_forward_tokens(
        _p(x), C.c_int(T), C.c_int(d), C.c_int(F), C.c_int(m), C.c_int(K), C.c_int(way),
        _p(topk_idx), _p(topk_w), _p(unit), _p(ew1), _p(ew3), _p(ew2), _p(uw1), _p(uw3), _p(uw2),
        C.c_int(ns), C.c_int(Fs), _p(sw1), _p(sw3), _p(sw2), C.c_int(1 if add_residual else 0),
        _p(tl), C.c_int(n_tok), _p(out))
    return out


def united_mean(w, way):
    """Element-wise mean over each group of `way` consecutive experts.  w [m,...] -> [G,...] double."""
    w = _f32(w)
    m = w.shape[0]
    G = (m + way - 1) // way
    n_elem = int(np.prod(w.shape[1:]))
    u = np.empty((G,) + w.shape[1:], np.float64)
    _load().oracle_united_mean(_p(w), C.c_int(m), C.c_int(way), C.c_size_t(n_elem), _p(u))
    return u


def united_loss(calib_x, way, experts, united):
    """Per-group distillation loss on the calibration tokens.  Returns [G] double."""
    calib_x = _f32(calib_x)
    n, d = calib_x.shape
    ew1, ew3, ew2 = (_f32(a) for a in experts)
    uw1, uw3, uw2 = (_f32(a) for a in united)
    m, F = ew1.shape[0], ew1.shape[1]
    G = (m + way - 1) // way
    assert uw1.shape[0] == G
    loss = np.empty((G,), np.float64)
    _load().oracle_united_loss(_p(calib_x), C.c_int(n), C.c_int(d), C.c_int(F), C.c_int(m), C.c_int(way),
                               _p(ew1), _p(ew3), _p(ew2), _p(uw1), _p(uw3), _p(uw2), _p(loss))
    return loss


@dataclass
class Route:
    s64: np.ndarray
    s32: np.ndarray
    topk_idx: np.ndarray
    topk_w: np.ndarray
    margin: np.ndarray
    expert_cnt: np.ndarray
    expert_unit: np.ndarray
    in_s1: np.ndarray
    rows: Rows


def route(x, gate_w, gate_bias, K, way, threshold, use_full_brownout=False, score_fn=0, n_shared=0) -> Route:
    """Gate -> TopK -> counts -> Algorithm 1 -> row lists, in that order."""
    s64, s32 = gate_logits(x, gate_w, gate_bias)
    idx, w, margin = topk(s64, s32, K, score_fn)
    m = gate_w.shape[0]
    cnt = expert_counts(idx, m)
    unit, in_s1 = brownout_decide(cnt, way, threshold, use_full_brownout)
    rows = build_rows(idx, w, m, way, n_shared, unit)
    return Route(s64, s32, idx, w, margin, cnt, unit, in_s1, rows)


def forward_tokens_lazy(x_rows, topk_idx_rows, topk_w_rows, unit, m, get_weights, n_shared=0, add_residual=False):
    """The layer equation for a few tokens when the weights are too large to hold as one float
    array: x_rows [n,d], topk_idx_rows / topk_w_rows [n,K] are the sampled tokens' data and
    get_weights(kind, index) returns one FFN's (w1 [F,d], w3 [F,d], w2 [d,F]) as float arrays,
    kind in {"expert", "united", "shared"}.  Every term FFN(x_t) of the equation is evaluated by
    ffn() (one call per distinct FFN, on the rows of all sampled tokens that have a term in it:
    rows are independent there, and the call spreads them over the host cores); the terms of a
    token are then added in double in the equation's order: residual, shared experts, the TopK
    entries in order (dropped experts contribute nothing).  Returns [n,d] double."""
    x_rows = _f32(x_rows)
    n, d = x_rows.shape
    K = topk_idx_rows.shape[1]
    # which sampled tokens have a term in which FFN: (kind, index) -> [(token q, slot)]
    terms = {}
    for q in range(n):
        for s in range(n_shared):
            terms.setdefault(("shared", s), []).append((q, s))
        for j in range(K):
            u = int(unit[int(topk_idx_rows[q, j])])
            if u < 0:
                continue
            key = ("expert", u) if u < m else ("united", u - m)
            terms.setdefault(key, []).append((q, n_shared + j))
    term_y = {}
    for key, lst in terms.items():
        qs = np.array([q for q, _ in lst], np.int64)
        y = ffn(x_rows[qs], *get_weights(*key))
        for i, (q, slot) in enumerate(lst):
            term_y[(q, slot)] = y[i]
    out = np.zeros((n, d), np.float64)
    for q in range(n):
        if add_residual:
            out[q] += x_rows[q].astype(np.float64)
        for s in range(n_shared):
            out[q] += term_y[(q, s)]
        for j in range(K):
            if (q, n_shared + j) in term_y:
                out[q] += float(topk_w_rows[q, j]) * term_y[(q, n_shared + j)]
    return out
