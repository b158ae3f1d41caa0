"""Control plane (Algorithm 2 and the queueing model it sits on), CPU only: the library's controller
against the plain statement of the algorithm, the P90 against numpy, the serving loop against the M/D/1
closed form the paper quotes, and the behaviour the paper describes under a burst."""
import math
import os

import numpy as np
import pytest

from oracle import salc_oracle as SO
from paper_2507_17133_amd import binding as B
from paper_2507_17133_amd import salc

if not os.path.exists(B.LIB_PATH):
    from paper_2507_17133_amd import build as _build
    _build.build()


def test_update_matches_algorithm_2_on_a_grid():
    for thr in np.linspace(0.0, 1.0, 11):
        for lat in (0.0, 0.1, 0.1999, 0.2, 0.22, 0.25, 0.2501, 0.4):
            for inc, shr in ((0.1, 0.8), (0.05, 0.5), (0.0, 1.0)):
                want = SO.salc_update(thr, lat, 0.25, 0.8, inc, shr)
                assert B.salc_update(thr, lat, 0.25, 0.8, inc, shr) == want


def test_update_worked_values():
    # constants of the paper's burst experiment: SLO 0.25 s, warning factor 0.8, increment 0.1, shrink 0.8
    assert B.salc_update(0.5, 0.10, 0.25) == pytest.approx(0.6)      # below the 0.20 s warning line: +0.1
    assert B.salc_update(0.5, 0.22, 0.25) == 0.5                     # inside the buffer zone: unchanged
    assert B.salc_update(0.5, 0.30, 0.25) == pytest.approx(0.4)      # above the SLO: x0.8
    assert B.salc_update(0.95, 0.10, 0.25) == 1.0                    # kept inside [0, 1]
    assert B.salc_update(0.0, 0.30, 0.25) == 0.0
    assert B.salc_update(0.5, 0.20, 0.25) == 0.5                     # exactly on the warning line: not below it
    assert B.salc_update(0.5, 0.25, 0.25) == 0.5                     # exactly on the SLO: not above it


def test_update_rejects_bad_parameters():
    assert math.isnan(B.salc_update(0.5, 0.1, 0.0))
    assert math.isnan(B.salc_update(0.5, 0.1, 0.25, warning_factor=1.5))
    assert math.isnan(B.salc_update(0.5, 0.1, 0.25, shrink_ratio=1.2))
    assert math.isnan(B.salc_update(0.5, float("nan"), 0.25))
    assert math.isnan(B.latency_p90([]))


def test_p90_is_the_nearest_rank_percentile():
    rng = np.random.default_rng(0)
    for n in (1, 2, 9, 10, 11, 100, 1001):
        v = rng.exponential(1.0, n)
        assert B.latency_p90(v.tolist()) == SO.p90(v.tolist())
        assert B.latency_p90(v.tolist()) == np.sort(v)[math.ceil(0.9 * n) - 1]
    assert B.latency_p90(list(range(1, 11))) == 9.0
    assert B.latency_p90([3.0]) == 3.0


def test_serving_loop_matches_the_md1_closed_form():
    # constant service time, Poisson arrivals, no control: the mean response time of the paper's
    # request model, W = lambda tau^2 / (2 (1 - lambda tau)) + tau
    tau = 0.1
    for rho in (0.3, 0.6, 0.8):
        lam = rho / tau
        arr = salc.poisson_arrivals([(0.0, lam)], 40000 * tau / rho, seed=1)
        tr = salc.serve(arr, lambda thr: tau)
        assert tr.latency.mean() == pytest.approx(SO.md1_response_time(lam, tau), rel=0.04)
        assert (tr.start >= tr.arrival).all() and (np.diff(tr.finish) >= tau - 1e-12).all()


def test_controller_holds_latency_under_a_burst():
    # service time grows with the threshold (more experts touched); the rate doubles at t = 75 s
    tau = lambda thr: 0.02 + 0.08 * thr
    slo = 0.25
    arr = salc.poisson_arrivals([(0.0, 6.0), (75.0, 12.0)], 250.0, seed=2)
    fixed = salc.serve(arr, tau)                                  # threshold 1: overloaded after the burst
    ctl = salc.serve(arr, tau, slo=slo)
    assert salc.violation_rate(fixed, slo, 75.0) > 0.9
    assert salc.violation_rate(ctl, slo, 75.0) < 0.25
    assert ctl.threshold[ctl.arrival < 60.0].mean() > ctl.threshold[ctl.arrival > 100.0].mean()
    assert (ctl.threshold >= 0.0).all() and (ctl.threshold <= 1.0).all()
