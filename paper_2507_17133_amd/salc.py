"""Serving-loop harness around the SLO-aware latency controller (Algorithm 2 of the paper).

The controller itself (`salc_update`, `latency_p90`) lives in the C library; this module is the host loop
that would sit in a serving engine: requests arrive, one at a time they are served by an iteration whose
duration depends on the brownout threshold in force, and after every iteration the controller looks at the
P90 latency of the recent time window and moves the threshold.  The iteration time comes from a callable,
so the same loop runs against a latency table measured on the GPU (bench.py --salc) or a synthetic curve
(the CPU tests).  Arrivals are synthetic: a Poisson process with a piecewise constant rate, the shape of
the paper's burst experiment (SLO Violations Rate: the rate doubles at t = 75 s of a 250 s trace).
"""
from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from .binding import latency_p90, salc_update


def poisson_arrivals(rates: Sequence[Tuple[float, float]], duration: float, seed: int = 0) -> np.ndarray:
    """Arrival times in [0, duration) of a Poisson process whose rate is piecewise constant:
    rates = [(t_start, rate), ...] with ascending t_start, the first at 0."""
    rng = np.random.default_rng(seed)
    out: List[float] = []
    for i, (t0, lam) in enumerate(rates):
        t1 = rates[i + 1][0] if i + 1 < len(rates) else duration
        t = t0
        while lam > 0:
            t += rng.exponential(1.0 / lam)
            if t >= t1:
                break
            out.append(t)
    return np.asarray(out, np.float64)


@dataclass
class Trace:
    arrival: np.ndarray
    start: np.ndarray
    finish: np.ndarray
    threshold: np.ndarray        # threshold each request was served with

    @property
    def latency(self) -> np.ndarray:
        return self.finish - self.arrival


def serve(arrival: np.ndarray, service_time: Callable[[float], float], slo: Optional[float] = None,
          threshold0: float = 1.0, window: float = 5.0, warning_factor: float = 0.8, increment: float = 0.1,
          shrink_ratio: float = 0.8) -> Trace:
    """Single server, first come first served.  With slo=None the threshold stays at threshold0 (the
    system without brownout control); otherwise the controller runs after every completed request on the
    latencies of the requests that finished within the last `window` seconds."""
    n = len(arrival)
    start, finish, thr_used = np.empty(n), np.empty(n), np.empty(n)
    thr, free_at, lo = float(threshold0), 0.0, 0
    for i in range(n):
        start[i] = max(arrival[i], free_at)
        thr_used[i] = thr
        finish[i] = start[i] + float(service_time(thr))
        free_at = finish[i]
        if slo is not None:
            while finish[lo] < finish[i] - window:
                lo += 1
            recent = (finish[lo:i + 1] - arrival[lo:i + 1]).tolist()
            thr = salc_update(thr, latency_p90(recent), slo, warning_factor, increment, shrink_ratio)
    return Trace(np.asarray(arrival, np.float64), start, finish, thr_used)


def violation_rate(trace: Trace, slo: float, t_from: float = 0.0) -> float:
    sel = trace.arrival >= t_from
    return float((trace.latency[sel] > slo).mean()) if sel.any() else 0.0
