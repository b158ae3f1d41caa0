"""TEST INFRASTRUCTURE ONLY: plain Python statements of the paper's control-plane formulas, against which
the library's controller and the serving-loop harness are checked.  Nothing under the package imports it.

  salc_update        Algorithm 2 (SLO-Aware Latency Control Algorithm), one call
  p90                get_recent_P90_latency of Algorithm 2: sort, take the value at the 90th percentile rank
  md1_response_time  the M/D/1 mean response time of "Theoretical Foundations of LLM Service Modeling",
                     W = lambda tau^2 / (2 (1 - lambda tau)) + tau
Reading taken where the paper is silent: the threshold is kept inside [0, 1]; the P90 of n values is the one
of rank ceil(0.9 n).
"""
import math


def salc_update(threshold, latency, slo, warning_factor, increment, shrink_ratio):
    warning_line = slo * warning_factor
    if latency < warning_line:
        threshold = threshold + increment
    elif latency > slo:
        threshold = threshold * shrink_ratio
    return min(1.0, max(0.0, threshold))


def p90(latencies):
    s = sorted(latencies)
    return s[math.ceil(0.9 * len(s)) - 1]


def md1_response_time(lam, tau):
    return lam * tau * tau / (2.0 * (1.0 - lam * tau)) + tau
