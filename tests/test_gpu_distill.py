"""GPU parity of the united-expert distillation (section "United Expert Model", MSE equation): the library's
trainer through the C ABI against the float64 oracle, on the same seeded calibration tokens and teachers."""
import numpy as np
import pytest
import torch

import paper_2507_17133_amd as P
from oracle import distill_oracle as DO
from paper_2507_17133_amd import workloads as WL
from tests._util import npf

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _setup(cfg, n):
    torch.cuda.set_device(0)
    L = WL.make_layer(cfg, 0, "cpu")
    calib = WL.make_activations(cfg, 0, "cpu", name="calib", n=n)
    experts = tuple(a.to(DEV) for a in L.experts)
    return L, calib, experts


def _teachers(L, lo, hi):
    ex = [npf(a).astype(np.float64) for a in L.experts]
    return [(ex[0][i], ex[1][i], ex[2][i]) for i in range(lo, hi)]


# Tolerance on the loss history.  The oracle works in float64; the library rounds the student's weights,
# SwiGLU output, dY and the activation gradients to bf16 (2^-9 relative each) before every GEMM and holds the
# teacher outputs in half precision.  These are zero-mean perturbations of a sum over n*d = 16384 terms, so
# the loss itself moves by ~1e-3 relative; the bound below leaves room for the drift of 30 Adam steps whose
# normalised update turns small gradient errors into full-size steps on weights with near-zero gradient.
LOSS_RTOL = 2e-2


def test_loss_history_follows_the_oracle():
    cfg = WL.LayerConfig("distill", T=128, d=128, F=192, m=7, K=2, way=3)
    steps, lr, n = 30, 2e-3, 128
    L, calib, experts = _setup(cfg, n)
    c = P.config_of(cfg)
    united, loss0 = P.moe_build_united(c, experts, calib.to(DEV))
    start = [npf(u).astype(np.float64) for u in united]
    hist = npf(P.moe_distill_united(c, experts, united, calib.to(DEV), steps, lr))
    torch.cuda.synchronize()
    assert hist.shape == (3, steps + 1)
    x = npf(calib).astype(np.float64)
    for g in range(2):
        teachers = _teachers(L, 3 * g, 3 * g + 3)
        w_ref, h_ref = DO.distill(x, tuple(s[g] for s in start), teachers, steps, lr)
        assert np.allclose(hist[g], h_ref, rtol=LOSS_RTOL), (g, hist[g], h_ref)
        assert hist[g][-1] < 0.8 * hist[g][0]                                  # it did learn something
        # the trained bf16 weights, evaluated by the oracle, reach the loss the library reports
        got = tuple(npf(u[g]).astype(np.float64) for u in united)
        assert abs(DO.loss(x, got, teachers) - hist[g][-1]) <= LOSS_RTOL * hist[g][-1]
        # and they moved where the oracle's weights moved (Adam's normalised update takes full-size steps on
        # weights whose gradient is rounding noise, so single weights may differ by up to lr per step and side)
        for a, b, s0 in zip(got, w_ref, start):
            assert np.abs(a - b).max() <= 2.0 * lr * steps
            da, db = (a - s0[g]).ravel(), (b - s0[g]).ravel()
            cos = float(da @ db / np.sqrt((da @ da) * (db @ db)))
            print("group", g, "movement cosine", cos, "max diff", np.abs(a - b).max())
            assert cos >= 0.9
    # the first entry is the loss of the starting point, which moe_build_united reports too
    assert np.allclose(hist[:, 0], npf(loss0), rtol=3e-2, atol=1e-6)
    # single-member group: the student is the member, loss 0
    assert (hist[2] == 0).all()
    for k in range(3):
        assert torch.equal(united[k][2], experts[k][6])


def test_zero_steps_reports_the_loss_and_keeps_the_student():
    cfg = WL.LayerConfig("distill0", T=64, d=64, F=128, m=4, K=2, way=2)
    L, calib, experts = _setup(cfg, 192)
    c = P.config_of(cfg)
    united = tuple(u.to(DEV) for u in WL.make_random_united(cfg, 3, "cpu"))
    before = [u.clone() for u in united]
    hist = npf(P.moe_distill_united(c, experts, united, calib.to(DEV), 0, 1e-3))
    assert hist.shape == (2, 1)
    x = npf(calib).astype(np.float64)
    for g in range(2):
        want = DO.loss(x, tuple(npf(b[g]).astype(np.float64) for b in before), _teachers(L, 2 * g, 2 * g + 2))
        assert abs(hist[g, 0] - want) <= 1e-2 * want
    for a, b in zip(united, before):
        assert torch.equal(a, b)


def test_identical_teachers_are_a_fixed_point_up_to_rounding():
    # both members equal: the parameter mean is the member, the loss floor is 0 and the gradient is rounding
    # noise only, so the loss must stay negligible against the output power
    cfg = WL.LayerConfig("distill_fix", T=64, d=64, F=64, m=2, K=1, way=2)
    L, calib, experts = _setup(cfg, 64)
    experts = tuple(a[:1].repeat(2, 1, 1).contiguous() for a in experts)
    c = P.config_of(cfg)
    united, _ = P.moe_build_united(c, experts, calib.to(DEV))
    hist = npf(P.moe_distill_united(c, experts, united, calib.to(DEV), 3, 1e-5))
    x = npf(calib).astype(np.float64)
    t = tuple(npf(a[0]).astype(np.float64) for a in experts)
    power = (DO.ffn(x, *t) ** 2).sum() / x.shape[0]
    assert (hist[0] <= 1e-4 * power).all(), (hist, power)


def test_bad_arguments_are_rejected():
    cfg = WL.LayerConfig("distill_bad", T=64, d=64, F=64, m=2, K=1, way=2)
    L, calib, experts = _setup(cfg, 96)                                        # 96 is not a multiple of 64
    c = P.config_of(cfg)
    united, _ = P.moe_build_united(c, experts)
    with pytest.raises(P.MoeError) as ei:
        P.moe_distill_united(c, experts, united, calib.to(DEV), 1, 1e-3)
    assert ei.value.status == -2
    ok = calib[:64].contiguous().to(DEV)
    with pytest.raises(P.MoeError) as ei:
        P.moe_distill_united(c, experts, united, ok, -1, 1e-3, workspace=torch.empty(1 << 24, dtype=torch.uint8, device=DEV))
    assert ei.value.status == -1
    with pytest.raises(P.MoeError):
        P.moe_distill_united(c, experts, united, ok, 1, 1e-3, workspace=torch.empty(1024, dtype=torch.uint8, device=DEV))
