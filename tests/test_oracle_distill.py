"""Pins of the distillation oracle (CPU): gradients against finite differences, fixed point, the closed
form of the best possible student output, descent."""
import numpy as np

from oracle import distill_oracle as DO


def _problem(seed=0, n=24, d=8, F=12, k=3):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(n, d))
    teachers = [(rng.normal(size=(F, d)) / np.sqrt(d), rng.normal(size=(F, d)) / np.sqrt(d),
                 rng.normal(size=(d, F)) / np.sqrt(F)) for _ in range(k)]
    student = tuple(sum(t[j] for t in teachers) / k for j in range(3))
    return x, student, teachers


def test_gradients_match_central_differences():
    x, student, teachers = _problem()
    val, grads = DO.loss_and_grads(x, student, teachers)
    assert np.isclose(val, DO.loss(x, student, teachers), rtol=1e-12)
    rng = np.random.default_rng(1)
    h = 1e-6
    for j in range(3):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in student[j].shape)
            plus = [p.copy() for p in student]
            minus = [p.copy() for p in student]
            plus[j][idx] += h
            minus[j][idx] -= h
            num = (DO.loss(x, tuple(plus), teachers) - DO.loss(x, tuple(minus), teachers)) / (2 * h)
            assert np.isclose(grads[j][idx], num, rtol=1e-5, atol=1e-9), (j, idx, grads[j][idx], num)


def test_single_teacher_is_a_fixed_point():
    x, _, teachers = _problem(k=1)
    val, grads = DO.loss_and_grads(x, teachers[0], teachers)
    assert val == 0.0 and all((g == 0).all() for g in grads)
    w, hist = DO.distill(x, teachers[0], teachers, steps=3, lr=1e-2)
    assert (hist == 0).all() and all((a == b).all() for a, b in zip(w, teachers[0]))


def test_loss_floor_is_the_spread_of_the_teachers():
    # over all possible student outputs the MSE equation is minimised by the mean teacher output, where it
    # equals the mean squared deviation of the teachers from their mean: no student can go below that
    x, student, teachers = _problem(seed=3)
    outs = np.stack([DO.ffn(x, *t) for t in teachers])
    floor = ((outs - outs.mean(0)) ** 2).sum() / (len(teachers) * x.shape[0])
    hu = DO.ffn(x, *student)
    assert np.isclose(DO.loss(x, student, teachers), floor + ((hu - outs.mean(0)) ** 2).sum() / x.shape[0], rtol=1e-10)
    w, hist = DO.distill(x, student, teachers, steps=60, lr=5e-3)
    assert (hist >= floor * (1 - 1e-12)).all()


def test_training_descends():
    x, student, teachers = _problem(seed=5, n=64)
    w, hist = DO.distill(x, student, teachers, steps=40, lr=2e-3)
    assert len(hist) == 41
    assert hist[-1] < 0.9 * hist[0]
    assert (np.diff(hist) <= 1e-3 * hist[0]).all()           # small steps: no step makes it noticeably worse
