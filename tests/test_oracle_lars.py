"""Pins for the LARS oracle and the poly schedule: hand-computed trust ratios and
updates, the rule's invariants, and the schedule's closed form.  No HIP path here.

Hyper-parameters are the paper's (momentum 0.9, weight decay 0.0005, poly power 2:
caption of the AlexNet accuracy table) unless a case needs others.
"""
import math

import numpy as np
import pytest

import oracle
from paper_1709_05011_amd import synth

ETA, MOM, WD = 0.001, 0.9, 0.0005


def _f(*vals):
    return np.array(vals, dtype=np.float32)


def test_trust_ratio_hand_values():
    # ||w|| = 5, ||g|| = 1 (to float32 rounding of 0.6, 0.8): lambda = 0.005 / 1.0025
    w, g, v = [_f(3, 4)], [_f(0.6, 0.8)], [_f(0, 0)]
    trust, norms = oracle.lars_step(w, g, v, ETA, MOM, WD, 1.0)
    assert norms[0, 0] == 5.0
    assert abs(norms[0, 1] - 1.0) < 1e-7
    assert abs(trust[0] - 0.004987531172069826) < 1e-9
    # ||w|| = 1, ||g|| = 1/2 exactly: lambda = 0.001 / 0.5005
    w, g, v = [_f(.5, .5, .5, .5)], [_f(.25, -.25, .25, -.25)], [np.zeros(4, np.float32)]
    trust, norms = oracle.lars_step(w, g, v, ETA, MOM, WD, 1.0)
    assert norms[0, 0] == 1.0 and norms[0, 1] == 0.5
    assert abs(trust[0] - 0.0019980019980019984) < 1e-15


def test_two_steps_hand_values():
    w, g, v = [_f(3, 4)], [_f(0.6, 0.8)], [_f(0, 0)]
    oracle.lars_step(w, g, v, ETA, MOM, WD, 1.0)
    # v1 = lambda * (0.6 + 0.0015, 0.8 + 0.002) = (0.003, 0.004); w1 = (2.997, 3.996)
    np.testing.assert_allclose(v[0], [0.003, 0.004], rtol=2e-7)
    np.testing.assert_allclose(w[0], [2.997, 3.996], rtol=2e-7)
    trust, _ = oracle.lars_step(w, g, v, ETA, MOM, WD, 1.0)
    # ||w1|| = 4.995: lambda2 = 0.004995 / (1 + 0.0024975)
    assert abs(trust[0] - 0.004982556066224604) < 1e-9
    np.testing.assert_allclose(v[0], [0.005697, 0.007596], rtol=2e-6)
    np.testing.assert_allclose(w[0], [2.991303, 3.988404], rtol=2e-7)


@pytest.mark.parametrize("wd,want", [(0.0005, 2.0), (0.00005, 20.0)])
def test_zero_gradient_gives_eta_over_beta_and_pure_decay(wd, want):
    w, g, v = [_f(3, 4)], [_f(0, 0)], [_f(0.5, -0.25)]
    w0, v0 = w[0].copy(), v[0].copy()
    trust, _ = oracle.lars_step(w, g, v, ETA, MOM, wd, 1.0)
    assert abs(trust[0] - want) < 1e-12 * want
    # v <- m v + gamma*eta*w  (weight decay and momentum only), w <- w - v
    v_ref = MOM * v0.astype(np.float64) + 1.0 * ETA * w0.astype(np.float64)
    np.testing.assert_allclose(v[0], v_ref, rtol=2e-7)
    np.testing.assert_allclose(w[0], w0 - v_ref, rtol=2e-7)


def test_zero_norm_fallbacks():
    # ||w|| = 0: lambda = 1, plain momentum SGD step (nothing to decay)
    w, g, v = [_f(0, 0, 0)], [_f(1, -2, 0.5)], [_f(0, 0, 0)]
    trust, _ = oracle.lars_step(w, g, v, ETA, 0.0, WD, 0.25)
    assert trust[0] == 1.0
    np.testing.assert_array_equal(v[0], _f(0.25, -0.5, 0.125))
    np.testing.assert_array_equal(w[0], _f(-0.25, 0.5, -0.125))
    # g = 0 and no decay: denominator 0, lambda = 1, update is v <- m v
    w, g, v = [_f(1, 2)], [_f(0, 0)], [_f(0.5, 0.5)]
    trust, _ = oracle.lars_step(w, g, v, ETA, 0.5, 0.0, 1.0)
    assert trust[0] == 1.0
    np.testing.assert_array_equal(v[0], _f(0.25, 0.25))
    np.testing.assert_array_equal(w[0], _f(0.75, 1.75))
    # empty tensor and empty list are legal
    trust, _ = oracle.lars_step([np.zeros(0, np.float32)], [np.zeros(0, np.float32)], [np.zeros(0, np.float32)],
                                ETA, MOM, WD, 1.0)
    assert trust[0] == 1.0
    trust, _ = oracle.lars_step([], [], [], ETA, MOM, WD, 1.0)
    assert trust.shape == (0,)


@pytest.mark.parametrize("wd", [0.0, 0.0005])
def test_trust_ratio_invariant_to_joint_scaling(wd):
    w = synth.normal((1000,), 1)
    g = synth.normal((1000,), 2, std=0.01)
    t1, _ = oracle.lars_step([w.copy()], [g], [np.zeros_like(w)], ETA, MOM, wd, 1.0)
    s = np.float32(8.0)  # power of two: scaling is exact in float32
    t2, _ = oracle.lars_step([w * s], [g * s], [np.zeros_like(w)], ETA, MOM, wd, 1.0)
    assert abs(t1[0] - t2[0]) <= 1e-14 * t1[0]


def test_step_length_is_lr_times_eta_without_decay_and_momentum():
    # beta = 0, m = 0: ||delta w|| / ||w|| = gamma * eta whatever g is -- the defining property.
    for seed, gstd in [(3, 1.0), (4, 1e-3), (5, 50.0)]:
        w = synth.normal((4096,), seed)
        g = synth.normal((4096,), seed + 10, std=gstd)
        w0 = w.astype(np.float64)
        w1 = w.copy()
        oracle.lars_step([w1], [g], [np.zeros_like(w)], ETA, 0.0, 0.0, 0.5)
        ratio = np.linalg.norm(w1.astype(np.float64) - w0) / np.linalg.norm(w0)
        assert abs(ratio - 0.5 * ETA) < 1e-4 * 0.5 * ETA  # float32 storage of w limits this


def test_trust_ratio_linear_in_eta():
    w, g = synth.normal((777,), 6), synth.normal((777,), 7)
    t1, _ = oracle.lars_step([w.copy()], [g], [np.zeros_like(w)], 0.001, MOM, WD, 1.0)
    t2, _ = oracle.lars_step([w.copy()], [g], [np.zeros_like(w)], 0.004, MOM, WD, 1.0)
    assert abs(t2[0] / t1[0] - 4.0) < 1e-13


def test_tensors_are_independent_of_list_order_and_grouping():
    sizes = [64, 1, 4097, 300, 2048]
    w = [synth.normal((n,), 100 + i) for i, n in enumerate(sizes)]
    g = [synth.normal((n,), 200 + i, std=0.02) for i, n in enumerate(sizes)]
    v = [synth.normal((n,), 300 + i, std=0.001) for i, n in enumerate(sizes)]
    wa, va = [a.copy() for a in w], [a.copy() for a in v]
    ta, _ = oracle.lars_step(wa, g, va, ETA, MOM, WD, 0.7)
    perm = [3, 0, 4, 2, 1]
    wb, vb = [w[i].copy() for i in perm], [v[i].copy() for i in perm]
    tb, _ = oracle.lars_step(wb, [g[i] for i in perm], vb, ETA, MOM, WD, 0.7)
    for j, i in enumerate(perm):
        assert ta[i] == tb[j]
        assert np.array_equal(wa[i], wb[j]) and np.array_equal(va[i], vb[j])
    wc, vc = [a.copy() for a in w], [a.copy() for a in v]
    t1, _ = oracle.lars_step(wc[:2], g[:2], vc[:2], ETA, MOM, WD, 0.7)
    t2, _ = oracle.lars_step(wc[2:], g[2:], vc[2:], ETA, MOM, WD, 0.7)
    assert np.array_equal(np.concatenate([t1, t2]), ta)
    assert all(np.array_equal(a, b) for a, b in zip(wa, wc))


def test_update_against_numpy_float64_formula_on_random_tensors():
    w = synth.normal((5000,), 8)
    g = synth.normal((5000,), 9, std=0.03)
    v = synth.normal((5000,), 10, std=0.002)
    w64, g64, v64 = (a.astype(np.float64) for a in (w, g, v))
    nw, ng = math.sqrt(math.fsum(w64 * w64)), math.sqrt(math.fsum(g64 * g64))
    lam = ETA * nw / (ng + WD * nw)
    v_ref = MOM * v64 + 0.3 * lam * (g64 + WD * w64)
    trust, norms = oracle.lars_step([w], [g], [v], ETA, MOM, WD, 0.3)
    assert abs(trust[0] - lam) < 1e-13 * lam
    assert abs(norms[0, 0] - nw) < 1e-12 * nw and abs(norms[0, 1] - ng) < 1e-12 * ng
    np.testing.assert_allclose(v, v_ref, rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(w, w64 - v_ref, rtol=1e-6, atol=1e-12)


def test_poly_schedule_closed_form():
    T = synth.poly_total_iters()  # 90 epochs * 1.28 M images / 32768
    assert T == 3516
    assert oracle.poly_lr(1.0, 0, T) == 1.0
    assert oracle.poly_lr(1.0, T, T) == 0.0
    assert oracle.poly_lr(1.0, T + 5, T) == 0.0
    assert abs(oracle.poly_lr(1.0, 1000, T) - (1 - 1000 / 3516) ** 2) < 1e-15
    assert abs(oracle.poly_lr(0.2, 879, T) - 0.2 * 0.75 ** 2) < 1e-15  # a quarter of the way
    assert abs(oracle.poly_lr(3.0, 10, 40, 1.0) - 2.25) < 1e-15


# ---- per-tensor coefficients, skip list, warm-up schedule ----

def _rand_lists(sizes, seed):
    w = [synth.normal((n,), seed + 3 * i) for i, n in enumerate(sizes)]
    g = [synth.normal((n,), seed + 3 * i + 1, std=0.01) for i, n in enumerate(sizes)]
    v = [synth.normal((n,), seed + 3 * i + 2, std=0.001) for i, n in enumerate(sizes)]
    return w, g, v


def test_per_tensor_form_with_scalar_arrays_equals_the_plain_rule():
    sizes = [5, 1, 300, 64]
    w1, g1, v1 = _rand_lists(sizes, 900)
    w2, v2 = [a.copy() for a in w1], [a.copy() for a in v1]
    t1, n1 = oracle.lars_step(w1, g1, v1, ETA, MOM, WD, 0.7)
    t2, n2 = oracle.lars_step_ex(w2, g1, v2, 123.0, MOM, 456.0, 0.7, eta_per_tensor=[ETA] * 4, wd_per_tensor=[WD] * 4,
                                 skip=[0] * 4)
    np.testing.assert_array_equal(t1, t2)
    for a, b in zip(w1 + v1, w2 + v2):
        np.testing.assert_array_equal(a, b)


def test_per_tensor_hand_values_and_skip():
    # tensor 0: ||w|| = 5, ||g|| = 1, eta 0.002, beta 0.001 -> lambda = 0.01 / 1.005
    # tensor 1: skipped -> lambda = 1: v = m v + gamma (g + beta w), the plain momentum step with weight decay
    # tensor 2: no array entry differs from the scalars' role: eta 0.001, beta 0 -> lambda = 0.001 * 2 / 0.5
    w = [_f(3, 4), _f(1, -2), _f(0, 2)]
    g = [_f(0.6, 0.8), _f(0.5, 0.25), _f(0.3, 0.4)]
    v = [_f(0, 0), _f(0.125, -0.5), _f(0, 0)]
    w0, v0 = [a.astype(np.float64) for a in w], [a.astype(np.float64) for a in v]
    trust, _ = oracle.lars_step_ex(w, g, v, 9.0, 0.5, 9.0, 0.25, eta_per_tensor=[0.002, 0.7, 0.001],
                                   wd_per_tensor=[0.001, 0.01, 0.0], skip=[0, 1, 0])
    assert abs(trust[0] - 0.01 / 1.005) < 1e-9
    assert trust[1] == 1.0
    assert abs(trust[2] - 0.004) < 1e-9
    v1_ref = 0.5 * v0[1] + 0.25 * (np.array([0.5, 0.25]) + 0.01 * w0[1])
    np.testing.assert_allclose(v[1], v1_ref, rtol=2e-7)
    np.testing.assert_allclose(w[1], w0[1] - v1_ref, rtol=2e-7)
    v2_ref = 0.25 * 0.004 * np.array([0.3, 0.4], dtype=np.float32).astype(np.float64)
    np.testing.assert_allclose(v[2], v2_ref, rtol=3e-7)


def test_skip_only_changes_the_skipped_tensors():
    sizes = [33, 7, 129]
    w1, g1, v1 = _rand_lists(sizes, 950)
    w2, v2 = [a.copy() for a in w1], [a.copy() for a in v1]
    oracle.lars_step_ex(w1, g1, v1, ETA, MOM, WD, 0.5)
    t2, _ = oracle.lars_step_ex(w2, g1, v2, ETA, MOM, WD, 0.5, skip=[0, 1, 0])
    np.testing.assert_array_equal(w1[0], w2[0])
    np.testing.assert_array_equal(w1[2], w2[2])
    assert t2[1] == 1.0 and not np.array_equal(w1[1], w2[1])


def test_warmup_schedule_endpoints_ramp_and_decay():
    base, start, W, T = 3.2, 0.1, 195, 3516           # 5 epochs of 39 iterations each at batch 32K; 90 epochs in all
    assert oracle.warmup_poly_lr(base, start, 0, W, T) == start
    assert abs(oracle.warmup_poly_lr(base, start, W, W, T) - base) < 1e-15          # the ramp reaches the base rate ...
    assert abs(oracle.warmup_poly_lr(base, start, W - 1, W, T) - (start + (base - start) * (W - 1) / W)) < 1e-12
    mid = oracle.warmup_poly_lr(base, start, 97, W, T)                                # ... linearly
    assert abs(mid - (start + (base - start) * 97 / 195)) < 1e-12
    for t in (W + 1, 1000, 3000, T - 1):
        want = base * (1 - (t - W) / (T - W)) ** 2
        assert abs(oracle.warmup_poly_lr(base, start, t, W, T) - want) < 1e-12
    assert oracle.warmup_poly_lr(base, start, T, W, T) == 0.0
    # without warm-up it is the plain poly policy
    for t in (0, 17, 2000):
        assert oracle.warmup_poly_lr(base, start, t, 0, T) == oracle.poly_lr(base, t, T)
    # monotone: up during the ramp, down afterwards
    vals = [oracle.warmup_poly_lr(base, start, t, W, T) for t in range(0, T + 1, 13)]
    peak = int(np.argmax(vals))
    assert all(a < b for a, b in zip(vals[:peak], vals[1:peak + 1])) and all(a > b for a, b in zip(vals[peak:], vals[peak + 1:]))
