"""Pins for the oracle's update and pipelined driver (arXiv 1811.03619,
Algorithm 1: the compute thread decompresses the aggregated gradient of
iteration t-K and applies w[t] = w[t-1] - gamma * g_sum[t-K]; the K slots for
iterations <= 0 start as zero; K = 2 is the optimal width, so the staleness
is exactly one iteration -- Sec. 3.1).

Closed forms and hand arithmetic only; no expected value comes from the
oracle.
"""
import math

import numpy as np
import pytest

from paper_1811_03619_amd import workloads as W

F = np.float32


def delayed_recurrence(a, delay, T):
    """s_t for  s_{t} = s_{t-1} - a * s_{t-1-delay}, with s_j = 1 for j <= 0
    and no step taken while the delayed slot is still the zero slot."""
    s = {j: 1.0 for j in range(-delay - 1, 1)}
    for t in range(1, T + 1):
        s[t] = s[t - 1] - (a * s[t - 1 - delay] if t - delay >= 1 else 0.0)
    return [s[t] for t in range(T + 1)]


def test_closed_form_of_the_staleness_one_recurrence():
    # s_{t+1} = s_t - a s_{t-1}, s_0 = s_1 = 1  has the solution
    # (r1^(t+1) - r2^(t+1)) / (r1 - r2), r = (1 +- sqrt(1-4a))/2.
    a = 0.04
    d = math.sqrt(1 - 4 * a)
    r1, r2 = (1 + d) / 2, (1 - d) / 2
    s = delayed_recurrence(a, 1, 10)
    for t in range(11):
        assert abs(s[t] - (r1 ** (t + 1) - r2 ** (t + 1)) / (r1 - r2)) < 1e-14
    assert abs(s[10] - 0.6825982976) < 1e-12
    assert abs(delayed_recurrence(a, 0, 10)[10] - 0.96 ** 10) < 1e-14


@pytest.mark.parametrize("width", [1, 2, 3])
def test_quadratic_uses_exactly_the_gradient_of_width_minus_one_iterations_ago(orc, width):
    # loss 0.5*||w - w*||^2 on each of p = 4 identical workers, gradients summed
    # by the ring: effective step a = p*lr = 0.04; w_t - w* = s_t (w_0 - w*).
    p, n, lr, T = 4, 4096 * 4 + 9, 0.01, 10
    wstar = W.gaussian(n, 1.0, 31)
    w0 = np.zeros(n, dtype=F)
    ws, _ = orc.pipe_sgd_run(orc.NONE, lambda r, w, t: w - wstar, w0, p, T, lr, width=width)
    s = delayed_recurrence(p * lr, width - 1, T)
    got = (ws[0].astype(np.float64) - wstar) / (w0.astype(np.float64) - wstar)
    assert np.max(np.abs(got - s[T])) < 2e-6
    others = [delayed_recurrence(p * lr, d, T)[T] for d in range(3) if d != width - 1]
    assert all(abs(s[T] - o) > 1e-2 for o in others)        # the pin separates the staleness values
    for r in range(1, p):
        assert np.array_equal(ws[r], ws[0])                  # same w[0] + deterministic staleness


def test_first_width_minus_one_updates_are_no_ops(orc):
    # Alg. 1, communication thread line 1: the slots of iterations <= 0 are zero.
    n, p = 5000, 2
    w0 = W.gaussian(n, 1.0, 33)
    ws, _ = orc.pipe_sgd_run(orc.NONE, lambda r, w, t: np.ones(n, F), w0, p, 1, 0.1, width=2)
    assert np.array_equal(ws[0], w0)
    ws, _ = orc.pipe_sgd_run(orc.NONE, lambda r, w, t: np.ones(n, F), w0, p, 1, 0.5, width=1)
    assert np.array_equal(ws[0], w0 - F(1.0))                # 0.5 * (1+1)


def test_update_is_a_single_rounding_fused_multiply_add(orc):
    # lr = g = 1 + 2^-12: lr*g = 1 + 2^-11 + 2^-24 exactly; w = 1 + 2^-11.
    # One rounding:  w - lr*g = -2^-24.  Rounding the product first (tie to
    # even -> 1 + 2^-11) would give 0.
    g = np.array([1 + 2.0 ** -12], dtype=F)
    w = np.array([1 + 2.0 ** -11], dtype=F)
    orc.sgd_update(orc.NONE, g, None, w, None, lr=1 + 2.0 ** -12)
    assert w[0] == F(-2.0 ** -24)
    # momentum: v = m*v + g with one rounding, then w = w - lr*v with one.
    m = 1 + 2.0 ** -12
    v = np.array([1 + 2.0 ** -12], dtype=F)                  # m*v = 1 + 2^-11 + 2^-24
    g = np.array([-(1 + 2.0 ** -11)], dtype=F)
    w = np.array([0.0], dtype=F)
    orc.sgd_update(orc.NONE, g, None, w, v, lr=2.0, momentum=m)
    assert v[0] == F(2.0 ** -24) and w[0] == F(-2.0 ** -23)


def test_exact_dyadic_step_and_grad_scale(orc):
    w = np.array([1.0, -2.0, 0.5, 0.0], dtype=F)
    g = np.array([0.5, 0.25, -1.0, 8.0], dtype=F)
    orc.sgd_update(orc.NONE, g, None, w, None, lr=0.5)
    assert w.tolist() == [0.75, -2.125, 1.0, -4.0]
    w = np.array([1.0, -2.0, 0.5, 0.0], dtype=F)
    orc.sgd_update(orc.NONE, g, None, w, None, lr=0.5, grad_scale=0.25)     # mean over 4 workers
    assert w.tolist() == [0.9375, -2.03125, 0.625, -1.0]


def test_momentum_constant_gradient_closed_form(orc):
    # v_t = g (1 - m^t)/(1 - m);  w_T = w_0 - lr * sum_t v_t
    n, m, lr, T = 3000, 0.9, 0.01, 25
    g = W.gaussian(n, 1.0, 35)
    w = np.zeros(n, dtype=F)
    v = np.zeros(n, dtype=F)
    for _ in range(T):
        orc.sgd_update(orc.NONE, g, None, w, v, lr=lr, momentum=m)
    gd = g.astype(np.float64)
    vT = gd * (1 - m ** T) / (1 - m)
    wT = -lr * gd * sum((1 - m ** t) / (1 - m) for t in range(1, T + 1))
    assert np.max(np.abs(v - vT) / np.abs(vT)) < 5e-6
    assert np.max(np.abs(w - wT) / np.abs(wT)) < 5e-6


def test_zero_momentum_leaves_v_alone_and_zero_slot_is_a_no_op(orc):
    n = 4096 + 5
    w0 = W.gaussian(n, 1.0, 37)
    for mode in (orc.NONE, orc.TRUNC16, orc.QUANT8):
        slot = np.zeros(n, dtype=orc.payload_dtype(mode))
        sc = np.zeros(2, F) if mode == orc.QUANT8 else None
        w = w0.copy()
        orc.sgd_update(mode, slot, sc, w, None, lr=0.1)
        assert np.array_equal(w.view(np.uint32), w0.view(np.uint32))
        v0 = W.gaussian(n, 1.0, 39)
        v, w = v0.copy(), w0.copy()
        orc.sgd_update(mode, slot, sc, w, v, lr=0.5, momentum=0.5)
        assert np.array_equal(v, v0 * F(0.5))
        assert np.array_equal(w, w0 - F(0.5) * (v0 * F(0.5)))   # all exact: powers of two


@pytest.mark.parametrize("mode", [1, 2])
def test_update_consumes_the_compressed_slot(orc, mode):
    # Alg. 1 lines 4-5: decompress, then step.  Stepping on the compressed
    # slot must equal stepping (uncompressed mode) on its decompressed value.
    n = 4096 * 2 + 100
    x = W.gaussian(n, 3e-4, 41)
    pay, sc = orc.compress(mode, x)
    w1 = W.gaussian(n, 1.0, 43)
    v1 = W.gaussian(n, 0.1, 45)
    w2, v2 = w1.copy(), v1.copy()
    orc.sgd_update(mode, pay, sc, w1, v1, lr=0.01, momentum=0.9)
    orc.sgd_update(orc.NONE, orc.decompress(mode, pay, sc), None, w2, v2, lr=0.01, momentum=0.9)
    assert np.array_equal(w1, w2) and np.array_equal(v1, v2)


def test_float64_brute_force_small_quadratic_with_momentum(orc):
    # 3 parameters, p = 4 workers with different targets, heavy-ball with the
    # one-iteration-stale aggregated gradient, written out in float64.
    p, lr, m, T = 4, 0.01, 0.9, 30
    targets = [np.array([1.0, -2.0, 0.5]) * (k + 1) for k in range(p)]
    w0 = np.array([0.3, 0.1, -0.7])
    w, v, slot = w0.copy(), np.zeros(3), np.zeros(3)
    for t in range(1, T + 1):
        A = sum(w - tk for tk in targets)        # gradients at w[t-1], summed
        v = m * v + slot                         # ... but the step uses last iteration's sum
        w = w - lr * v
        slot = A
    ws, vs = orc.pipe_sgd_run(orc.NONE, lambda r, ww, t: (ww - targets[r]).astype(F), w0.astype(F),
                              p, T, lr, momentum=m, width=2)
    assert np.max(np.abs(ws[0] - w)) < 1e-5 and np.max(np.abs(vs[0] - v)) < 1e-4
    for r in range(1, p):
        assert np.array_equal(ws[r], ws[0]) and np.array_equal(vs[r], vs[0])


@pytest.mark.parametrize("mode", [1, 2])
def test_replicas_stay_bit_identical_under_lossy_compression(orc, mode):
    # every worker steps on the same compressed bytes (Alg. 1: same w[0],
    # deterministic staleness), so the p models never drift apart.
    p, n = 4, 4096 * 4 + 321
    wstar = W.gaussian(n, 1.0, 47)
    noise = [W.gaussian(n, 0.05, 49, (0, r, 0, 0)) for r in range(p)]
    ws, vs = orc.pipe_sgd_run(mode, lambda r, w, t: (w - wstar + noise[r]).astype(F),
                              np.zeros(n, F), p, 6, 0.01, momentum=0.9, width=2)
    for r in range(1, p):
        assert np.array_equal(ws[r], ws[0]) and np.array_equal(vs[r], vs[0])
    # and it still descends
    assert np.linalg.norm(ws[0] - wstar) < np.linalg.norm(wstar)
