"""Pins of the CPU oracle's arithmetic (sumGradients + applyUpdate) against things
other than itself: a library SGD routine, closed forms, unrolled sums, exact
rational arithmetic, and the binary64 build as a bound on binary32 rounding."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import OraclePS


def _rng(seed=0):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- hardsync == SGD on the mean gradient
@pytest.mark.parametrize("momentum,wd", [(0.0, 0.0), (0.9, 0.0), (0.9, 5e-4), (0.0, 5e-4)])
def test_hardsync_equals_library_sgd_on_the_averaged_gradient(momentum, wd):
    """Eq. 3 and the mu*lambda = const argument (Sec. 5.3): a hardsync step with lambda learners
    is one SGD step on the mean of their gradients.  torch.optim.SGD (rate outside the velocity,
    dampening 0) is algebraically the same recursion when the rate is constant."""
    rng = _rng(1)
    P, lam, steps, lr = 257, 5, 25, 0.05
    w0 = (0.1 * rng.standard_normal(P)).astype(np.float32)
    grads = (0.01 * rng.standard_normal((steps, lam, P))).astype(np.float32)
    ps64 = OraclePS(w0, lam, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=lr, momentum=momentum,
                    weight_decay=wd, precision=64)
    ps32 = OraclePS(w0, lam, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=lr, momentum=momentum,
                    weight_decay=wd, precision=32)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    # the oracle's hyper-parameters are binary32 numbers; give the library routine the same values
    opt = torch.optim.SGD([p], lr=float(np.float32(lr)), momentum=float(np.float32(momentum)),
                          weight_decay=float(np.float32(wd)))
    for s in range(steps):
        for l in range(lam):
            for ps in (ps64, ps32):
                rc, r = ps.push(grads[s, l], s, l)
                assert rc == 0 and r.staleness == 0
        p.grad = torch.tensor(grads[s].astype(np.float64).mean(axis=0))
        opt.step()
    ref = p.detach().numpy()
    scale = np.abs(ref).max()
    assert np.abs(ps64.theta - ref).max() <= 1e-12 * scale
    assert np.abs(ps32.theta.astype(np.float64) - ref).max() <= 2e-6 * scale   # binary32 rounding only
    assert ps64.ts == steps


def test_mu_lambda_equivalence():
    """Sec. 5.3: (sigma, mu, lambda) = (0, mu0*lambda0, 1) and (0, mu0, lambda0) are the same SGD: one learner
    pushing the mean of lambda gradients equals lambda learners pushing one each."""
    rng = _rng(2)
    P, lam, steps = 64, 8, 10   # lambda a power of two: the mean is exact in binary64
    w0 = rng.standard_normal(P).astype(np.float32)
    many = OraclePS(w0, lam, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.1, momentum=0.9, precision=64)
    one = OraclePS(w0, 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.1, momentum=0.9, precision=64)
    for s in range(steps):
        g = rng.integers(-8, 8, size=(lam, P)).astype(np.float32)
        for l in range(lam):
            many.push(g[l], s, l)
        one.push(g.mean(axis=0).astype(np.float32), s, 0)
    assert np.abs(many.theta - one.theta).max() <= 1e-13 * np.abs(one.theta).max()


# ---------------------------------------------------------------- lambda-softsync == per-gradient (async) updates
def test_c_equal_one_is_a_loop_of_single_gradient_steps():
    """n = lambda: the update rule is the Async one (Eq. 4), one step per gradient, here with the
    rate alpha0/max(1, sigma_i).  Without momentum theta_end = theta_0 - sum_i alpha_i g_i."""
    rng = _rng(3)
    lam, P, n_pushes, a0 = 6, 33, 120, 0.25
    w0 = rng.standard_normal(P).astype(np.float32)
    ps = OraclePS(w0, lam, lam, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=a0, precision=64)
    learner_ts = np.zeros(lam, np.int64)
    total = np.zeros(P, np.float64)
    for i in range(n_pushes):
        l = int(rng.integers(lam))
        g = rng.standard_normal(P).astype(np.float32)
        sigma = i - learner_ts[l]                    # i updates so far: brute-force staleness
        rc, r = ps.push(g, learner_ts[l], l)
        assert rc == 0 and r.applied == 1 and r.staleness == sigma
        total += (a0 / max(1, sigma)) * g.astype(np.float64)
        learner_ts[l] = i + 1
    assert np.abs(ps.theta - (w0.astype(np.float64) - total)).max() <= 1e-12 * np.abs(total).max()


def test_momentum_with_changing_rate_matches_the_unrolled_sum():
    """v_u = -sum_{j<=u} m^(u-j) alpha_j gbar_j and theta_u = theta_0 + sum_{t<=u} v_t: the recursion
    unrolled.  Distinguishes 'rate inside the velocity' from 'rate outside' because alpha_j varies."""
    rng = _rng(4)
    lam, P, a0, m = 4, 9, 0.5, 0.9
    ps = OraclePS(np.zeros(P, np.float32), lam, lam, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=a0,
                  momentum=m, precision=64)
    m = float(np.float32(m))
    stamps = [0, 0, 0, 0, 1, 2, 3, 4, 8, 2, 10, 11]   # staleness 0,1,2,3,3,3,3,3,0,7,0,0
    alphas, grads = [], []
    for i, ts in enumerate(stamps):
        g = rng.standard_normal(P).astype(np.float32)
        rc, r = ps.push(g, ts, -1)
        assert rc == 0 and r.staleness == i - ts
        alphas.append(a0 / max(1, i - ts))
        grads.append(g.astype(np.float64))
    assert len(set(alphas)) > 3
    U = len(stamps)
    v = [-sum(m ** (u - j) * alphas[j] * grads[j] for j in range(u + 1)) for u in range(U)]
    theta = sum(v)
    assert np.abs(ps.velocity - v[-1]).max() <= 1e-13
    assert np.abs(ps.theta - theta).max() <= 1e-12


# ---------------------------------------------------------------- closed forms
def test_constant_gradient_closed_forms():
    P = 5
    ones = np.ones(P, np.float32)
    # no momentum: theta_u = 1 - u*alpha (dyadic: exact in binary32)
    ps = OraclePS(ones, 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=2.0 ** -6)
    for u in range(40):
        ps.push(ones, u, 0)
    assert np.array_equal(ps.theta, np.full(P, 1 - 40 * 2.0 ** -6, np.float32))
    # momentum: v_u = -alpha (1 - m^u)/(1 - m);  theta_u = 1 - alpha/(1-m) * (u - m (1-m^u)/(1-m))
    a, m, U = 0.01, 0.9, 60
    ps = OraclePS(ones, 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=a, momentum=m, precision=64)
    for u in range(U):
        ps.push(ones, u, 0)
    a, m = float(np.float32(a)), float(np.float32(m))
    v_closed = -a * (1 - m ** U) / (1 - m)
    th_closed = 1 - a / (1 - m) * (U - m * (1 - m ** U) / (1 - m))
    assert abs(ps.velocity[0] - v_closed) <= 1e-14
    assert abs(ps.theta[0] - th_closed) <= 1e-13
    # zero gradients, weight penalty only: theta_u = theta_0 (1 - alpha*wd)^u
    a, wd, U = 0.5, 0.25, 30
    ps = OraclePS(ones, 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=a, weight_decay=wd, precision=64)
    for u in range(U):
        ps.push(np.zeros(P, np.float32), u, 0)
    assert abs(ps.theta[0] - (1 - a * wd) ** U) <= 1e-15


def test_average_uses_arrival_order_and_one_over_c():
    """The binary32 sum is sequential in arrival order and the mean is sum * fl(1/c): checked with
    exact rational arithmetic rounded step by step through numpy's binary32 scalars."""
    rng = _rng(5)
    c, P = 7, 64
    g = (rng.standard_normal((c, P)) * 10.0 ** rng.integers(-3, 3, size=(c, P))).astype(np.float32)
    ps = OraclePS(np.zeros(P, np.float32), c, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=1.0)
    for l in range(c):
        ps.push(g[l], 0, l)
    inv_c = np.float32(1.0) / np.float32(c)
    for k in range(P):
        s = Fraction(float(g[0, k]))
        for l in range(1, c):
            s = Fraction(float(np.float32(float(s + Fraction(float(g[l, k]))))))   # round to nearest binary32
        want = -np.float32(float(s * Fraction(float(inv_c))))
        assert ps.theta[k] == want
    # a different arrival order gives (somewhere) different bits: the order is part of the definition
    ps2 = OraclePS(np.zeros(P, np.float32), c, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=1.0)
    for l in reversed(range(c)):
        ps2.push(g[l], 0, l)
    assert np.abs(ps2.theta - ps.theta).max() <= 1e-6 * np.abs(ps.theta).max()
    assert not np.array_equal(ps2.theta, ps.theta)


def test_binary32_ops_are_rounded_one_by_one():
    """No fused multiply-add and no reassociation in the binary32 build: every element equals the same
    steps done with numpy binary32 scalars (each numpy scalar op rounds once)."""
    rng = _rng(6)
    P = 200
    f = np.float32
    w0 = rng.standard_normal(P).astype(f)
    g1, g2 = rng.standard_normal(P).astype(f), rng.standard_normal(P).astype(f)
    lr, m, wd = f(0.37), f(0.9), f(5e-4)
    ps = OraclePS(w0, 2, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=lr, momentum=m, weight_decay=wd)
    v = np.zeros(P, f)
    th = w0.copy()
    for rep in range(3):
        ps.push(g1, rep, 0)
        ps.push(g2, rep, 1)
        gbar = (g1 + g2) * (f(1) / f(2))
        gbar = gbar + wd * th
        v = m * v - lr * gbar
        th = th + v
    assert th.dtype == f and np.array_equal(ps.theta, th) and np.array_equal(ps.velocity, v)


def test_per_gradient_modulation():
    """Sec. 5.1 footnote: staler gradients get smaller rates.  theta_end = theta_0 - alpha0/c * sum_l g_l/max(1,sigma_l)."""
    P, lam = 4, 3
    ps = OraclePS(np.zeros(P, np.float32), lam, 1, oracle.SOFTSYNC, oracle.LR_PER_GRADIENT, alpha0=0.75, precision=64)
    one = np.ones(P, np.float32)
    for l in range(lam):
        ps.push(one, 0, l)            # update 1: sigma 0,0,0 -> theta = -0.75
    ps.push(one, 0, 0)                # sigma 1 -> weight 1
    ps.push(one, 1, 1)                # sigma 0 -> weight 1
    ps.push(one, 1, 2)
    for l in range(lam):
        ps.push(one, 2, l)            # update 3: now ts_cur = 2
    ps.push(4 * one, 0, 0)            # sigma 3 -> weight 1/3
    ps.push(2 * one, 1, 1)            # sigma 2 -> weight 1/2
    ps.push(one, 3, 2)                # sigma 0
    want = -0.75 * 3 - 0.75 / 3 * (4 / 3 + 1 + 1)
    assert abs(ps.theta[0] - want) <= 1e-15
    assert np.array_equal(ps.lr_log, np.full(4, 0.75, np.float32))


def test_static_n_rate_and_lr_scale():
    """alpha = alpha0/n (Eq. 6) and the hardsync factor sqrt(lambda*mu/B) handed in as lr_scale (Sec. 3.2)."""
    one = np.ones(1, np.float32)
    ps = OraclePS(np.zeros(1, np.float32), 8, 4, oracle.SOFTSYNC, oracle.LR_STATIC_N, alpha0=1.0, precision=64)
    ps.push(one, 0, 0)
    ps.push(one, 0, 1)
    assert ps.theta[0] == -0.25
    scale = float(np.float32(np.sqrt(30 * 4 / 128)))
    ps = OraclePS(np.zeros(1, np.float32), 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.5, lr_scale=scale, precision=64)
    ps.push(one, 0, 0)
    assert ps.theta[0] == -0.5 * scale
    ps.set_alpha0(0.05)              # rate schedule hook (Sec. 4.2: alpha0 divided by 10 at given epochs)
    ps.push(one, 1, 0)
    assert abs(ps.theta[0] + 0.5 * scale + float(np.float32(0.05)) * scale) <= 1e-16


def test_binary32_drift_from_binary64_is_far_below_the_parity_tolerance():
    """Bounds legitimate binary32 rounding on a long lambda-softsync run: the 1e-5*||theta||_inf parity budget
    is not consumed by it."""
    from oracle.adapter import OracleServer
    from synth import configs, replay
    w = configs.C5.scaled(n_params=4096, n_pushes=2000)
    learner, step = w.arrival_trace()
    s32, s64 = OracleServer(w, precision=32), OracleServer(w, precision=64)
    replay.replay(s32, learner, step, w.n_learners)
    replay.replay(s64, learner, step, w.n_learners)
    t64 = s64.ps.theta
    drift = np.abs(s32.ps.theta.astype(np.float64) - t64).max() / np.abs(t64).max()
    assert drift < 2e-6
    assert s32.ps.ts == s64.ps.ts == 2000
    assert np.array_equal(s32.ps.lr_log, s64.ps.lr_log)


def test_norms():
    ps = OraclePS(np.full(1000, 2.0, np.float32), 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.5, momentum=0.5)
    ps.push(np.full(1000, 4.0, np.float32), 0, 0)     # gbar 4, v = -2, theta = 0
    ps.push(np.full(1000, 2.0, np.float32), 1, 0)     # gbar 2, v = -1 - 1 = -2, theta = -2
    n = ps.norms()
    assert n == dict(theta_sq=4000.0, theta_inf=2.0, v_sq=4000.0, gbar_sq=4000.0)


def test_norms_of_a_random_state_with_weight_penalty():
    """Non-constant vectors, momentum and a weight penalty: the norms against sums written out here in numpy binary64
    from the definitions.  ||gbar||^2 is taken of the averaged gradient AS THE RATE MULTIPLIES IT, i.e. with the
    penalty term wd*theta (of the weights before the update) already added: that is the reading, and the variant
    without the penalty differs by far more than the tolerance on this input."""
    rng = _rng(21)
    P, lam, wd, m, lr = 3001, 3, 0.25, 0.5, 0.125
    w0 = rng.standard_normal(P).astype(np.float32)
    ps = OraclePS(w0, lam, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=lr, momentum=m, weight_decay=wd)
    for step in range(3):
        gs = (0.5 * rng.standard_normal((lam, P))).astype(np.float32)
        if step == 2:                  # the latest update: its averaged gradient from the weights just before it
            before = ps.theta.astype(np.float64)
            mean = ((gs[0] + gs[1]) + gs[2]) * (np.float32(1) / np.float32(3))
            gbar_with = mean.astype(np.float64) + wd * before
            gbar_without = mean.astype(np.float64)
        for l in range(lam):
            assert ps.push(gs[l], step, l)[0] == 0
    assert ps.ts == 3
    n = ps.norms()
    th, ve = ps.theta.astype(np.float64), ps.velocity.astype(np.float64)
    assert n["theta_sq"] == pytest.approx(float(np.sum(th * th)), rel=1e-12)
    assert n["v_sq"] == pytest.approx(float(np.sum(ve * ve)), rel=1e-12)
    assert n["theta_inf"] == float(np.abs(th).max())
    assert n["gbar_sq"] == pytest.approx(float(np.sum(gbar_with * gbar_with)), rel=1e-6)      # binary32 rounding of gbar itself
    assert abs(n["gbar_sq"] - float(np.sum(gbar_without * gbar_without))) > 0.05 * n["gbar_sq"]


# ---------------------------------------------------------------- AdaGrad (named for the ImageNet 1-softsync runs, Sec. 5.5)
@pytest.mark.parametrize("wd", [0.0, 5e-4])
def test_adagrad_equals_library_adagrad_on_the_averaged_gradient(wd):
    """The cited diagonal AdaGrad rule: torch.optim.Adagrad (no rate decay, accumulator from 0) in binary64 on the
    mean gradient of each hardsync step."""
    rng = _rng(7)
    P, lam, steps, lr, eps = 129, 4, 30, 0.05, 1e-6
    w0 = (0.1 * rng.standard_normal(P)).astype(np.float32)
    grads = (0.01 * rng.standard_normal((steps, lam, P))).astype(np.float32)
    kw = dict(alpha0=lr, weight_decay=wd, optimizer=oracle.OPT_ADAGRAD, adagrad_eps=eps)
    ps64 = OraclePS(w0, lam, 1, oracle.HARDSYNC, oracle.LR_CONST, precision=64, **kw)
    ps32 = OraclePS(w0, lam, 1, oracle.HARDSYNC, oracle.LR_CONST, precision=32, **kw)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adagrad([p], lr=float(np.float32(lr)), weight_decay=float(np.float32(wd)), eps=float(np.float32(eps)),
                              lr_decay=0.0, initial_accumulator_value=0.0)
    for s in range(steps):
        for l in range(lam):
            ps64.push(grads[s, l], s, l)
            ps32.push(grads[s, l], s, l)
        p.grad = torch.tensor(grads[s].astype(np.float64).mean(axis=0))
        opt.step()
    ref = p.detach().numpy()
    assert np.abs(ps64.theta - ref).max() <= 1e-12 * np.abs(ref).max()
    assert np.abs(ps32.theta.astype(np.float64) - ref).max() <= 2e-6 * np.abs(ref).max()
    h_ref = opt.state[p]["sum"].numpy()
    assert np.abs(ps64.velocity - h_ref).max() <= 1e-13 * h_ref.max()       # the accumulator lives in the second state vector


def test_adagrad_closed_form_and_staleness_modulated_rate():
    """Constant gradient g: h_u = u g^2 and theta_u = theta_0 - sum_j alpha_j g / (sqrt(j) |g| + eps); the rate alpha_j is
    still alpha0 / max(1, sigma_j)."""
    g, a0, eps = 0.25, 0.5, 1e-3
    ps = OraclePS(np.zeros(3, np.float32), 4, 4, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=a0,
                  optimizer=oracle.OPT_ADAGRAD, adagrad_eps=eps, precision=64)
    stamps = [0, 0, 0, 2, 4, 1, 6]               # staleness 0,1,2,1,0,4,0
    want = 0.0
    for j, ts in enumerate(stamps, start=1):
        rc, r = ps.push(np.full(3, g, np.float32), ts, -1)
        assert rc == 0 and r.staleness == (j - 1) - ts
        want -= (a0 / max(1, (j - 1) - ts)) * g / (np.sqrt(j) * g + float(np.float32(eps)))
    assert abs(ps.theta[0] - want) <= 1e-14
    assert abs(ps.velocity[0] - len(stamps) * g * g) <= 1e-15
    with pytest.raises(oracle.OracleError):      # AdaGrad replaces momentum here, it does not combine with it
        OraclePS(np.zeros(1, np.float32), 1, 1, oracle.HARDSYNC, optimizer=oracle.OPT_ADAGRAD, momentum=0.9)


def test_adagrad_binary32_ops_are_rounded_one_by_one():
    rng = _rng(8)
    f = np.float32
    P = 300
    w0 = rng.standard_normal(P).astype(f)
    g1, g2 = rng.standard_normal(P).astype(f), rng.standard_normal(P).astype(f)
    lr, wd, eps = f(0.11), f(5e-4), f(1e-8)
    ps = OraclePS(w0, 2, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=lr, weight_decay=wd, optimizer=oracle.OPT_ADAGRAD,
                  adagrad_eps=eps)
    h, th = np.zeros(P, f), w0.copy()
    for rep in range(4):
        ps.push(g1, rep, 0)
        ps.push(g2, rep, 1)
        gbar = (g1 + g2) * (f(1) / f(2))
        gbar = gbar + wd * th
        h = h + gbar * gbar
        th = th - (lr * gbar) / (np.sqrt(h) + eps)
    assert th.dtype == f and np.array_equal(ps.theta, th) and np.array_equal(ps.velocity, h)
