"""Pins of the oracle's parameter-server tree (Sec. 3.3: a node averages its learners' gradients and relays the
average; the root applies the update): special cases that reduce to the flat server, exact arithmetic on dyadic
numbers, a trace worked by hand, brute-force staleness from the constituents' timestamps."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import OraclePS, leaf_mean


def _rng(seed):
    return np.random.default_rng(seed)


def test_leaf_mean_is_a_sequential_binary32_sum_times_one_over_k():
    rng = _rng(0)
    k, n = 5, 40
    g = (rng.standard_normal((k, n)) * 10.0 ** rng.integers(-2, 3, size=(k, n))).astype(np.float32)
    out = leaf_mean(list(g))
    inv_k = np.float32(1) / np.float32(k)
    for i in range(n):
        s = Fraction(float(g[0, i]))
        for l in range(1, k):
            s = Fraction(float(np.float32(float(s + Fraction(float(g[l, i]))))))
        assert out[i] == np.float32(float(s * Fraction(float(inv_k))))
    assert np.abs(leaf_mean(list(g), precision=64) - g.astype(np.float64).mean(axis=0)).max() <= 1e-6 * np.abs(g).max()
    assert np.array_equal(leaf_mean([g[0]]), g[0])          # one learner: the message itself


def test_single_learner_leaves_equal_the_flat_server():
    """A tree whose nodes have one learner each relays every gradient unchanged: same bits as pushGradient."""
    rng = _rng(1)
    P, lam = 50, 6
    w0 = rng.standard_normal(P).astype(np.float32)
    kw = dict(alpha0=0.1, momentum=0.9, weight_decay=5e-4)
    flat = OraclePS(w0, lam, 2, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, **kw)
    tree = OraclePS(w0, lam, 2, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, max_aggregate=1, **kw)
    ts = np.zeros(lam, np.int64)
    for i in range(60):
        l = int(rng.integers(lam))
        g = rng.standard_normal(P).astype(np.float32)
        (rc1, a), (rc2, b) = flat.push(g, ts[l], l), tree.push_aggregate(leaf_mean([g]), [ts[l]])
        assert rc1 == rc2 == 0
        assert (a.staleness, a.ts_after, a.pending, a.applied, a.lr_used) == (b.staleness, b.ts_after, b.pending, b.applied, b.lr_used)
        ts[l] = flat.ts
    assert np.array_equal(flat.theta, tree.theta) and np.array_equal(flat.velocity, tree.velocity)
    assert np.array_equal(flat.clocks, tree.clocks) and np.array_equal(flat.hist, tree.hist)


@pytest.mark.parametrize("precision", [32, 64])
def test_tree_equals_flat_mean(precision):
    """lambda = 12 learners under 4 nodes of 3, 1-softsync: mathematically the root's mean of relayed averages is the flat
    mean of all 12 gradients.  Exact on small integers (every partial sum is representable); to rounding otherwise."""
    rng = _rng(2)
    P, lam, k = 30, 12, 3
    w0 = rng.integers(-4, 4, P).astype(np.float32)
    for exact in (True, False):
        flat = OraclePS(w0, lam, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=0.75, precision=precision)
        tree = OraclePS(w0, lam, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=0.75, max_aggregate=k, precision=precision)
        for step in range(5):
            g = (rng.integers(-64, 64, (lam, P)) * 3).astype(np.float32) if exact else rng.standard_normal((lam, P)).astype(np.float32)
            for l in range(lam):
                flat.push(g[l], step, l)
            for j in range(lam // k):
                rc, r = tree.push_aggregate(leaf_mean(list(g[j * k:(j + 1) * k]), precision), [step] * k)
                assert rc == 0 and r.applied == (j == lam // k - 1)
        assert flat.ts == tree.ts == 5
        if exact:
            assert np.array_equal(flat.theta, tree.theta)       # multiples of 3: every node average and partial sum is exact
        elif precision == 64:
            assert np.abs(flat.theta - tree.theta).max() <= 1e-6 * np.abs(flat.theta).max()   # the relayed message is binary32
        else:
            assert np.abs(flat.theta.astype(np.float64) - tree.theta).max() <= 1e-5 * np.abs(flat.theta).max()


def test_exact_tree_on_multiples_of_three():
    """Gradients that are multiples of 3*2^-6: every node average and every sum is exact, so tree == flat bit for bit."""
    rng = _rng(3)
    P, lam, k = 20, 12, 3
    flat = OraclePS(np.zeros(P, np.float32), lam, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=0.75, precision=64)
    tree = OraclePS(np.zeros(P, np.float32), lam, 1, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=0.75, max_aggregate=k, precision=64)
    for step in range(4):
        g = (rng.integers(-32, 32, (lam, P)) * 3).astype(np.float32) / 64
        for l in range(lam):
            flat.push(g[l], step, l)
        for j in range(lam // k):
            tree.push_aggregate(leaf_mean(list(g[j * k:(j + 1) * k]), 64), [step] * k)
    assert np.abs(flat.theta - tree.theta).max() <= 1e-15


def test_worked_trace_with_overshoot():
    """By hand.  lambda = 4, 1-softsync (c = 4), nodes of 3, alpha0 = 0.5, theta0 = 0, one parameter.
    Message 1: average 2.0 of three gradients stamped (0,0,0): count 3 < 4, no update.
    Message 2: average 4.0 of three gradients stamped (0,0,0): count 6 >= 4 -> update over SIX gradients:
      mean = (3*2 + 3*4)/6 = 3, <sigma> = 0, theta = -1.5, timestamp 1, clock of 6 zeros.
    Message 3: average 8.0 stamped (0,1,1): staleness 1,0,0; count 3.  Message 4: a single gradient 2.0 stamped 0
      (staleness 1): count 4 -> update: mean = (3*8 + 2)/4 = 6.5, <sigma> = (1+0+0+1)/4 = 0.5 -> divisor 1,
      theta = -1.5 - 3.25 = -4.75, timestamp 2, clock (0,1,1,0)."""
    for precision in (32, 64):
        ps = OraclePS(np.zeros(1, np.float32), 4, 1, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=0.5, max_aggregate=3,
                      precision=precision)
        rc, r = ps.push_aggregate([2.0], [0, 0, 0])
        assert (rc, r.applied, r.pending, r.ts_after) == (0, 0, 3, 0)
        rc, r = ps.push_aggregate([4.0], [0, 0, 0])
        assert (rc, r.applied, r.pending, r.ts_after, r.lr_used) == (0, 1, 0, 1, 0.5)
        assert ps.theta[0] == -1.5
        rc, r = ps.push_aggregate([8.0], [0, 1, 1])
        assert (rc, r.applied, r.pending, r.staleness) == (0, 0, 3, 1)
        rc, r = ps.push(np.array([2.0], np.float32), 0, 3)
        assert (rc, r.applied, r.ts_after, r.staleness) == (0, 1, 2, 1)
        assert ps.theta[0] == -4.75
        clocks = ps.clocks
        assert [list(c) for c in clocks] == [[0, 0, 0, 0, 0, 0], [0, 1, 1, 0]]
        assert list(ps.avg_staleness) == [0.0, 0.5]
        assert list(ps.hist) == [8, 2] and ps.n_pushes == 10 and ps.sigma_sum == 2


def test_staleness_of_constituents_by_brute_force():
    rng = _rng(5)
    lam, k, c = 9, 3, 6
    ps = OraclePS(np.zeros(2, np.float32), lam, 1, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=0.01, c_override=c,
                  max_aggregate=k)
    stamps_all, arrivals = [], []
    for i in range(80):
        m = int(rng.integers(1, k + 1))
        ts = [max(0, ps.ts - int(rng.integers(0, 3))) for _ in range(m)]
        before = ps.ts
        rc, r = ps.push_aggregate(np.ones(2, np.float32), ts)
        assert rc == 0 and r.staleness == max(before - t for t in ts)
        stamps_all += ts
        arrivals += [before] * m
    sig = np.array(arrivals) - np.array(stamps_all)
    assert np.array_equal(ps.hist.astype(np.int64), np.bincount(sig))
    assert ps.sigma_sum == sig.sum() and ps.n_pushes == len(sig)
    pos = 0
    for u, clock in enumerate(ps.clocks if isinstance(ps.clocks, list) else list(ps.clocks)):
        n = len(clock)
        assert c <= n <= c + k - 1                                      # at least c, overshoot by at most one message
        assert list(clock) == stamps_all[pos:pos + n]
        exact = Fraction(u) - Fraction(int(sum(stamps_all[pos:pos + n])), n)     # (i-1) - mean(i_k), Eq. 2
        assert abs(ps.avg_staleness[u] - float(exact)) <= 1e-15 * max(1.0, float(exact))
        pos += n
    assert ps.pending == len(sig) - pos


def test_aggregate_rejections():
    g = np.ones(3, np.float32)
    ps = OraclePS(np.zeros(3, np.float32), 6, 1, oracle.SOFTSYNC, max_aggregate=3)
    assert ps.push_aggregate(g, [0, 0, 0, 0])[0] == oracle.EINVAL                 # larger than the declared fan-in
    assert ps.push_aggregate(g, [0, 1])[0] == oracle.EFUTURE_TS
    assert ps.push_aggregate(g, [])[0] == oracle.EINVAL
    assert ps.n_pushes == 0 and ps.pending == 0 and ps.n_rejected == 2
    hard = OraclePS(np.zeros(3, np.float32), 4, 1, oracle.HARDSYNC, oracle.LR_CONST, max_aggregate=2)
    assert hard.push_aggregate(g, [0, 0])[0] == 0 and hard.push_aggregate(g, [0, 0])[1].applied == 1
    assert hard.push_aggregate(g, [0, 1])[0] == oracle.EHARDSYNC_STALE
    per = OraclePS(np.zeros(3, np.float32), 4, 1, oracle.SOFTSYNC, oracle.LR_PER_GRADIENT, max_aggregate=2)
    assert per.push_aggregate(g, [0, 0])[0] == oracle.EINVAL                      # a relayed average cannot be re-weighted


def test_hardsync_step_under_a_tree_averages_exactly_lambda_gradients():
    """Eq. 3: a hardsync step is the mean of one gradient from each of the lambda learners.  With relayed averages of up
    to 3 gradients and lambda = 4, a second average of 3 would make 6: refused, nothing changes; the single gradient
    that completes the four is taken and the step is theta - alpha * (3*a + b)/4, all dyadic, exact in binary32."""
    ps = OraclePS(np.full(2, 8.0, np.float32), 4, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.5, max_aggregate=3)
    a, b = np.full(2, 2.0, np.float32), np.full(2, 10.0, np.float32)
    assert ps.push_aggregate(a, [0, 0, 0])[0] == oracle.OK
    rc, _ = ps.push_aggregate(a, [0, 0, 0])
    assert rc == oracle.EHARDSYNC_DUP and (ps.pending, ps.ts, ps.n_rejected) == (3, 0, 1)
    assert ps.push_aggregate(a, [0, 0])[0] == oracle.EHARDSYNC_DUP
    rc, r = ps.push_aggregate(b, [0])
    assert rc == oracle.OK and r.applied == 1 and ps.ts == 1
    assert np.array_equal(ps.theta, np.full(2, 8.0 - 0.5 * (3 * 2.0 + 10.0) / 4, np.float32))      # 8 - 2 = 6
    assert list(ps.clocks[0]) == [0, 0, 0, 0] and ps.n_pushes == 4
