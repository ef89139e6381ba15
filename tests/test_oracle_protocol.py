"""Pins of the CPU oracle's protocol side (timestamps, staleness, vector clocks,
trigger, rejection) against what the paper fixes: printed values, worked traces
computed by hand from its definitions, brute force, and invariants."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import OraclePS
from synth import replay as sreplay
from synth import trace as strace

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- c = floor(lambda/n)
def test_c_values_printed_by_the_paper():
    for lam, n, c in _lines("softsync_c_values.txt"):
        assert oracle.gradients_per_update(int(lam), int(n)) == int(c)


@pytest.mark.parametrize("lam", [1, 2, 7, 18, 30, 54])
def test_c_closed_form(lam):
    for n in range(1, lam + 1):
        assert oracle.gradients_per_update(lam, n) == lam // n
    assert oracle.gradients_per_update(lam, 1, oracle.HARDSYNC) == lam  # Eq. 3 averages all lambda
    assert oracle.gradients_per_update(30, 4) == 7  # floor, not round
    assert oracle.gradients_per_update(30, 4, c_override=8) == 8


# ---------------------------------------------------------------- worked traces
def _parse_traces():
    traces, cur = {}, None
    for tok in _lines("worked_traces.txt"):
        if tok[0] == "trace":
            cur = dict(lam=int(tok[2]), n=int(tok[3]), m=float(tok[4]), pushes=[], clocks=[])
            traces[tok[1]] = cur
        elif tok[0] == "push":
            cur["pushes"].append(dict(learner=int(tok[1]), g=float(tok[2]), ts=int(tok[3]), sigma=int(tok[4]),
                                      applied=int(tok[5]), ts_after=int(tok[6]),
                                      theta=None if tok[7] == "-" else float(tok[7])))
        elif tok[0] == "clock":
            cur["clocks"].append((int(tok[1]), float(tok[2]), [int(t) for t in tok[3:]]))
    return traces


@pytest.mark.parametrize("name", ["A", "B", "C", "D", "E"])
@pytest.mark.parametrize("precision", [32, 64])
def test_worked_trace(name, precision):
    t = _parse_traces()[name]
    ps = OraclePS(np.zeros(1, np.float32), t["lam"], t["n"], oracle.SOFTSYNC, oracle.LR_AVG_STALENESS,
                  alpha0=0.5, momentum=t["m"], precision=precision)
    learner_ts = [0] * t["lam"]
    for p in t["pushes"]:
        l = p["learner"]
        assert learner_ts[l] == p["ts"], "the learner's pulled timestamp differs from the hand trace"
        rc, r = ps.push(np.array([p["g"]], np.float32), learner_ts[l], l)
        assert rc == 0
        assert (r.staleness, r.applied, r.ts_after) == (p["sigma"], p["applied"], p["ts_after"])
        if p["applied"]:
            assert ps.theta[0] == p["theta"]  # dyadic numbers: exact in both precisions
        learner_ts[l] = ps.pull(False)[1]
    clocks, avg = ps.clocks, ps.avg_staleness
    for idx, sig, stamps in t["clocks"]:
        assert list(clocks[idx]) == stamps
        assert avg[idx] == sig


# ---------------------------------------------------------------- brute force from the log
def _run_softsync(lam, n, n_pushes, seed=11, c_override=0, jitter=None, straggler_prob=0.0):
    learner, step = strace.softsync_trace(seed, lam, n_pushes, straggler_prob=straggler_prob, jitter=jitter)
    ps = OraclePS(np.zeros(3, np.float32), lam, n, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=0.01,
                  c_override=c_override)

    class S:
        def push(self, l, s, ts):
            rc, r = ps.push(np.full(3, 1e-3, np.float32), ts, l)
            return rc, int(r.staleness), int(r.applied)

        def pull_ts(self):
            return ps.ts

    log = sreplay.replay(S(), learner, step, lam)
    return ps, log, learner


@pytest.mark.parametrize("lam,n", [(4, 1), (30, 1), (30, 2), (30, 4), (30, 30), (18, 1), (54, 54), (5, 3)])
def test_staleness_and_clocks_by_brute_force(lam, n):
    n_pushes = 700
    ps, log, learner = _run_softsync(lam, n, n_pushes)
    c = lam // n
    # recount everything from the arrival order alone, with the definitions of Sec. 3.1
    updates_before = np.arange(n_pushes) // c             # weight timestamp j when push i arrives
    assert np.array_equal(log["ts_at_arrival"], updates_before)
    assert np.array_equal(log["staleness"], updates_before - log["ts_pushed"])   # sigma = j - i
    assert np.array_equal(log["applied"], (np.arange(n_pushes) % c == c - 1).astype(np.int64))
    assert ps.ts == n_pushes // c == ps.n_updates          # starts at 0, +1 per update
    assert ps.pending == n_pushes % c                      # leftovers stay pending, unapplied
    assert ps.n_pushes == n_pushes
    # vector clock of update i (advancing ts_{i-1} -> ts_i): the c stamps that triggered it,
    # all < i, and <sigma> = (i-1) - mean(stamps)   (Eq. 2), as an exact rational
    clocks, avg = ps.clocks, ps.avg_staleness
    for u in range(ps.n_updates):
        stamps = log["ts_pushed"][u * c:(u + 1) * c]
        assert np.array_equal(clocks[u].astype(np.int64), stamps)
        i = u + 1
        assert stamps.max() < i
        exact = Fraction(i - 1) - Fraction(int(stamps.sum()), c)
        assert avg[u] == float(exact) or abs(avg[u] - float(exact)) <= 1e-15 * max(1.0, float(exact))
    # histogram and counters
    hist = np.bincount(log["staleness"])
    assert np.array_equal(ps.hist.astype(np.int64), hist)
    assert ps.sigma_sum == int(log["staleness"].sum())
    assert ps.sigma_max == int(log["staleness"].max())
    # rate log: alpha0 / max(1, <sigma>) rounded once to binary32
    want = np.array([np.float32(float(np.float32(0.01)) / max(1.0, a)) for a in avg], np.float32)
    assert np.array_equal(ps.lr_log, want)


@pytest.mark.parametrize("lam,c", [(30, 30), (30, 15), (30, 7), (30, 1), (54, 1)])
def test_staleness_conservation_law(lam, c):
    """With 'pull right after your push': every update adds one unit of pending staleness to each
    of the lambda-1 learners still computing, and a push turns pending staleness into recorded
    staleness; hence  sum(recorded sigma) + sum_l (ts_cur - ts_l) = (lambda-1) * ts_cur."""
    n_pushes = 1500
    learner, step = strace.softsync_trace(5, lam, n_pushes, straggler_prob=0.1)
    ps = OraclePS(np.zeros(1, np.float32), lam, 1, oracle.SOFTSYNC, oracle.LR_CONST, c_override=c)
    learner_ts = np.zeros(lam, np.int64)
    for i in range(n_pushes):
        l = learner[i]
        rc, r = ps.push(np.zeros(1, np.float32), learner_ts[l], l)
        assert rc == 0
        learner_ts[l] = ps.ts
        assert ps.sigma_sum + int((ps.ts - learner_ts).sum()) == (lam - 1) * ps.ts


def test_long_run_mean_staleness_is_about_n():
    """Sec. 5.1: <sigma> stays close to n for n-softsync (lambda = 30: ~1 for n=1, ~2 for n=2).
    Exact long-run value under the pull-after-push learner is (lambda-1)/c."""
    for n, c in [(1, 30), (2, 15), (30, 1)]:
        ps, log, _ = _run_softsync(30, n, 12000, seed=3)
        mean = log["staleness"][3000:].mean()
        assert abs(mean - 29.0 / c) < 0.05 * 29.0 / c + 0.02
        assert abs(mean - n) < 0.08 * n


def test_homogeneous_cluster_staleness_bound():
    """Sec. 5.1: in a homogeneous cluster 1-softsync sigma is in {0,1,2}, 2-softsync in {0..4},
    and lambda-softsync rarely exceeds 2n.  Learner durations 1 +- 5 % reproduce that."""
    for n, bound in [(1, 2), (2, 4), (30, 60)]:
        ps, log, _ = _run_softsync(30, n, 6000, seed=9, jitter=0.05)
        assert log["staleness"].max() <= bound
    ps, log, _ = _run_softsync(30, 30, 6000, seed=9, jitter=0.05)
    assert abs(np.median(log["staleness"][600:]) - 29) <= 1   # "a large fraction close to 30"


# ---------------------------------------------------------------- hardsync
def test_hardsync_staleness_is_always_zero_and_is_a_barrier():
    lam, rounds = 6, 20
    learner, step = strace.hardsync_trace(2, lam, rounds)
    ps = OraclePS(np.zeros(2, np.float32), lam, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.1)

    class S:
        def push(self, l, s, ts):
            rc, r = ps.push(np.ones(2, np.float32), ts, l)
            return rc, int(r.staleness), int(r.applied)

        def pull_ts(self):
            return ps.ts

    log = sreplay.replay(S(), learner, step, lam, hardsync=True)
    assert not log["staleness"].any()
    assert ps.ts == rounds and ps.pending == 0
    assert not ps.avg_staleness.any()
    assert np.array_equal(ps.hist, [lam * rounds])
    for r in range(rounds):   # each learner exactly once per step
        assert sorted(learner[r * lam:(r + 1) * lam]) == list(range(lam))


def test_rejections_change_nothing():
    g = np.ones(4, np.float32)
    ps = OraclePS(np.zeros(4, np.float32), 3, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.5)
    assert ps.push(g, 1, 0)[0] == oracle.EFUTURE_TS               # a gradient cannot come from the future
    assert ps.push(g, 0, 3)[0] == oracle.EINVAL                   # no such learner
    assert ps.push(g, 0, 0)[0] == 0
    assert ps.push(g, 0, 0)[0] == oracle.EHARDSYNC_DUP            # a learner contributes once per step
    assert ps.push(g, 0, 1)[0] == 0
    assert ps.pending == 2 and ps.n_pushes == 2 and ps.n_rejected == 3
    rc, r = ps.push(g, 0, 2)
    assert rc == 0 and r.applied == 1 and ps.ts == 1
    assert ps.push(g, 0, 0)[0] == oracle.EHARDSYNC_STALE          # staleness must be zero under hardsync
    assert ps.push(g, 1, 0)[0] == 0                               # learner 0 may contribute again in the new step
    assert np.array_equal(ps.theta, np.full(4, -0.5, np.float32))
    soft = OraclePS(np.zeros(4, np.float32), 3, 3, oracle.SOFTSYNC)
    assert soft.push(g, 5, 0)[0] == oracle.EFUTURE_TS and soft.n_updates == 0 and soft.pending == 0
    for bad in (dict(n_learners=0), dict(n_learners=3, n_split=4), dict(n_learners=3, n_split=0)):
        with pytest.raises(oracle.OracleError):
            OraclePS(np.zeros(1, np.float32), protocol=oracle.SOFTSYNC, **bad)


def test_single_learner_softsync_degenerates_to_hardsync():
    """Caption of the (sigma, mu, lambda) trade-off figure: for lambda = 1 softsync is hardsync."""
    rng = np.random.default_rng(0)
    w0 = rng.standard_normal(50).astype(np.float32)
    soft = OraclePS(w0, 1, 1, oracle.SOFTSYNC, oracle.LR_AVG_STALENESS, alpha0=0.1, momentum=0.9)
    hard = OraclePS(w0, 1, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.1, momentum=0.9)
    for i in range(40):
        g = rng.standard_normal(50).astype(np.float32)
        (_, a), (_, b) = soft.push(g, soft.ts, 0), hard.push(g, hard.ts, 0)
        assert a.staleness == b.staleness == 0 and a.applied == b.applied == 1
    assert np.array_equal(soft.theta, hard.theta) and soft.ts == hard.ts == 40


def test_pull_returns_weights_and_their_timestamp():
    ps = OraclePS(np.arange(4, dtype=np.float32), 2, 2, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=1.0)
    w, ts = ps.pull()
    assert ts == 0 and np.array_equal(w, np.arange(4, dtype=np.float32))
    assert ps.pull(False) == (None, 0)           # timestamp inquiry only
    ps.push(np.ones(4, np.float32), 0, 0)
    w, ts = ps.pull()
    assert ts == 1 and np.array_equal(w, np.arange(4, dtype=np.float32) - 1)
