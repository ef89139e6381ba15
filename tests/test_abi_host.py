"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, and its control plane (timestamps, staleness, clocks, rates, rejections; RUDRA_FLAG_CONTROL_ONLY:
no device work at all) agrees bit for bit with the CPU oracle on the workloads' arrival traces."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_1509_04210_amd as R
from oracle import OraclePS
from paper_1509_04210_amd import binding as B
from synth.learners import LR_MODE, PROTOCOL
from synth import configs, replay

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "rudra_ps.h")).read()
    declared = set(re.findall(r"\b(rudra_ps_[a-z_]+)\s*\(", header))
    assert {"rudra_ps_create", "rudra_ps_push_gradient", "rudra_ps_pull_weights", "rudra_ps_stats"} <= declared
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/rudra_ps.h but not exported"
    assert len(declared) >= 18


def test_struct_layouts_match_the_header():
    """Field order of the ctypes mirrors == field order in the header (a transposed field would shift everything)."""
    header = open(os.path.join(ROOT, "include", "rudra_ps.h")).read()

    def fields(struct_name):
        body = re.search(r"typedef struct \{([^}]*)\} " + struct_name + ";", header).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        names = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            names += [n.strip().lstrip("*").strip() for n in decl.split(None, 1)[1].split(",")]
        return names

    assert fields("rudra_ps_config_t") == [f[0] for f in B.Config._fields_]
    assert fields("rudra_push_result_t") == [f[0] for f in B.PushResult._fields_]
    assert fields("rudra_ps_stats_t") == [f[0] for f in B.Stats._fields_]


def test_strerror_and_null_arguments():
    assert R.strerror(0) == "ok"
    assert "newer" in R.strerror(B.EFUTURE_TS)
    L = R.lib()
    assert L.rudra_ps_create(None, None, None) == B.EINVAL
    assert L.rudra_ps_push_gradient(None, None, 0, 0, None) == B.EINVAL
    assert L.rudra_ps_destroy(None) == B.OK
    for bad in (dict(n_params=0, n_learners=1), dict(n_params=1, n_learners=0), dict(n_params=1, n_learners=3, n_split=4),
                dict(n_params=1, n_learners=3, n_split=0), dict(n_params=1, n_learners=3, launch_block=100),
                dict(n_params=1, n_learners=3, launch_unroll=3), dict(n_params=1, n_learners=3, launch_unroll=8, launch_vec=4),
                dict(n_params=1, n_learners=3, flags=1 << 20), dict(n_params=1, n_learners=3, optimizer=2),
                dict(n_params=1, n_learners=3, optimizer=B.OPT_ADAGRAD, momentum=0.9),
                dict(n_params=1, n_learners=3, optimizer=B.OPT_ADAGRAD, adagrad_eps=-1.0), dict(n_params=1, n_learners=3, launch_alternate=3),
                dict(n_params=1, n_learners=3, launch_waves_per_cu=1), dict(n_params=1, n_learners=3, alpha0=float("nan")),
                dict(n_params=1, n_learners=3, lr_scale=0.0),                                         # a zeroed config
                dict(n_params=1, n_learners=3, protocol=B.HARDSYNC, lr_mode=B.LR_STATIC_N, n_split=0),  # alpha0/0
                dict(n_params=1, n_learners=1 << 25),                                                 # clock of 2^25 entries
                dict(n_params=1, n_learners=1 << 20, clock_ring=1 << 10),                             # ring of 2^30 timestamps
                dict(n_params=1, n_learners=4, max_aggregate=4096, c_override=0xFFFFFFFF)):           # c + max_aggregate - 1 wraps in 32 bits
        with pytest.raises(R.RudraError) as e:
            R.ParameterServer(flags=bad.pop("flags", B.FLAG_CONTROL_ONLY), **bad)
        assert e.value.status == B.EINVAL


def test_rejections_mirror_the_oracle():
    ps = R.ParameterServer(4, 3, protocol=B.HARDSYNC, lr_mode=B.LR_CONST, alpha0=0.5, flags=B.FLAG_CONTROL_ONLY)
    ora = OraclePS(np.zeros(4, np.float32), 3, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.5)
    g = np.ones(4, np.float32)
    script = [(1, 0), (0, 3), (0, -2), (0, 0), (0, 0), (0, 1), (0, 2), (0, 0), (1, 0), (1, 1), (2, 1), (1, 2)]
    for ts, learner in script:
        rc_h, r = ps.push_gradient(0, ts, learner)
        rc_o, ro = ora.push(g, ts, learner)
        assert rc_h == rc_o, (ts, learner)
        if rc_h == 0:
            assert (r.staleness, r.ts_after, r.pending, r.applied, r.lr_used) == \
                   (ro.staleness, ro.ts_after, ro.pending, ro.applied, ro.lr_used)
    st = ps.stats()
    assert (st.n_pushes, st.n_updates, st.n_rejected, st.pending) == (ora.n_pushes, ora.n_updates, ora.n_rejected, ora.pending)
    assert st.n_rejected == 6 and st.ts_cur == 2
    with pytest.raises(R.RudraError) as e:      # no weights exist in control-only mode
        ps.pull_weights(0x1000)
    assert e.value.status == B.ESTATE


class _Control:
    def __init__(self, w, **kw):
        self.ps = R.ParameterServer(w.n_params, w.n_learners, 0, w.n_split, PROTOCOL[w.protocol], LR_MODE[w.lr_mode],
                                    w.alpha0, w.lr_scale, w.momentum, w.weight_decay, w.c_override,
                                    flags=B.FLAG_CONTROL_ONLY, optimizer=B.OPT_ADAGRAD if w.optimizer == "adagrad" else B.OPT_SGD,
                                    adagrad_eps=w.adagrad_eps, **kw)

    def push(self, l, s, ts):
        rc, r = self.ps.push_gradient(0, ts, l)
        return rc, r.staleness, r.applied

    def push_batch(self, msgs):
        rc, handled, res = self.ps.push_batch([0] * len(msgs), [ts for _, _, ts in msgs], [l for l, _, _ in msgs])
        return rc, handled, [r.staleness for r in res], [r.applied for r in res]

    def pull_ts(self):
        return self.ps.pull_weights(0)


class _OracleControl:
    """The oracle on a one-element vector: its protocol side does not depend on P."""

    def __init__(self, w):
        self.ps = OraclePS(np.zeros(1, np.float32), w.n_learners, w.n_split, oracle.HARDSYNC if w.protocol == "hardsync" else oracle.SOFTSYNC,
                           {"const": 0, "static_n": 1, "avg_staleness": 2, "per_gradient": 3}[w.lr_mode], w.alpha0,
                           w.lr_scale, w.momentum, w.weight_decay, w.c_override,
                           optimizer=oracle.OPT_ADAGRAD if w.optimizer == "adagrad" else oracle.OPT_SGD)
        self.g = np.zeros(1, np.float32)

    def push(self, l, s, ts):
        rc, r = self.ps.push(self.g, ts, l)
        return rc, int(r.staleness), int(r.applied)

    def push_batch(self, msgs):
        out = [self.push(l, s, ts) for l, s, ts in msgs]
        return 0, len(msgs), [o[1] for o in out], [o[2] for o in out]

    def pull_ts(self):
        return self.ps.ts


def _same_protocol_state(hip, ora):
    st, o = hip.ps.stats(), ora.ps
    assert (st.ts_cur, st.n_pushes, st.n_updates, st.pending, st.c) == (o.ts, o.n_pushes, o.n_updates, o.pending, o.c)
    assert (st.sigma_sum, st.sigma_max, st.n_rejected) == (o.sigma_sum, o.sigma_max, o.n_rejected)
    assert np.array_equal(np.array(hip.ps.staleness_hist(), np.uint64), o.hist)
    clocks, avg, lr = o.clocks, o.avg_staleness, o.lr_log
    for u in range(o.n_updates):
        ts, a, r = hip.ps.vector_clock(u)
        assert ts == list(clocks[u]) and a == avg[u] and np.float32(r) == lr[u]


@pytest.mark.parametrize("name", list(configs.ALL))
def test_batched_pushes_leave_the_protocol_state_of_single_pushes(name):
    """rudra_ps_push_batch == the same messages through the oracle one by one (control plane; chunks of 1..40)."""
    w = configs.ALL[name]
    n = min(w.n_pushes, 3000)
    learner, step = w.arrival_trace(n)
    chunks = np.random.default_rng(11).integers(1, 41, size=64)
    hard = w.protocol == "hardsync"
    hip, ora = _Control(w, clock_ring=8192), _OracleControl(w)
    lh = replay.replay_batched(hip, learner, step, w.n_learners, chunks, hardsync=hard, c=w.c)
    lo = replay.replay_batched(ora, learner, step, w.n_learners, chunks, hardsync=hard, c=w.c)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    _same_protocol_state(hip, ora)


def test_a_rejected_message_stops_the_batch_where_single_pushes_would_reject_it():
    ps = R.ParameterServer(4, 3, n_split=3, lr_mode=B.LR_CONST, alpha0=0.5, flags=B.FLAG_CONTROL_ONLY)      # c = 1
    ora = OraclePS(np.zeros(4, np.float32), 3, 3, oracle.SOFTSYNC, oracle.LR_CONST, alpha0=0.5)
    g = np.zeros(4, np.float32)
    ts, learners = [0, 1, 1, 9, 2, 0], [0, 1, 2, 0, 1, 7]            # message 3 comes from the future
    rc, handled, res = ps.push_batch([0] * 6, ts, learners)
    assert (rc, handled, len(res)) == (B.EFUTURE_TS, 3, 3)
    want = [ora.push(g, t, l) for t, l in zip(ts[:4], learners[:4])]
    assert [w[0] for w in want] == [0, 0, 0, oracle.EFUTURE_TS]
    for r, (_, ro) in zip(res, want):
        assert (r.staleness, r.ts_after, r.pending, r.applied, r.lr_used) == (ro.staleness, ro.ts_after, ro.pending, ro.applied, ro.lr_used)
    st = ps.stats()
    assert (st.ts_cur, st.n_pushes, st.n_rejected) == (3, 3, 1) == (ora.ts, ora.n_pushes, ora.n_rejected)
    rc, handled, res = ps.push_batch([0] * 2, ts[4:], learners[4:])    # the rest: message 5 names an unknown learner
    assert (rc, handled) == (B.EINVAL, 1) and ps.stats().ts_cur == 4
    assert ps.push_batch([], [], [])[:2] == (B.OK, 0)
    assert R.lib().rudra_ps_push_batch(None, None, None, None, 0, None, None) == B.EINVAL


@pytest.mark.parametrize("name", list(configs.ALL))
def test_control_plane_equals_oracle_on_every_workload_trace(name):
    w = configs.ALL[name]
    n = min(w.n_pushes, 6000)
    learner, step = w.arrival_trace(n)
    hip, ora = _Control(w, clock_ring=8192), _OracleControl(w)
    lh = replay.replay(hip, learner, step, w.n_learners, hardsync=w.protocol == "hardsync")
    lo = replay.replay(ora, learner, step, w.n_learners, hardsync=w.protocol == "hardsync")
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    st = hip.ps.stats()
    o = ora.ps
    assert (st.ts_cur, st.n_pushes, st.n_updates, st.pending, st.c) == (o.ts, o.n_pushes, o.n_updates, o.pending, o.c)
    assert (st.sigma_sum, st.sigma_max) == (o.sigma_sum, o.sigma_max)
    assert st.bytes_absorbed == o.n_pushes * 4 * w.n_params
    assert np.array_equal(np.array(hip.ps.staleness_hist(), np.uint64), o.hist)
    clocks, avg, lr = o.clocks, o.avg_staleness, o.lr_log
    for u in range(o.n_updates):
        ts, a, r = hip.ps.vector_clock(u)
        assert ts == list(clocks[u]) and a == avg[u] and np.float32(r) == lr[u]
    if o.n_updates:
        assert st.last_avg_staleness == avg[-1] and np.float32(st.last_lr) == lr[-1]
    with pytest.raises(R.RudraError):
        hip.ps.vector_clock(o.n_updates)          # has not happened yet


def test_clock_ring_evicts_old_updates():
    ps = R.ParameterServer(1, 2, n_split=2, flags=B.FLAG_CONTROL_ONLY, clock_ring=4)
    for i in range(10):
        ps.push_gradient(0, i, 0)
    assert ps.vector_clock(9)[0] == [9] and ps.vector_clock(6)[0] == [6]
    with pytest.raises(R.RudraError) as e:
        ps.vector_clock(5)
    assert e.value.status == B.ERANGE


def test_set_lr_changes_later_updates_only():
    ps = R.ParameterServer(1, 1, protocol=B.HARDSYNC, lr_mode=B.LR_CONST, alpha0=0.5, flags=B.FLAG_CONTROL_ONLY)
    assert ps.push_gradient(0, 0, 0)[1].lr_used == 0.5
    ps.set_lr(0.05)
    assert np.float32(ps.push_gradient(0, 1, 0)[1].lr_used) == np.float32(0.05)
    assert ps.vector_clock(0)[2] == 0.5


@pytest.mark.parametrize("lam,n", [(1000, 1), (1000, 16), (1000, 1000), (4097, 64)])
def test_many_learners(lam, n):
    """Learner counts far beyond the workloads' (c = 1000, 62, 1, 64): control plane against the oracle."""
    from dataclasses import replace
    w = replace(configs.C3(1), name="many", n_learners=lam, n_split=n, n_pushes=3 * lam + 17, straggler_prob=0.05)
    learner, step = w.arrival_trace()
    hip, ora = _Control(w, clock_ring=8192), _OracleControl(w)
    lh = replay.replay(hip, learner, step, w.n_learners)
    lo = replay.replay(ora, learner, step, w.n_learners)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    _same_protocol_state(hip, ora)
    assert hip.ps.stats().c == lam // n


def test_bad_rate_configurations_are_rejected_like_the_oracle_rejects_them():
    """alpha0/n with n = 0 under hardsync would be an infinite rate, and a factor of 0 a frozen model: both sides refuse."""
    for kw in (dict(protocol=oracle.HARDSYNC, lr_mode=oracle.LR_STATIC_N, n_split=0), dict(lr_scale=0.0)):
        with pytest.raises(oracle.OracleError) as e:
            OraclePS(np.zeros(1, np.float32), 3, **{"n_split": 1, **kw})
        assert e.value.code == oracle.EINVAL
    ps = R.ParameterServer(1, 3, protocol=B.HARDSYNC, lr_mode=B.LR_STATIC_N, n_split=2, alpha0=0.5, flags=B.FLAG_CONTROL_ONLY)
    ora = OraclePS(np.zeros(1, np.float32), 3, 2, oracle.HARDSYNC, oracle.LR_STATIC_N, alpha0=0.5)
    for l in range(3):
        rc, r = ps.push_gradient(0, 0, l)
        rco, ro = ora.push(np.zeros(1, np.float32), 0, l)
        assert rc == rco == 0 and r.lr_used == ro.lr_used
    assert r.applied == 1 and r.lr_used == 0.25


def test_hardsync_aggregate_cannot_overshoot_lambda():
    """Eq. 3 averages exactly lambda gradients: a relayed average that would carry the count past lambda is refused
    (the oracle refuses it the same way); one that completes the step exactly is taken."""
    ps = R.ParameterServer(1, 4, protocol=B.HARDSYNC, lr_mode=B.LR_CONST, alpha0=0.5, flags=B.FLAG_CONTROL_ONLY, max_aggregate=3)
    ora = OraclePS(np.zeros(1, np.float32), 4, 1, oracle.HARDSYNC, oracle.LR_CONST, alpha0=0.5, max_aggregate=3)
    g = np.ones(1, np.float32)
    for stamps, want in ([[0, 0, 0], B.OK], [[0, 0, 0], B.EHARDSYNC_DUP], [[0, 0], B.EHARDSYNC_DUP], [[0], B.OK], [[1, 1, 1], B.OK], [[1, 1], B.EHARDSYNC_DUP]):
        rc, r = ps.push_aggregate(0, stamps)
        rco, ro = ora.push_aggregate(g, stamps)
        assert rc == rco == want, stamps
        if rc == 0:
            assert (r.ts_after, r.pending, r.applied) == (ro.ts_after, ro.pending, ro.applied)
    st = ps.stats()
    assert (st.ts_cur, st.pending, st.n_rejected, st.n_pushes) == (1, 3, 3, 7) == (ora.ts, ora.pending, ora.n_rejected, ora.n_pushes)
    t, avg, _ = ps.vector_clock(0)
    assert t == [0, 0, 0, 0] and avg == 0.0


@pytest.mark.parametrize("P", [1, 3, 4, 255, 72_000_000, (1 << 30) + 5, (1 << 32) + 7, 1 << 34, (1 << 35) + 1])
@pytest.mark.parametrize("block,vec,grid_cap", [(0, 0, 0), (64, 1, 0), (256, 4, 0), (1024, 2, 0), (64, 1, 1000)])
def test_launch_shapes_up_to_2_to_the_35_parameters(P, block, vec, grid_cap):
    """Host arithmetic of the launch shape (no device involved): every float4 position belongs to exactly one tile, the
    grid never makes grid * block reach 2^32 (HIP refuses such a launch), and a capped grid is covered by striding."""
    ps = R.ParameterServer(P, 2, flags=B.FLAG_CONTROL_ONLY, launch_block=block, launch_vec=vec, launch_grid=grid_cap, launch_unroll=2 if vec else 0)
    for batched in (False, True):
        grid, blk, ntiles, lds = ps.launch_shape(batched)
        per_tile = blk * (1 if batched else (vec or 1))
        n4 = P // 4
        assert blk == (block or 64) and ntiles == -(-n4 // per_tile)
        assert 1 <= grid and grid * blk < 1 << 32
        assert grid == max(1, min(ntiles, grid_cap or ntiles, ((1 << 32) - 1) // blk))
        assert lds <= 64 * 1024
    if P >= 1 << 34 and (block or 64) == 64 and not grid_cap:
        assert grid < ntiles                       # the case that used to ask for 2^32 threads or more


def test_plain_sgd_keeps_no_second_state_vector_and_says_so():
    """(control-only servers own no device memory at all; the statement about velocity is checked on the GPU)"""
    ps = R.ParameterServer(8, 2, flags=B.FLAG_CONTROL_ONLY)
    with pytest.raises(R.RudraError) as e:
        ps.pull_velocity(0x1000)
    assert e.value.status == B.ESTATE
    with pytest.raises(R.RudraError) as e:
        ps.weights_acquire()
    assert e.value.status == B.ESTATE
    assert ps.weights_release(0) == B.ESTATE
