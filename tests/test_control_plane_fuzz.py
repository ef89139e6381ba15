"""Randomised host-side checks (no GPU): arbitrary message sequences, valid and invalid, through the library's
control plane (RUDRA_FLAG_CONTROL_ONLY) and through the CPU oracle must give the same status codes, staleness,
clocks, rates and counters; and concurrent callers are serialised."""
import threading

import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import paper_1509_04210_amd as R
from oracle import OraclePS
from paper_1509_04210_amd import binding as B

LR_MODES = [oracle.LR_CONST, oracle.LR_STATIC_N, oracle.LR_AVG_STALENESS, oracle.LR_PER_GRADIENT]


@settings(max_examples=150, deadline=None)
@given(lam=st.integers(1, 9), data=st.data())
def test_random_message_sequences(lam, data):
    hard = data.draw(st.booleans())
    n = 1 if hard else data.draw(st.integers(1, lam))
    c_override = data.draw(st.sampled_from([0, 0, 0, 1, 3, 11]))
    max_agg = data.draw(st.sampled_from([0, 0, 1, 2, 5]))
    lr_mode = data.draw(st.sampled_from(LR_MODES if max_agg <= 1 else LR_MODES[:3]))
    alpha0 = data.draw(st.sampled_from([0.5, 0.01, 0.3]))
    lr_scale = data.draw(st.sampled_from([1.0, 0.96875]))
    proto = oracle.HARDSYNC if hard else oracle.SOFTSYNC
    ps = R.ParameterServer(3, lam, 0, n, proto, lr_mode, alpha0, lr_scale, c_override=c_override,
                           flags=B.FLAG_CONTROL_ONLY, clock_ring=4096, max_aggregate=max_agg)
    ora = OraclePS(np.zeros(3, np.float32), lam, n, proto, lr_mode, alpha0, lr_scale, c_override=c_override,
                   max_aggregate=max_agg)
    g = np.ones(3, np.float32)
    for _ in range(data.draw(st.integers(1, 80))):
        # timestamps around the current one (past, present, future), learners around the valid range
        ts = max(0, ora.ts + data.draw(st.integers(-4, 1)))
        learner = data.draw(st.integers(-2, lam))
        kind = data.draw(st.integers(0, 4))
        if kind == 4:                              # a run of messages in one call: stops at the first one the oracle rejects
            msgs = [(max(0, ora.ts + data.draw(st.integers(-4, 2))), data.draw(st.integers(-1, lam))) for _ in range(data.draw(st.integers(0, 7)))]
            rc_h, handled, res = ps.push_batch([0] * len(msgs), [m[0] for m in msgs], [m[1] for m in msgs])
            rc_o, k = 0, 0
            for ts_m, l_m in msgs:
                rc_o, ro = ora.push(g, ts_m, l_m)
                if rc_o != 0:
                    break
                r = res[k]
                assert (r.staleness, r.ts_after, r.pending, r.applied, np.float32(r.lr_used)) == \
                       (ro.staleness, ro.ts_after, ro.pending, ro.applied, np.float32(ro.lr_used))
                k += 1
            assert (rc_h, handled) == (rc_o, k)
            assert ps.pull_weights(0) == ora.ts
            continue
        if kind == 0:      # a relayed average of 1..max+1 gradients (one too many is rejected)
            stamps = [max(0, ora.ts + data.draw(st.integers(-3, 1))) for _ in range(data.draw(st.integers(1, max(1, max_agg) + 1)))]
            rc_h, r = ps.push_aggregate(0, stamps)
            rc_o, ro = ora.push_aggregate(g, stamps)
        else:
            rc_h, r = ps.push_gradient(0, ts, learner)
            rc_o, ro = ora.push(g, ts, learner)
        assert rc_h == rc_o
        if rc_h == 0:
            assert (r.staleness, r.ts_after, r.pending, r.applied, np.float32(r.lr_used)) == \
                   (ro.staleness, ro.ts_after, ro.pending, ro.applied, np.float32(ro.lr_used))
        assert ps.pull_weights(0) == ora.ts
    s = ps.stats()
    assert (s.ts_cur, s.n_pushes, s.n_updates, s.n_rejected, s.pending, s.c, s.sigma_sum, s.sigma_max) == \
           (ora.ts, ora.n_pushes, ora.n_updates, ora.n_rejected, ora.pending, ora.c, ora.sigma_sum, ora.sigma_max)
    assert np.array_equal(np.array(ps.staleness_hist(), np.uint64), ora.hist)
    clocks, avg, lr = ora.clocks, ora.avg_staleness, ora.lr_log
    for u in range(ora.n_updates):
        t, a, r = ps.vector_clock(u)
        assert t == [int(x) for x in clocks[u]] and a == avg[u] and np.float32(r) == lr[u]


def test_concurrent_pushes_are_serialised():
    """The server takes its messages one at a time (Sec. 3.2): 8 threads pushing at once lose no message and every update
    has exactly c entries."""
    lam, c, per_thread = 8, 4, 2000
    ps = R.ParameterServer(1, lam, 0, 2, B.SOFTSYNC, B.LR_AVG_STALENESS, flags=B.FLAG_CONTROL_ONLY)
    L, h = R.lib(), ps._h
    errors = []

    def worker(l):
        import ctypes
        res = B.PushResult()
        for _ in range(per_thread):
            rc = L.rudra_ps_push_gradient(h, None, 0, l, ctypes.byref(res))     # ts 0 is never from the future
            if rc != 0:
                errors.append(rc)

    threads = [threading.Thread(target=worker, args=(l,)) for l in range(lam)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    s = ps.stats()
    assert not errors
    assert s.n_pushes == lam * per_thread and s.n_updates == lam * per_thread // c == s.ts_cur and s.pending == 0
    hist = ps.staleness_hist()
    assert sum(hist) == s.n_pushes and sum(i * v for i, v in enumerate(hist)) == s.sigma_sum
