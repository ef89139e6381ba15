"""The seeded input generators: reproducible, of the stated distribution, and (on the GPU,
see test_gpu_parity) bit-identical between the numpy and the device implementation."""
import numpy as np

from synth import configs, gradgen, trace


def test_values_are_a_pure_function_of_the_counter():
    key = gradgen.stream_key(123, gradgen.TAG_GRAD, 5, 17)
    a = gradgen.vector(key, 10000, 1e-3)
    idx = np.array([0, 1, 7, 9999, 4242], dtype=np.uint64)
    assert np.array_equal(gradgen.values_at(key, idx, 1e-3), a[idx.astype(np.int64)])
    assert np.array_equal(gradgen.vector(key, 10000, 1e-3, chunk=333), a)
    assert not np.array_equal(gradgen.vector(gradgen.stream_key(123, gradgen.TAG_GRAD, 5, 18), 10000, 1e-3), a)
    assert gradgen.stream_key(1, 2, 3, 4) == gradgen.stream_key(1, 2, 3, 4) != gradgen.stream_key(1, 2, 4, 3)


def test_distribution_moments():
    x = gradgen.vector(gradgen.stream_key(7, gradgen.TAG_GRAD), 1 << 20, 1e-3).astype(np.float64)
    assert abs(x.mean()) < 5e-6 and abs(x.std() / 1e-3 - 1) < 5e-3
    assert np.abs(x).max() < 4.9e-3 and np.abs(x)[x != 0].min() > 1e-9     # bounded, far from denormals
    kurt = ((x - x.mean()) ** 4).mean() / x.var() ** 2
    assert abs(kurt - (3 - 1.2 / 8)) < 0.03                               # Irwin-Hall of 8: 3 - 6/(5*8)
    # heavy tail of the 72M workload: 1 % of the entries times 100
    y = configs.C4.grad_at(3, 5, np.arange(1 << 20, dtype=np.uint64)).astype(np.float64)
    frac = (np.abs(y) > 6e-4).mean()        # beyond 6 std of the body: tail entries only (|z| > 0.06 of them)
    assert 0.008 < frac < 0.0115
    assert abs(y.std() / (1e-4 * np.sqrt(0.99 + 0.01 * 1e4)) - 1) < 0.05
    w = configs.C1.init_weights_at(np.arange(1 << 18, dtype=np.uint64)).astype(np.float64)
    assert abs(w.std() / 0.01 - 1) < 0.01


def test_traces_are_seeded_and_well_formed():
    l1, s1 = trace.softsync_trace(42, 30, 3000, straggler_prob=0.1)
    l2, s2 = trace.softsync_trace(42, 30, 3000, straggler_prob=0.1)
    assert np.array_equal(l1, l2) and np.array_equal(s1, s2)
    assert not np.array_equal(l1, trace.softsync_trace(43, 30, 3000, straggler_prob=0.1)[0])
    for l in range(30):   # each learner's steps arrive in order 0,1,2,...
        assert np.array_equal(s1[l1 == l], np.arange((l1 == l).sum()))
    counts = np.bincount(l1, minlength=30)
    assert counts.min() > 50 and counts.max() < 160      # Exp(1) durations, 10 % stragglers x3: mean 100
    lh, sh = trace.hardsync_trace(1, 30, 10)
    assert np.array_equal(np.sort(lh.reshape(10, 30), axis=1), np.tile(np.arange(30), (10, 1)))
    assert np.array_equal(sh.reshape(10, 30), np.repeat(np.arange(10), 30).reshape(10, 30))
    assert len({tuple(r) for r in lh.reshape(10, 30)}) > 1   # order differs from round to round


def test_workload_table():
    c = {k: w.c for k, w in configs.ALL.items()}
    assert c == {"C1": 4, "C2": 30, "C3-n1": 30, "C3-n2": 15, "C3-n4": 7, "C3-n4-c8": 8, "C3-n30": 1, "C4": 18, "C5": 1,
                 "C4-adagrad": 18}
    assert configs.C4.n_params == configs.C5.n_params == 72_000_000
    l, s = configs.C2.arrival_trace(95)
    assert len(l) == 95
