"""Parity of the HIP path (called through the C ABI) with the CPU oracle, element by element, on the same
seeded inputs.  Bar: theta and v within 1e-5 * ||.||_inf of the binary32 oracle; timestamps, staleness,
vector clocks, histogram, counters and learning rates bit-exact.  (Both sides evaluate the same sequence of
individually rounded binary32 operations, so in practice the floats are bit-identical too; that stronger
property is asserted separately so a regression shows which of the two broke.)"""
import numpy as np
import pytest
import torch

from oracle.adapter import OracleServer
from synth import configs, gradgen, replay

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def hipmod():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1509_04210_amd import binding
    from synth import learners
    binding.lib()            # fails loudly if the HIP library is not built
    gradgen.device_lib()
    return learners


def _with(w, **kw):
    return type(w)(**{**w.__dict__, **kw})


def _compare(hip, ora, w, check_bits=True):
    th = hip.weights().cpu().numpy()
    ref = ora.ps.theta
    scale = np.abs(ref).max()
    err = np.abs(th.astype(np.float64) - ref.astype(np.float64)).max()
    assert err <= TOL * scale, f"theta: max abs err {err:.3e} vs {TOL * scale:.3e}"
    if w.momentum != 0 or w.optimizer == "adagrad":
        ve = hip.velocity().cpu().numpy()
        vref = ora.ps.velocity
        verr = np.abs(ve.astype(np.float64) - vref.astype(np.float64)).max()
        assert verr <= TOL * max(np.abs(vref).max(), 1e-30), f"v: max abs err {verr:.3e}"
        if check_bits:
            assert np.array_equal(ve, vref), "velocity not bit-identical"
    if check_bits:
        assert np.array_equal(th, ref), "theta not bit-identical"
    st = hip.ps.stats()
    o = ora.ps
    assert (st.ts_cur, st.n_pushes, st.n_updates, st.pending, st.c) == (o.ts, o.n_pushes, o.n_updates, o.pending, o.c)
    assert (st.sigma_sum, st.sigma_max) == (o.sigma_sum, o.sigma_max)
    assert np.array_equal(np.array(hip.ps.staleness_hist(), np.uint64), o.hist)
    clocks, avg, lr = o.clocks, o.avg_staleness, o.lr_log
    for u in range(max(0, o.n_updates - 1024), o.n_updates):
        ts, a, r = hip.ps.vector_clock(u)
        assert ts == list(clocks[u]) and a == avg[u] and np.float32(r) == lr[u]
    return err / scale


def _run_both(learners, w, flags=0, n_pushes=None, **launch):
    learner, step = w.arrival_trace(n_pushes)
    hard = w.protocol == "hardsync"
    hip, ora = learners.HipServer(w, flags=flags, **launch), OracleServer(w)
    lh = replay.replay(hip, learner, step, w.n_learners, hardsync=hard)
    lo = replay.replay(ora, learner, step, w.n_learners, hardsync=hard)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    return hip, ora


# ---------------------------------------------------------------- inputs: device generator == numpy generator
@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4096, 100_003])
def test_device_generator_is_bit_identical_to_numpy(hipmod, n):
    for tail_per, std in [(0, 1e-3), (100, 1e-4)]:
        key = gradgen.stream_key(99, gradgen.TAG_GRAD, 3, n)
        buf = torch.full((n + 8,), 7.0, dtype=torch.float32, device="cuda")
        gradgen.fill_device(buf.data_ptr(), n, key, std, tail_per, 100.0, stream=0)
        torch.cuda.synchronize()
        got = buf.cpu().numpy()
        assert np.array_equal(got[:n], gradgen.vector(key, n, std, tail_per, 100.0))
        assert np.all(got[n:] == 7.0)       # nothing written past the end


# ---------------------------------------------------------------- every workload, at a size the oracle replays in seconds
# sizes span many tiles (64 to 4096 float4 positions each, depending on the launch shape) and leave a ragged tail
SMALL = {
    "C1": (configs.C1, 131072, 256),                 # the tiny config at its real size
    "C2": (configs.C2, 70_003, 900),                 # hardsync, momentum
    "C3-n1": (configs.C3(1), 50_001, 600),
    "C3-n2": (configs.C3(2), 50_002, 600),
    "C3-n4": (configs.C3(4), 50_003, 600),           # c = floor(30/4) = 7
    "C3-n4-c8": (configs.C3_N4_C8, 50_004, 600),     # the same with 8 gradients per update (c_override)
    "C3-n30": (configs.C3(30), 50_005, 600),
    "C4": (configs.C4, 90_007, 360),                 # c = 18, heavy-tailed gradients, momentum
    "C5": (configs.C5, 90_001, 700),                 # c = 1, momentum + weight penalty, staleness up to ~100
    "C4-adagrad": (configs.C4_ADAGRAD, 90_003, 360),  # AdaGrad instead of momentum
}


@pytest.mark.parametrize("name", list(SMALL))
def test_workload_parity_small(hipmod, name):
    base, P, n = SMALL[name]
    w = base.scaled(n_params=P, n_pushes=n)
    hip, ora = _run_both(hipmod, w)
    rel = _compare(hip, ora, w)
    print(f"{name}: P={P} pushes={n} updates={ora.ps.ts} rel err={rel:.2e}")
    hip.close()


def test_c2_full_size_hardsync(hipmod):
    """The 1.0M-parameter hardsync workload at its real size (a reduced number of rounds keeps the CPU replay short)."""
    w = configs.C2.scaled(n_pushes=30 * 40)
    hip, ora = _run_both(hipmod, w)
    _compare(hip, ora, w)
    assert hip.ps.stats().sigma_max == 0
    hip.close()


# ---------------------------------------------------------------- launch shapes, c from 1 past the fused limit, modes
@pytest.mark.parametrize("block,unroll,vec,grid,waves,alternate", [
    (64, 1, 1, 0, 0, 0), (256, 4, 1, 0, 32, 2), (256, 8, 1, 0, 4, 1), (512, 2, 2, 0, 0, 0), (1024, 2, 4, 0, 16, 0),
    (256, 4, 2, 3, 0, 1), (128, 1, 4, 7, 2, 2), (256, 2, 1, 1, 0, 0), (64, 4, 2, 0, 8, 0)])
def test_launch_shapes_give_the_same_bits(hipmod, block, unroll, vec, grid, waves, alternate):
    w = _with(configs.C4.scaled(n_params=33_331, n_pushes=18 * 4), weight_decay=5e-4)
    hip, ora = _run_both(hipmod, w, launch_block=block, launch_unroll=unroll, launch_vec=vec, launch_grid=grid,
                         launch_waves_per_cu=waves, launch_alternate=alternate)
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("c", [1, 2, 3, 5, 8, 9, 13, 17, 31, 64, 65, 70, 130])
def test_gradients_per_update_sweep(hipmod, c):
    """c below, at and beyond the 64 gradients one launch takes (larger sets are folded through the accumulator)."""
    w = _with(configs.C3(1).scaled(n_params=9_999, n_pushes=3 * c + 1), n_learners=max(c, 2), c_override=c,
              momentum=0.9)
    hip, ora = _run_both(hipmod, w, launch_unroll=8)
    _compare(hip, ora, w)
    assert hip.ps.stats().pending == (1 if c > 1 else 0)
    hip.close()


@pytest.mark.parametrize("lr_mode", ["const", "static_n", "avg_staleness", "per_gradient"])
@pytest.mark.parametrize("momentum,wd", [(0.0, 0.0), (0.9, 5e-4)])
def test_rate_modes(hipmod, lr_mode, momentum, wd):
    w = _with(configs.C3(4).scaled(n_params=20_002, n_pushes=350), lr_mode=lr_mode, momentum=momentum,
              weight_decay=wd, alpha0=0.05)
    hip, ora = _run_both(hipmod, w)
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("lr_mode,wd,eps", [("avg_staleness", 0.0, 1e-8), ("avg_staleness", 5e-4, 1e-3),
                                            ("per_gradient", 5e-4, 1e-8), ("const", 0.0, 0.0)])
def test_adagrad_modes(hipmod, lr_mode, wd, eps):
    """AdaGrad: sqrt and divide are correctly rounded on both sides, so the accumulator h and theta are bit-identical."""
    w = _with(configs.C3(4).scaled(n_params=30_003, n_pushes=420), optimizer="adagrad", adagrad_eps=eps, lr_mode=lr_mode,
              weight_decay=wd, alpha0=0.05)
    hip, ora = _run_both(hipmod, w, launch_unroll=2, launch_vec=2)
    th, h = hip.weights().cpu().numpy(), hip.velocity().cpu().numpy()
    assert np.abs(th.astype(np.float64) - ora.ps.theta).max() <= TOL * np.abs(ora.ps.theta).max()
    assert np.array_equal(th, ora.ps.theta) and np.array_equal(h, ora.ps.velocity)
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("lr_mode", ["avg_staleness", "per_gradient"])
def test_accumulate_at_push_gives_the_same_bits_as_the_fused_path(hipmod, lr_mode):
    from paper_1509_04210_amd import binding as B
    w = _with(configs.C3(2).scaled(n_params=40_001, n_pushes=300), lr_mode=lr_mode, momentum=0.9)
    hip, ora = _run_both(hipmod, w, flags=B.FLAG_PUSH_ACCUMULATE)
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 8, 1023, 1024, 1025, 4099])
def test_tiny_and_ragged_vectors(hipmod, P):
    w = _with(configs.C5.scaled(n_params=P, n_pushes=40), n_learners=5, n_split=2)
    hip, ora = _run_both(hipmod, w)
    _compare(hip, ora, w)
    hip.close()


def test_leftover_gradients_stay_pending(hipmod):
    w = configs.C3(1).scaled(n_params=5000, n_pushes=2 * 30 + 11)
    hip, ora = _run_both(hipmod, w)
    _compare(hip, ora, w)
    st = hip.ps.stats()
    assert st.pending == 11 and st.ts_cur == 2
    hip.close()


# ---------------------------------------------------------------- boundary behaviour on the device
def test_rejected_pushes_leave_the_weights_alone(hipmod):
    from paper_1509_04210_amd import binding as B
    w = _with(configs.C2.scaled(n_params=1000, n_pushes=6), n_learners=3)
    hip = hipmod.HipServer(w)
    before = hip.weights().cpu().numpy()
    g = torch.ones(1004, dtype=torch.float32, device="cuda")
    assert hip.ps.push_gradient(g.data_ptr() + 4, 0, 0)[0] == B.EINVAL          # not 16-byte aligned
    assert hip.ps.push_gradient(0, 0, 0)[0] == B.EINVAL                         # null
    assert hip.ps.push_gradient(g.data_ptr(), 1, 0)[0] == B.EFUTURE_TS
    assert hip.ps.push_gradient(g.data_ptr(), 0, 9)[0] == B.EINVAL
    assert hip.ps.push_gradient(g.data_ptr(), 0, 0)[0] == B.OK
    assert hip.ps.push_gradient(g.data_ptr(), 0, 0)[0] == B.EHARDSYNC_DUP
    hip.ps.sync()
    assert np.array_equal(hip.weights().cpu().numpy(), before)
    assert hip.ps.push_gradient(g.data_ptr(), 0, 1)[0] == B.OK
    rc, r = hip.ps.push_gradient(g.data_ptr(), 0, 2)
    assert rc == B.OK and r.applied == 1 and r.ts_after == 1
    assert hip.ps.push_gradient(g.data_ptr(), 0, 0)[0] == B.EHARDSYNC_STALE
    after = hip.weights().cpu().numpy()
    want = before - np.float32(w.alpha0) * (np.float32(3.0) * (np.float32(1) / np.float32(3)))
    assert np.array_equal(after, want.astype(np.float32))
    st = hip.ps.stats()
    assert st.n_rejected == 6 and st.n_pushes == 3 and st.last_hip_error == 0
    hip.close()


def test_pull_returns_weights_with_their_timestamp(hipmod):
    w = configs.C1.scaled(n_params=4097, n_pushes=8)
    hip, ora = _run_both(hipmod, w, n_pushes=4)            # exactly one update
    dst = torch.zeros(4097, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    ts = hip.ps.pull_weights(dst.data_ptr())
    hip.ps.sync()
    assert ts == 1 and np.array_equal(dst.cpu().numpy(), ora.ps.theta)
    assert hip.ps.pull_weights(0) == 1                     # timestamp inquiry: no copy
    hip.close()


def test_fused_norms(hipmod):
    from paper_1509_04210_amd import binding as B
    for shape in (dict(), dict(launch_block=512, launch_vec=2, launch_grid=5)):
        w = configs.C5.scaled(n_params=77_777, n_pushes=30)
        hip, ora = _run_both(hipmod, w, flags=B.FLAG_STATS_NORMS, **shape)
        _compare(hip, ora, w)
        st, ref = hip.ps.stats(), ora.ps.norms()
        assert st.norms_valid == 1
        for got, want in [(st.theta_sq, ref["theta_sq"]), (st.v_sq, ref["v_sq"]), (st.gbar_sq, ref["gbar_sq"])]:
            assert abs(got - want) <= 1e-5 * want
        assert st.theta_inf == ref["theta_inf"]            # a max of binary32 values: exact
        hip.close()


def test_kernel_timer_counts_every_update(hipmod):
    from paper_1509_04210_amd import binding as B
    w = configs.C5.scaled(n_params=50_000, n_pushes=300)    # more updates than the timer ring holds
    hip, ora = _run_both(hipmod, w, flags=B.FLAG_TIME_KERNELS)
    _compare(hip, ora, w)
    st = hip.ps.stats()
    assert st.kernel_launches == 300 and 0 < st.kernel_ms < 300 * 5.0
    hip.close()


# ---------------------------------------------------------------- full size and full length, in the launch shape bench.py times
def _sample_indices(P, seed, n_random, span=4096):
    rng = np.random.default_rng(seed)
    head = np.arange(0, min(P, 2 * span))                   # the first tiles
    tail = np.arange(max(0, P - span - 7), P)               # the last tiles and the ragged end
    rand = rng.integers(0, P, size=n_random)
    return np.unique(np.concatenate([head, tail, rand])).astype(np.uint64)


FULL = {"C4-adagrad": 16384, "C2": 3000, "C3-n1": 16384, "C3-n2": 16384, "C3-n4": 16384, "C3-n4-c8": 16384, "C3-n30": 16384, "C4": 16384,
        "C5": 16384}


@pytest.mark.parametrize("name", list(FULL))
def test_full_size_full_length_parity_on_sampled_elements(hipmod, name):
    """Every workload at its stated size AND length (C2: 1.0M x 30 000 pushes ... C4: 72M x 3600, C5: 72M x 5000),
    default launch shape (the one bench.py times).  The update is elementwise, so the oracle replays the same
    trace on sampled positions (first tiles, last tiles + tail, random) and every sampled theta/v must match;
    integer outputs are compared in full."""
    w = configs.ALL[name]
    idx = _sample_indices(w.n_params, 7, FULL[name])
    learner, step = w.arrival_trace()
    hard = w.protocol == "hardsync"
    hip, ora = hipmod.HipServer(w), OracleServer(w, index=idx)
    lh = replay.replay(hip, learner, step, w.n_learners, hardsync=hard)
    lo = replay.replay(ora, learner, step, w.n_learners, hardsync=hard)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    sel = torch.from_numpy(idx.astype(np.int64)).cuda()
    th = hip.weights()[sel].cpu().numpy()
    ref = ora.ps.theta
    assert np.abs(th.astype(np.float64) - ref).max() <= TOL * np.abs(ref).max()
    assert np.array_equal(th, ref)
    # the same steps in binary64 (no binary32 rounding at all): the tolerance also holds against that
    ora64 = OracleServer(w, index=idx[:2048], precision=64)
    replay.replay(ora64, learner, step, w.n_learners, hardsync=hard)
    ref64 = ora64.ps.theta
    drift = np.abs(th[:2048].astype(np.float64) - ref64).max() / np.abs(ref64).max()
    print(f"{name}: distance from the binary64 run {drift:.2e}")
    # AdaGrad divides by sqrt(h) ~ |gbar|: where the c gradients nearly cancel, the rounding of their binary32 sum is
    # amplified to a step of order alpha, so binary32 itself (oracle and GPU alike) sits further from binary64 there
    assert drift <= (1e-3 if w.optimizer == "adagrad" else TOL)
    if w.momentum != 0 or w.optimizer == "adagrad":
        ve = hip.velocity()[sel].cpu().numpy()
        vref = ora.ps.velocity
        assert np.abs(ve.astype(np.float64) - vref).max() <= TOL * np.abs(vref).max()
        assert np.array_equal(ve, vref)
    st = hip.ps.stats()
    o = ora.ps
    assert (st.ts_cur, st.n_pushes, st.pending, st.sigma_sum, st.sigma_max) == (o.ts, o.n_pushes, o.pending, o.sigma_sum, o.sigma_max)
    assert st.n_pushes == w.n_pushes and st.ts_cur == w.n_pushes // w.c
    assert np.array_equal(np.array(hip.ps.staleness_hist(), np.uint64), o.hist)
    lr = o.lr_log
    for u in range(max(0, o.n_updates - 1024), o.n_updates):
        assert np.float32(hip.ps.vector_clock(u)[2]) == lr[u]
    # properties that hold at any size: the whole state is finite, and positions the oracle did not sample moved too
    full = hip.weights()
    assert bool(torch.isfinite(full).all())
    hip.close()


# ---------------------------------------------------------------- double-buffered weights, zero-copy pull
def _read_device(ptr, n):
    """Copy n floats from a raw device address into a numpy array (synchronous hipMemcpy)."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    out = np.empty(n, np.float32)
    assert hip.hipMemcpy(out.ctypes.data, ptr, n * 4, 2) == 0       # 2 = device to host
    return out


@pytest.mark.parametrize("name", ["C4", "C5", "C4-adagrad"])
def test_double_buffer_gives_the_same_bits(hipmod, name):
    from paper_1509_04210_amd import binding as B
    base, P, n = SMALL[name]
    w = base.scaled(n_params=P, n_pushes=n)
    hip, ora = _run_both(hipmod, w, flags=B.FLAG_DOUBLE_BUFFER)
    _compare(hip, ora, w)
    hip.close()


def test_weights_view_stays_valid_while_the_next_update_runs(hipmod):
    """Sec. 3.3 pointer swap, server side: the weights of timestamp i remain readable, unchanged, until update i+2."""
    from paper_1509_04210_amd import binding as B
    w = configs.C3(2).scaled(n_params=70_001, n_pushes=15 * 6)
    learner, step = w.arrival_trace()
    hip, ora = hipmod.HipServer(w, flags=B.FLAG_DOUBLE_BUFFER), OracleServer(w)
    views, refs, ts_l = [], [], [0] * w.n_learners
    for i in range(len(learner)):
        l, s = int(learner[i]), int(step[i])
        _, _, applied = hip.push(l, s, ts_l[l])
        ora.push(l, s, ts_l[l])
        ts_l[l] = hip.pull_ts()
        if applied:
            ptr, ts = hip.ps.weights_view()
            assert ts == ora.ps.ts
            views.append(ptr)
            refs.append(ora.ps.theta)
            hip.ps.sync()
            assert np.array_equal(_read_device(ptr, w.n_params), refs[-1])              # the current weights
            if len(views) >= 2:                                                          # the previous ones: still intact
                assert views[-2] != ptr
                assert np.array_equal(_read_device(views[-2], w.n_params), refs[-2])
            if len(views) >= 3:
                assert views[-3] == ptr                                                  # two buffers, ping-pong
    assert len(views) == 6
    st = hip.ps.stats()
    assert st.n_weight_views == 6 and st.n_weight_copies == 0 and st.n_ts_inquiries == len(learner)
    hip.close()
    single = hipmod.HipServer(w)                  # without the flag there is one buffer
    p0, _ = single.ps.weights_view()
    for i in range(15):
        single.push(int(learner[i]), int(step[i]), 0)
    assert single.ps.weights_view() == (p0, 1)
    single.close()


def test_pointer_check_rejects_what_a_kernel_would_fault_on(hipmod):
    from paper_1509_04210_amd import binding as B
    w = _with(configs.C1.scaled(n_params=10_000, n_pushes=8), n_learners=2, n_split=1)
    hip = hipmod.HipServer(w, flags=B.FLAG_CHECK_POINTERS)
    before = hip.weights().cpu().numpy()
    host = np.zeros(10_016, np.float32)
    host_ptr = (host.ctypes.data + 15) & ~15
    import ctypes
    rt = ctypes.CDLL("libamdhip64.so")          # raw allocations: torch carves its tensors out of larger blocks
    rt.hipMalloc.argtypes, rt.hipMemset.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t], [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t]

    def raw(nbytes):
        p = ctypes.c_void_p()
        assert rt.hipMalloc(ctypes.byref(p), nbytes) == 0 and rt.hipMemset(p, 0, nbytes) == 0
        return p.value

    small, late_base = raw(20_000), raw(40_016)

    class _P:                                    # same accessors as a tensor, for the lines below
        def __init__(self, p): self.p = p
        def data_ptr(self): return self.p
    small, late = _P(small), _P(late_base)
    good = torch.ones(10_000, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    assert hip.ps.push_gradient(host_ptr, 0, 0)[0] == B.EINVAL                  # host memory
    assert hip.ps.push_gradient(small.data_ptr(), 0, 0)[0] == B.EINVAL          # too short
    assert hip.ps.push_gradient(late.data_ptr() + 32, 0, 0)[0] == B.EINVAL      # runs 16 bytes past its allocation
    assert hip.ps.push_gradient(0x10000, 0, 0)[0] == B.EINVAL                   # not a HIP pointer at all
    assert hip.ps.push_gradient(good.data_ptr(), 0, 0)[0] == B.OK
    rc, r = hip.ps.push_gradient(late.data_ptr() + 16, 0, 1)                    # fits exactly
    assert rc == B.OK and r.applied == 1
    after = hip.weights().cpu().numpy()
    assert np.array_equal(after, before - np.float32(w.alpha0) * (np.float32(1.0) * np.float32(0.5)))   # gradients: ones, zeros
    st = hip.ps.stats()
    assert st.n_rejected == 4 and st.last_hip_error == 0
    with pytest.raises(B.RudraError) as e:                                       # create() always checks init_weights
        B.ParameterServer(10_000, 2, host_ptr)
    assert e.value.status == B.EINVAL
    hip.close()


# ---------------------------------------------------------------- parameter-server tree (Sec. 3.3)
@pytest.mark.parametrize("k,n", [(1, 1000), (2, 4099), (3, 70_001), (7, 5), (18, 33_333), (64, 2050), (65, 2051), (130, 777)])
def test_leaf_mean_kernel(hipmod, k, n):
    """rudra_ps_leaf_mean == the oracle's node average, bit for bit (groups beyond 64 gradients are folded)."""
    import oracle
    from paper_1509_04210_amd import binding as B
    key = lambda j: gradgen.stream_key(5, gradgen.TAG_GRAD, j, n)
    bufs = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(k)]
    out = torch.full((n + 8,), 9.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for j, b in enumerate(bufs):
        gradgen.fill_device(b.data_ptr(), n, key(j), 1e-3, 100, 100.0, stream=0)
    B.leaf_mean([b.data_ptr() for b in bufs], n, out.data_ptr(), 0, 0)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = oracle.leaf_mean([gradgen.vector(key(j), n, 1e-3, 100, 100.0) for j in range(k)])
    assert np.array_equal(got[:n], want) and np.all(got[n:] == 9.0)


@pytest.mark.parametrize("name,lam,fan_in,n_split,P,n_pushes", [
    ("C4", 54, 3, 1, 60_001, 54 * 6 + 10),        # the paper's Rudra-adv ImageNet run: 54 learners, 1-softsync, here nodes of 3
    ("C5", 12, 4, 3, 30_002, 300),                # c = 4 = one relayed message per update
    ("C4-adagrad", 10, 4, 1, 20_003, 200),        # 10 learners in nodes of 4, 4, 2 (the last node never fills): c = 10 is overshot
    ("C2", 8, 2, 1, 10_001, 8 * 12),              # hardsync under a tree
])
def test_tree_parity(hipmod, name, lam, fan_in, n_split, P, n_pushes):
    base = configs.ALL[name]
    w = _with(base.scaled(n_params=P, n_pushes=n_pushes), n_learners=lam, n_split=n_split)
    learner, step = w.arrival_trace()
    hard = w.protocol == "hardsync"
    hip = hipmod.HipServer(w, ring=2 * fan_in + 2, avg_ring=w.c // fan_in + 4, max_aggregate=fan_in)
    ora = OracleServer(w, max_aggregate=fan_in)
    lh = replay.replay_tree(hip, learner, step, lam, fan_in, hardsync=hard)
    lo = replay.replay_tree(ora, learner, step, lam, fan_in, hardsync=hard)
    for key in lo:
        assert np.array_equal(lh[key], lo[key]), key
    assert lo["applied"].sum() >= 3
    th = hip.weights().cpu().numpy()
    assert np.abs(th.astype(np.float64) - ora.ps.theta).max() <= TOL * np.abs(ora.ps.theta).max()
    assert np.array_equal(th, ora.ps.theta)
    if w.momentum != 0 or w.optimizer == "adagrad":
        assert np.array_equal(hip.velocity().cpu().numpy(), ora.ps.velocity)
    st, o = hip.ps.stats(), ora.ps
    assert (st.ts_cur, st.n_pushes, st.pending, st.sigma_sum, st.sigma_max) == (o.ts, o.n_pushes, o.pending, o.sigma_sum, o.sigma_max)
    assert np.array_equal(np.array(hip.ps.staleness_hist(), np.uint64), o.hist)
    clocks, avg, lr = o.clocks, o.avg_staleness, o.lr_log
    for u in range(o.n_updates):
        t, a, r = hip.ps.vector_clock(u)
        assert t == [int(x) for x in clocks[u]] and a == avg[u] and np.float32(r) == lr[u]
    hip.close()


def test_tree_full_size_on_sampled_elements(hipmod):
    """72M parameters, 54 learners in 18 nodes of 3, 1-softsync (the shape of the paper's Rudra-adv ImageNet run)."""
    lam, fan_in = 54, 3
    w = _with(configs.C4.scaled(n_pushes=54 * 20), n_learners=lam)
    idx = _sample_indices(w.n_params, 11, 8192)
    learner, step = w.arrival_trace()
    hip = hipmod.HipServer(w, ring=2 * fan_in + 2, avg_ring=w.c // fan_in + 4, max_aggregate=fan_in)
    ora = OracleServer(w, index=idx, max_aggregate=fan_in)
    lh = replay.replay_tree(hip, learner, step, lam, fan_in)
    lo = replay.replay_tree(ora, learner, step, lam, fan_in)
    for key in lo:
        assert np.array_equal(lh[key], lo[key]), key
    sel = torch.from_numpy(idx.astype(np.int64)).cuda()
    assert np.array_equal(hip.weights()[sel].cpu().numpy(), ora.ps.theta)
    assert np.array_equal(hip.velocity()[sel].cpu().numpy(), ora.ps.velocity)
    assert hip.ps.stats().ts_cur == ora.ps.ts >= 19
    hip.close()


def test_vectors_beyond_4_gib(hipmod):
    """2^30 + 5 parameters: byte offsets pass 2^32 inside every stream, the tail is ragged, and the grid has 4.2M
    workgroups.  Oracle on sampled positions around the 4 GiB boundary, the ends, and random ones."""
    P = (1 << 30) + 5
    w = _with(configs.C5.scaled(n_params=P, n_pushes=6), n_learners=3, n_split=1)        # c = 3, momentum + decay
    around = np.arange((1 << 30) - 2048, P)                       # the last MiB-crossing tiles and the tail
    idx = np.unique(np.concatenate([_sample_indices(P, 3, 4096), around])).astype(np.uint64)
    learner, step = w.arrival_trace()
    hip, ora = hipmod.HipServer(w, ring=4), OracleServer(w, index=idx)
    lh = replay.replay(hip, learner, step, w.n_learners)
    lo = replay.replay(ora, learner, step, w.n_learners)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    sel = torch.from_numpy(idx.astype(np.int64)).cuda()
    assert np.array_equal(hip.weights()[sel].cpu().numpy(), ora.ps.theta)
    assert np.array_equal(hip.velocity()[sel].cpu().numpy(), ora.ps.velocity)
    assert hip.ps.stats().ts_cur == 2
    hip.close()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("optimizer", ["sgd", "adagrad"])
def test_subnormal_numbers_are_kept(hipmod, optimizer):
    """Weights, gradients, steps and squared gradients in (and below) the subnormal range of binary32: the kernel must not
    flush them to zero, the CPU does not."""
    w = _with(configs.C3(2).scaled(n_params=20_001, n_pushes=150), init_std=3e-38, grad_std=2e-38 if optimizer == "sgd" else 1e-20,
              alpha0=0.5, momentum=0.9 if optimizer == "sgd" else 0.0, weight_decay=0.25 if optimizer == "sgd" else 0.0, optimizer=optimizer, adagrad_eps=0.0 if optimizer == "sgd" else 1e-30)
    hip, ora = _run_both(hipmod, w)
    ref = ora.ps.theta
    probe = ref if optimizer == "sgd" else ora.ps.velocity            # AdaGrad: the squared-gradient sums are the tiny ones
    tiny = np.abs(probe[probe != 0]) < 1.1754944e-38
    assert tiny.mean() > 0.2                          # the case really lives among subnormals
    assert np.array_equal(hip.weights().cpu().numpy(), ref)
    assert np.array_equal(hip.velocity().cpu().numpy(), ora.ps.velocity)
    hip.close()


# ---------------------------------------------------------------- rudra_ps_push_batch: consecutive updates fused into one launch
def _run_both_batched(learners, w, chunks, flags=0, ring=None, **launch):
    learner, step = w.arrival_trace()
    hard = w.protocol == "hardsync"
    hip = learners.HipServer(w, flags=flags, ring=ring or (max(chunks) + w.c + 1), **launch)
    ora = OracleServer(w)
    lh = replay.replay_batched(hip, learner, step, w.n_learners, chunks, hardsync=hard, c=w.c)
    lo = replay.replay_batched(ora, learner, step, w.n_learners, chunks, hardsync=hard, c=w.c)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    return hip, ora


BATCH_CASES = {
    # name: (workload, chunk sizes cycled over the trace)
    "c1-momentum-decay": (configs.C5.scaled(n_params=40_003, n_pushes=400), [1, 2, 3, 7, 16, 64, 65, 100, 5]),
    "c1-sgd": (_with(configs.C3(30).scaled(n_params=9_999, n_pushes=300)), [64, 1, 63, 2, 128]),
    "c4-no-momentum": (configs.C1.scaled(n_params=131_072, n_pushes=256), [9, 4, 1, 31, 8]),
    "c7-stragglers": (configs.C3(4).scaled(n_params=20_001, n_pushes=500), [50, 3, 14, 70]),
    "c18-heavy-tail": (configs.C4.scaled(n_params=33_331, n_pushes=18 * 12), [40, 18, 5, 72]),
    "hardsync-c30": (configs.C2.scaled(n_params=10_007, n_pushes=30 * 9), [45, 30, 7, 90]),
    "adagrad": (_with(configs.C4_ADAGRAD.scaled(n_params=5_555, n_pushes=18 * 10), n_learners=6, weight_decay=5e-4), [13, 2, 30]),
    "per-gradient-weights": (_with(configs.C3(10).scaled(n_params=7_777, n_pushes=400), lr_mode="per_gradient", momentum=0.9), [25, 6, 64]),
    "c70-beyond-one-launch": (_with(configs.C3(1).scaled(n_params=4_099, n_pushes=70 * 4 + 3), n_learners=70, c_override=70, momentum=0.9), [150, 9]),
    "c33-two-updates-do-not-fit": (_with(configs.C3(1).scaled(n_params=4_099, n_pushes=33 * 7), n_learners=33, c_override=33), [100, 33, 98]),
    "tiny-vectors": (configs.C5.scaled(n_params=3, n_pushes=50), [8, 5]),
    # larger vectors (thousands of tiles), ragged tails
    "wide-c1-momentum-decay": (configs.C5.scaled(n_params=600_003, n_pushes=150), [1, 2, 3, 7, 16, 64, 65]),
    "wide-c18-heavy-tail": (configs.C4.scaled(n_params=524_288 + 2, n_pushes=18 * 8), [40, 18, 5, 72]),
    "wide-adagrad": (_with(configs.C4_ADAGRAD.scaled(n_params=555_555, n_pushes=6 * 10), n_learners=6, weight_decay=5e-4), [13, 2, 30]),
    "wide-per-gradient-weights": (_with(configs.C3(10).scaled(n_params=524_289, n_pushes=200), lr_mode="per_gradient", momentum=0.9), [25, 6, 64]),
    "wide-hardsync-c30": (configs.C2.scaled(n_pushes=30 * 6), [45, 30, 7, 90]),
}


@pytest.mark.parametrize("name", list(BATCH_CASES))
def test_batched_pushes_give_the_bits_of_single_pushes(hipmod, name):
    """Messages handed over in runs (rudra_ps_push_batch) against the oracle, which takes them one by one: same
    staleness / applied per message, same clocks and rates, same theta and v to the bit."""
    w, chunks = BATCH_CASES[name]
    hip, ora = _run_both_batched(hipmod, w, chunks)
    _compare(hip, ora, w)
    st = hip.ps.stats()
    assert st.n_apply_launches <= st.n_updates
    if w.c <= 32 and max(chunks) >= 2 * w.c:
        assert st.n_batched_updates > 0 and st.n_apply_launches < st.n_updates     # something was fused
    hip.close()


@pytest.mark.parametrize("unroll", [1, 4, 8])
@pytest.mark.parametrize("name", ["c1-momentum-decay", "c7-stragglers", "adagrad", "per-gradient-weights",
                                  "c33-two-updates-do-not-fit", "wide-c18-heavy-tail"])
def test_batched_loads_per_round_give_the_same_bits(hipmod, name, unroll):
    """A batched launch walks its gradient list one load ahead (long vectors) or 4 / 8 loads per round (the default for
    short ones); launch_unroll names the scheme.  Lists whose length is no multiple of the round included."""
    w, chunks = BATCH_CASES[name]
    hip, ora = _run_both_batched(hipmod, w, chunks, launch_unroll=unroll)
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("P", [1, 4, 5, 63, 64, 65, 257, 1024 + 3])
def test_batched_pushes_on_ragged_vectors(hipmod, P):
    w = configs.C5.scaled(n_params=P, n_pushes=40)
    hip, ora = _run_both_batched(hipmod, w, [6, 11, 2])
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("block,grid,waves,alternate", [(64, 0, 0, 0), (256, 3, 4, 1), (1024, 0, 32, 2), (128, 1, 0, 0)])
def test_batched_launch_shapes_give_the_same_bits(hipmod, block, grid, waves, alternate):
    for P in (50_001, 530_001):
        w = configs.C5.scaled(n_params=P, n_pushes=120)
        hip, ora = _run_both_batched(hipmod, w, [10, 33], launch_block=block, launch_grid=grid, launch_waves_per_cu=waves,
                                     launch_alternate=alternate, launch_vec=2)
        _compare(hip, ora, w)
        hip.close()


def test_batched_pushes_with_norms_timer_double_buffer_and_accumulate(hipmod):
    from paper_1509_04210_amd import binding as B
    for P in (77_777, 600_001):
        w = configs.C5.scaled(n_params=P, n_pushes=90)
        hip, ora = _run_both_batched(hipmod, w, [7, 20], flags=B.FLAG_STATS_NORMS | B.FLAG_TIME_KERNELS | B.FLAG_DOUBLE_BUFFER)
        _compare(hip, ora, w)
        st, ref = hip.ps.stats(), ora.ps.norms()
        assert st.norms_valid == 1 and st.kernel_launches == st.n_apply_launches < st.n_updates
        for got, want in [(st.theta_sq, ref["theta_sq"]), (st.v_sq, ref["v_sq"]), (st.gbar_sq, ref["gbar_sq"])]:
            assert abs(got - want) <= 1e-5 * want              # norms are those of the last update of the last launch
        assert st.theta_inf == ref["theta_inf"]
        hip.close()
    hip, ora = _run_both_batched(hipmod, w, [7, 20], flags=B.FLAG_PUSH_ACCUMULATE)     # the plain loop: nothing is fused
    _compare(hip, ora, w)
    assert hip.ps.stats().n_apply_launches == hip.ps.stats().n_updates
    hip.close()


def test_batched_c5_full_size_on_sampled_elements(hipmod):
    """The lambda-softsync workload at 72M parameters, 5000 pushes handed over 16 at a time (16 updates per launch)."""
    w = configs.C5
    idx = _sample_indices(w.n_params, 9, 16384)
    learner, step = w.arrival_trace()
    hip, ora = hipmod.HipServer(w, ring=16 + w.c + 1), OracleServer(w, index=idx)
    lh = replay.replay_batched(hip, learner, step, w.n_learners, [16])
    lo = replay.replay_batched(ora, learner, step, w.n_learners, [16])
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    sel = torch.from_numpy(idx.astype(np.int64)).cuda()
    th, ve = hip.weights()[sel].cpu().numpy(), hip.velocity()[sel].cpu().numpy()
    assert np.abs(th.astype(np.float64) - ora.ps.theta).max() <= TOL * np.abs(ora.ps.theta).max()
    assert np.array_equal(th, ora.ps.theta) and np.array_equal(ve, ora.ps.velocity)
    st = hip.ps.stats()
    assert (st.ts_cur, st.n_pushes, st.sigma_sum, st.sigma_max) == (ora.ps.ts, 5000, ora.ps.sigma_sum, ora.ps.sigma_max)
    assert st.n_apply_launches == -(-5000 // 16)
    assert bool(torch.isfinite(hip.weights()).all())
    hip.close()


# ---------------------------------------------------------------- the C ABI from a plain C++ program, against closed forms
def test_c_abi_from_a_plain_program_matches_closed_forms(hipmod):
    """tests/csrc/abi_gpu_check.cpp: hipMalloc'ed constant vectors pushed through the C ABI (single pushes, a batched
    run, a tree node + root), every result compared with a closed form that binary32 holds exactly.  Neither torch
    nor the oracle is involved: a pin of the HIP path that is independent of both."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "abi_gpu_check")
    assert os.path.exists(exe), f"{exe} is missing: run __graft_entry__.build()"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0 and "abi gpu check ok" in r.stdout, r.stdout + r.stderr


# ---------------------------------------------------------------- the hand-computed traces of tests/golden, on the GPU
@pytest.mark.parametrize("name", ["A", "B", "C", "D", "E"])
@pytest.mark.parametrize("P", [1, 261])
def test_worked_traces_on_the_gpu(hipmod, name, P):
    """tests/golden/worked_traces.txt (timestamps, staleness, clocks, <sigma>, rates and weights computed by hand from
    Sec. 3.1 / Eq. 6 with dyadic numbers) replayed through the C ABI: the same fixture that pins the oracle, checked here
    against the HIP path directly (every element of a constant vector must equal the hand value exactly)."""
    from paper_1509_04210_amd import binding as B
    from tests.test_oracle_protocol import _parse_traces
    t = _parse_traces()[name]
    dev = torch.device("cuda", 0)
    stream = torch.cuda.Stream(device=dev)
    init = torch.zeros(P, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    ps = B.ParameterServer(P, t["lam"], init.data_ptr(), t["n"], B.SOFTSYNC, B.LR_AVG_STALENESS, alpha0=0.5, momentum=t["m"],
                           stream=stream.cuda_stream)
    bufs, out = [], torch.empty(P, dtype=torch.float32, device=dev)
    learner_ts = [0] * t["lam"]
    for p in t["pushes"]:
        l = p["learner"]
        assert learner_ts[l] == p["ts"]
        bufs.append(torch.full((P,), p["g"], dtype=torch.float32, device=dev))       # kept alive: borrowed by the server
        torch.cuda.synchronize()
        rc, r = ps.push_gradient(bufs[-1].data_ptr(), learner_ts[l], l)
        assert rc == 0 and (r.staleness, r.applied, r.ts_after) == (p["sigma"], p["applied"], p["ts_after"])
        if p["applied"]:
            ps.pull_weights(out.data_ptr())
            ps.sync()
            assert bool((out == p["theta"]).all()), (out[:4].tolist(), p["theta"])
        learner_ts[l] = ps.pull_weights(0)
    for idx, sig, stamps in t["clocks"]:
        ts, avg, _ = ps.vector_clock(idx)
        assert ts == stamps and avg == sig
    ps.destroy()


# ---------------------------------------------------------------- randomly drawn configurations (fixed seeds)
@pytest.mark.parametrize("seed", range(24))
def test_random_configurations(hipmod, seed):
    """Protocol, c, rate mode, optimizer, penalty, vector length, launch shape, flags and the way the messages are handed
    over (one by one or in runs) drawn at random from a seed; every combination must give the oracle's bits."""
    from paper_1509_04210_amd import binding as B
    rng = np.random.default_rng(1000 + seed)
    lam = int(rng.integers(1, 41))
    hard = bool(rng.integers(0, 4) == 0)
    n_split = 1 if hard else int(rng.integers(1, lam + 1))
    optimizer = "adagrad" if rng.integers(0, 4) == 0 else "sgd"
    momentum = 0.0 if optimizer == "adagrad" or rng.integers(0, 2) == 0 else float(rng.choice([0.5, 0.9, 0.99]))
    lr_mode = str(rng.choice(["const", "static_n", "avg_staleness", "per_gradient"]))
    base = configs.C2 if hard else configs.C3(1)
    w = _with(base, name=f"random-{seed}", n_params=int(rng.choice([1, 3, 64, 255, 4097, 20_001, 131_075])), n_learners=lam,
              n_split=n_split, protocol="hardsync" if hard else "softsync", lr_mode=lr_mode, momentum=momentum,
              weight_decay=float(rng.choice([0.0, 5e-4])), optimizer=optimizer, adagrad_eps=float(rng.choice([1e-8, 1e-3])),
              alpha0=float(rng.choice([0.001, 0.01, 0.1])), n_pushes=int(rng.integers(1, 6)) * lam + int(rng.integers(0, lam)),
              tail_per=int(rng.choice([0, 100])), straggler_prob=float(rng.choice([0.0, 0.2])), seed=int(rng.integers(1, 1 << 30)))
    flags = int(rng.choice([0, 0, B.FLAG_DOUBLE_BUFFER, B.FLAG_PUSH_ACCUMULATE, B.FLAG_TIME_KERNELS | B.FLAG_CHECK_POINTERS]))
    unroll = int(rng.choice([0, 1, 2, 4]))
    launch = dict(launch_block=int(rng.choice([0, 64, 256, 1024])), launch_unroll=unroll,
                  launch_vec=int(rng.choice([0, 1, 2])) if unroll != 4 else 0, launch_grid=int(rng.choice([0, 0, 1, 5])),
                  launch_waves_per_cu=int(rng.choice([0, 2, 13, 32])), launch_alternate=int(rng.choice([0, 1, 2])))
    if rng.integers(0, 2):
        chunks = [int(x) for x in rng.integers(1, 3 * w.c + 2, size=5)]
        hip, ora = _run_both_batched(hipmod, w, chunks, flags=flags, **launch)
    else:
        hip, ora = _run_both(hipmod, w, flags=flags, **launch)
    _compare(hip, ora, w)
    hip.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_configurations_up_to_a_few_generations_of_waves(hipmod, seed):
    """The same draw over vector lengths from below one tile to 2.2M parameters, where the library picks 8, 4, 2 or 1
    gradient loads per round by itself (and 8, 4 or one-ahead in batched launches), or is told to."""
    from paper_1509_04210_amd import binding as B
    rng = np.random.default_rng(77000 + seed)
    lam = int(rng.integers(1, 41))
    hard = bool(rng.integers(0, 4) == 0)
    n_split = 1 if hard else int(rng.integers(1, lam + 1))
    optimizer = "adagrad" if rng.integers(0, 4) == 0 else "sgd"
    momentum = 0.0 if optimizer == "adagrad" or rng.integers(0, 2) == 0 else float(rng.choice([0.5, 0.9, 0.99]))
    lr_mode = str(rng.choice(["const", "static_n", "avg_staleness", "per_gradient"]))
    base = configs.C2 if hard else configs.C3(1)
    P = int(rng.choice([2, 5, 257, 4097, 65_537, 131_075, 262_147, 300_001, 524_293, 700_001, 1_048_579, 1_300_003, 2_200_001]))
    w = _with(base, name=f"random-short-{seed}", n_params=P, n_learners=lam, n_split=n_split, protocol="hardsync" if hard else "softsync",
              lr_mode=lr_mode, momentum=momentum, weight_decay=float(rng.choice([0.0, 5e-4])), optimizer=optimizer,
              adagrad_eps=float(rng.choice([1e-8, 1e-3])), alpha0=float(rng.choice([0.001, 0.01, 0.1])),
              n_pushes=int(rng.integers(1, 4)) * lam + int(rng.integers(0, lam)), tail_per=int(rng.choice([0, 100])),
              straggler_prob=float(rng.choice([0.0, 0.2])), seed=int(rng.integers(1, 1 << 30)))
    flags = int(rng.choice([0, 0, 0, B.FLAG_DOUBLE_BUFFER, B.FLAG_PUSH_ACCUMULATE, B.FLAG_STATS_NORMS]))
    launch = dict(launch_unroll=int(rng.choice([0, 0, 0, 1, 2, 4, 8])), launch_waves_per_cu=int(rng.choice([0, 0, 13, 32])),
                  launch_alternate=int(rng.choice([0, 1, 2])))
    if rng.integers(0, 2):
        chunks = [int(x) for x in rng.integers(1, 3 * w.c + 2, size=5)]
        hip, ora = _run_both_batched(hipmod, w, chunks, flags=flags, **launch)
    else:
        hip, ora = _run_both(hipmod, w, flags=flags, **launch)
    _compare(hip, ora, w)
    hip.close()


# ---------------------------------------------------------------- bench.py keeps its contract
def test_bench_prints_one_json_line_with_the_agreed_fields(hipmod):
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "8", "--warmup", "2", "--no-extra", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
                "dtype", "data", "config", "roofline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 8 and j["warmup"] == 2 and j["dtype"] == "f32" and j["vs_baseline"] is None
    assert "workload" in j["config"] and "model" not in j["config"]
    roof = j["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12 and 0.3 < roof["frac"] < 1.0
    assert abs(j["value"] * j["ms_per_step"] / 1e3 - 1.0) < 1e-9          # value = steps / wall time
    r2 = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r2.returncode != 0 and "ONE GPU" in r2.stderr


# ---------------------------------------------------------------- many learners: c far beyond one launch's 64 pointers
@pytest.mark.parametrize("lam,n,batched", [(1000, 1, False), (1000, 16, False), (300, 1, True), (1000, 16, True)])
def test_many_learners_on_the_gpu(hipmod, lam, n, batched):
    """c = 1000 (fifteen folds of 64 into the accumulator, then the fused launch), 62 (one launch) and 300, also handed
    over in runs that span several updates."""
    w = _with(configs.C3(1).scaled(n_params=2_051, n_pushes=2 * lam + 40), n_learners=lam, n_split=n, momentum=0.9, weight_decay=5e-4)
    if batched:
        hip, ora = _run_both_batched(hipmod, w, [lam // n + 9, 3 * (lam // n)], ring=4 * lam + 16)
    else:
        hip, ora = _run_both(hipmod, w)
    _compare(hip, ora, w)
    hip.close()
