"""More GPU parity cases, through the C ABI, against the CPU oracle: the whole 72M-element vector compared element by
element, the weighted fold path (per-gradient weights with more gradients than one launch takes), relayed averages
combined with every server flag, and a reader on a second stream that copies the weights of one timestamp while later
updates are enqueued (the computation / communication buffer pair of Sec. 3.3)."""
import numpy as np
import pytest
import torch

from oracle.adapter import LR_MODE, OPTIMIZER, PROTOCOL, OracleServer
from oracle import OraclePS
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


# ---------------------------------------------------------------- the full 72M-element vector, element by element
class _FullVectorOracle:
    """The oracle on ALL n_params elements.  The gradient of (learner, step) is generated on the device by the input
    generator (whose bit identity with the numpy generator is tested separately) and copied to the host, because hashing
    72M elements per gradient in numpy would take minutes; the arithmetic is the oracle's alone."""

    def __init__(self, w):
        self.w = w
        self.buf = torch.empty(w.n_params, dtype=torch.float32, device="cuda")
        self.host = torch.empty(w.n_params, dtype=torch.float32, pin_memory=True)
        self.ps = OraclePS(self._vector(w.init_key(), w.init_std, 0), w.n_learners, w.n_split, PROTOCOL[w.protocol], LR_MODE[w.lr_mode],
                           w.alpha0, w.lr_scale, w.momentum, w.weight_decay, w.c_override, optimizer=OPTIMIZER[w.optimizer],
                           adagrad_eps=w.adagrad_eps)

    def _vector(self, key, std, tail_per):
        gradgen.fill_device(self.buf.data_ptr(), self.w.n_params, key, std, tail_per, self.w.tail_factor, stream=0)
        torch.cuda.synchronize()
        self.host.copy_(self.buf)
        torch.cuda.synchronize()
        return self.host.numpy()

    def push(self, learner, step, ts):
        w = self.w
        rc, res = self.ps.push(self._vector(w.grad_key(learner, step), w.grad_std, w.tail_per), ts, learner)
        return rc, int(res.staleness), int(res.applied)

    def pull_ts(self):
        return self.ps.ts


@pytest.mark.parametrize("name,n_pushes", [("C4", 18 * 3), ("C5", 20)])
def test_full_vector_parity_at_72m(hipmod, name, n_pushes):
    """The two 72M-parameter workloads in the launch shape bench.py times, a short stretch of their traces (C4: three
    applyUpdates of 18 heavy-tailed gradients with momentum; C5: twenty single-gradient updates with momentum and weight
    penalty), theta and v compared over ALL 72 000 000 elements: within 1e-5 * ||.||_inf, and bit for bit."""
    w = configs.ALL[name].scaled(n_pushes=n_pushes)
    learner, step = w.arrival_trace()
    hip, ora = hipmod.HipServer(w), _FullVectorOracle(w)
    lh = replay.replay(hip, learner, step, w.n_learners)
    lo = replay.replay(ora, learner, step, w.n_learners)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    assert ora.ps.ts == n_pushes // w.c == hip.pull_ts()
    for got, ref, what in ((hip.weights(), ora.ps.theta, "theta"), (hip.velocity(), ora.ps.velocity, "v")):
        got = got.cpu().numpy()
        assert got.shape == ref.shape == (72_000_000,)
        err = np.abs(got.astype(np.float64) - ref).max()
        assert err <= TOL * np.abs(ref).max(), f"{what}: max abs err {err:.3e}"
        assert np.array_equal(got, ref), f"{what} not bit-identical over the whole vector"
    hip.close()
    torch.cuda.empty_cache()


# ---------------------------------------------------------------- weighted fold path: per-gradient weights, c > 64
@pytest.mark.parametrize("c,batched", [(65, False), (130, False), (200, True)])
def test_per_gradient_weights_with_more_gradients_than_one_launch_takes(hipmod, c, batched):
    """Sec. 5.1 footnote mode with c beyond the 64 pointers of one launch: the leading groups are folded into the
    accumulator WITH their staleness weights, the rest goes through the weighted fused kernel."""
    w = _with(configs.C3(1).scaled(n_params=6_007, n_pushes=3 * c + 5), n_learners=c, lr_mode="per_gradient", momentum=0.9,
              weight_decay=5e-4, straggler_prob=0.3)
    learner, step = w.arrival_trace()
    ora = OracleServer(w)
    if batched:
        hip = hipmod.HipServer(w, ring=4 * c + 16)
        chunks = [c // 2 + 3, 2 * c]
        lh = replay.replay_batched(hip, learner, step, w.n_learners, chunks)
        lo = replay.replay_batched(ora, learner, step, w.n_learners, chunks)
    else:
        hip = hipmod.HipServer(w)
        lh = replay.replay(hip, learner, step, w.n_learners)
        lo = replay.replay(ora, learner, step, w.n_learners)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    assert lo["staleness"].max() >= 2                  # some weights really differ from 1
    assert np.array_equal(hip.weights().cpu().numpy(), ora.ps.theta)
    assert np.array_equal(hip.velocity().cpu().numpy(), ora.ps.velocity)
    assert hip.ps.stats().ts_cur == ora.ps.ts == 3
    hip.close()


def test_relayed_averages_with_more_messages_than_one_launch_takes(hipmod):
    """A root that collects 70 relayed averages of 2 gradients per update (c = 140): the fold path with message weights."""
    lam, fan_in = 140, 2
    w = _with(configs.C3(1).scaled(n_params=3_001, n_pushes=lam * 3), n_learners=lam, momentum=0.9)
    learner, step = w.arrival_trace()
    hip = hipmod.HipServer(w, ring=2 * fan_in + 2, avg_ring=lam // fan_in + 4, max_aggregate=fan_in)
    ora = OracleServer(w, max_aggregate=fan_in)
    lh = replay.replay_tree(hip, learner, step, lam, fan_in)
    lo = replay.replay_tree(ora, learner, step, lam, fan_in)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    assert ora.ps.ts >= 2
    assert np.array_equal(hip.weights().cpu().numpy(), ora.ps.theta)
    assert np.array_equal(hip.velocity().cpu().numpy(), ora.ps.velocity)
    hip.close()


# ---------------------------------------------------------------- the tree root under every flag, randomly drawn
def _compare_tree(hip, ora, w):
    th = hip.weights().cpu().numpy()
    assert np.abs(th.astype(np.float64) - ora.ps.theta).max() <= TOL * max(np.abs(ora.ps.theta).max(), 1e-30)
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


@pytest.mark.parametrize("seed", range(16))
def test_random_tree_configurations(hipmod, seed):
    """rudra_ps_push_aggregate with protocol, fan-in, c, rate mode, optimizer, penalty, vector length, launch shape and
    server flags (accumulate at push, double buffer, fused norms, timer, pointer check) drawn from a seed."""
    from paper_1509_04210_amd import binding as B
    rng = np.random.default_rng(5000 + seed)
    fan_in = int(rng.integers(2, 6))
    hard = bool(rng.integers(0, 4) == 0)
    lam = fan_in * int(rng.integers(1, 9)) if hard else int(rng.integers(fan_in, 41))      # hardsync: every node fills
    n_split = 1 if hard else int(rng.integers(1, max(2, lam // fan_in)))
    optimizer = "adagrad" if rng.integers(0, 4) == 0 else "sgd"
    momentum = 0.0 if optimizer == "adagrad" or rng.integers(0, 2) == 0 else float(rng.choice([0.5, 0.9]))
    base = configs.C2 if hard else configs.C3(1)
    w = _with(base, name=f"random-tree-{seed}", n_params=int(rng.choice([3, 255, 4097, 20_001, 131_075])), n_learners=lam,
              n_split=n_split, protocol="hardsync" if hard else "softsync", lr_mode=str(rng.choice(["const", "static_n", "avg_staleness"])),
              momentum=momentum, weight_decay=float(rng.choice([0.0, 5e-4])), optimizer=optimizer,
              alpha0=float(rng.choice([0.001, 0.01, 0.1])), n_pushes=int(rng.integers(2, 6)) * lam + int(rng.integers(0, lam)),
              tail_per=int(rng.choice([0, 100])), straggler_prob=float(rng.choice([0.0, 0.2])), seed=int(rng.integers(1, 1 << 30)))
    flags = [0, B.FLAG_PUSH_ACCUMULATE, B.FLAG_DOUBLE_BUFFER, B.FLAG_STATS_NORMS, B.FLAG_DOUBLE_BUFFER | B.FLAG_STATS_NORMS,
             B.FLAG_PUSH_ACCUMULATE | B.FLAG_STATS_NORMS | B.FLAG_DOUBLE_BUFFER, B.FLAG_TIME_KERNELS | B.FLAG_CHECK_POINTERS,
             B.FLAG_PUSH_ACCUMULATE | B.FLAG_DOUBLE_BUFFER][seed % 8]
    launch = dict(launch_block=int(rng.choice([0, 64, 256])), launch_unroll=int(rng.choice([0, 1, 2])),
                  launch_grid=int(rng.choice([0, 0, 5])), launch_waves_per_cu=int(rng.choice([0, 13, 32])),
                  launch_alternate=int(rng.choice([0, 1, 2])))
    learner, step = w.arrival_trace()
    hip = hipmod.HipServer(w, flags=flags, ring=2 * fan_in + 2, avg_ring=w.c // fan_in + fan_in + 4, max_aggregate=fan_in, **launch)
    ora = OracleServer(w, max_aggregate=fan_in)
    lh = replay.replay_tree(hip, learner, step, lam, fan_in, hardsync=hard)
    lo = replay.replay_tree(ora, learner, step, lam, fan_in, hardsync=hard)
    for k in lo:
        assert np.array_equal(lh[k], lo[k]), k
    assert ora.ps.ts >= 1
    _compare_tree(hip, ora, w)
    if flags & B.FLAG_STATS_NORMS:
        st, ref = hip.ps.stats(), ora.ps.norms()
        assert st.norms_valid == 1
        for got, want in [(st.theta_sq, ref["theta_sq"]), (st.v_sq, ref["v_sq"]), (st.gbar_sq, ref["gbar_sq"])]:
            assert abs(got - want) <= 1e-5 * max(want, 1e-30)
        assert st.theta_inf == ref["theta_inf"]
    hip.close()


def test_plain_sgd_keeps_no_velocity(hipmod):
    from paper_1509_04210_amd import binding as B
    w = configs.C1.scaled(n_params=4099, n_pushes=8)
    hip = hipmod.HipServer(w)
    dst = torch.empty(w.n_params, dtype=torch.float32, device="cuda")
    with pytest.raises(B.RudraError) as e:
        hip.ps.pull_velocity(dst.data_ptr())
    assert e.value.status == B.ESTATE
    hip.close()


# ---------------------------------------------------------------- concurrent pull: a reader on another stream
def _slow_work(stream, big_a, big_b, reps):
    """Keeps `stream` busy for tens of milliseconds (plain device copies of a large tensor)."""
    with torch.cuda.stream(stream):
        for _ in range(reps):
            big_b.copy_(big_a)


@pytest.mark.parametrize("double_buffer", [True, False])
def test_reader_stream_copies_one_timestamp_while_later_updates_are_enqueued(hipmod, double_buffer):
    """rudra_ps_weights_acquire / _release: a second stream is kept busy, then copies the weights of timestamp ts; in the
    meantime the host enqueues the updates ts+1, ts+2 (and ts+3).  The launch that overwrites the buffer of ts must wait
    for the reader: the copy equals the oracle's theta(ts) bit for bit, and so do the final weights."""
    from paper_1509_04210_amd import binding as B
    w = configs.C3(2).scaled(n_params=2_000_003, n_pushes=15 * 5)                 # c = 15, five updates
    learner, step = w.arrival_trace()
    hip = hipmod.HipServer(w, flags=B.FLAG_DOUBLE_BUFFER if double_buffer else 0, ring=15 * 5 + 1)
    ora = OracleServer(w)
    reader = torch.cuda.Stream()
    big_a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")             # 1 GiB
    big_b = torch.empty_like(big_a)
    snapshot = torch.zeros(w.n_params, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    ts_l = [0] * w.n_learners
    view_ts, theta_at_view, ticket = None, None, None
    n_updates = 0
    for i in range(len(learner)):
        l, s = int(learner[i]), int(step[i])
        _, _, applied = hip.push(l, s, ts_l[l])
        ora.push(l, s, ts_l[l])
        ts_l[l] = hip.pull_ts()
        n_updates += applied
        if applied and n_updates == 2:
            _slow_work(reader, big_a, big_b, 40)                                  # the reader is busy for a while ...
            ptr, view_ts, ticket = hip.ps.weights_acquire(reader.cuda_stream)
            assert view_ts == 2 == ora.ps.ts
            theta_at_view = ora.ps.theta.copy()
            with torch.cuda.stream(reader):                                       # ... then copies the weights of timestamp 2
                _copy_from_address(snapshot, ptr, w.n_params, reader)
            assert hip.ps.weights_release(ticket, reader.cuda_stream) == B.OK
    assert n_updates == 5
    hip.ps.sync()
    torch.cuda.synchronize()
    assert np.array_equal(snapshot.cpu().numpy(), theta_at_view), "the reader saw weights of another timestamp"
    assert np.array_equal(hip.weights().cpu().numpy(), ora.ps.theta)
    st = hip.ps.stats()
    assert st.n_weight_acquires == 1 and st.n_reader_waits == 1
    # a release that comes after the overwriting launch was enqueued says so
    _, _, late = hip.ps.weights_acquire(reader.cuda_stream)
    assert hip.ps.weights_release(late, reader.cuda_stream) == B.OK               # nothing enqueued in between: fine
    hip.close()


@pytest.mark.parametrize("double_buffer", [True, False])
def test_pull_on_a_reader_stream_while_later_updates_are_enqueued(hipmod, double_buffer):
    """rudra_ps_pull_weights_on: after the updates 1, 2 and 4 a busy second stream is handed a pull (acquire, copy, release in
    one call) and the host goes on enqueueing updates.  Each copy equals the oracle's theta of its timestamp bit for bit,
    the final weights too, and the launches that overwrite a buffer a copy reads were made to wait for it."""
    from paper_1509_04210_amd import binding as B
    w = configs.C3(2).scaled(n_params=2_000_003, n_pushes=15 * 6)                 # c = 15, six updates
    learner, step = w.arrival_trace()
    hip = hipmod.HipServer(w, flags=B.FLAG_DOUBLE_BUFFER if double_buffer else 0, ring=15 * 6 + 1)
    ora = OracleServer(w)
    reader = torch.cuda.Stream()
    big_a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")             # 1 GiB
    big_b = torch.empty_like(big_a)
    snapshots, wanted = {}, {}
    torch.cuda.synchronize()
    ts_l = [0] * w.n_learners
    n_updates = 0
    for i in range(len(learner)):
        l, s = int(learner[i]), int(step[i])
        _, _, applied = hip.push(l, s, ts_l[l])
        ora.push(l, s, ts_l[l])
        ts_l[l] = hip.pull_ts()
        n_updates += applied
        if applied and n_updates in (1, 2, 4):
            _slow_work(reader, big_a, big_b, 20)                                  # the reader is busy for a while ...
            snapshots[n_updates] = torch.zeros(w.n_params + 1, dtype=torch.float32, device="cuda")
            dst = snapshots[n_updates].data_ptr() + (4 if n_updates == 4 else 0)  # the third pull into a misaligned buffer
            assert hip.ps.pull_weights_on(dst, reader.cuda_stream) == n_updates == ora.ps.ts
            wanted[n_updates] = (ora.ps.theta.copy(), 1 if n_updates == 4 else 0)
    assert n_updates == 6
    hip.ps.sync()
    torch.cuda.synchronize()
    for ts, (theta, off) in wanted.items():
        assert np.array_equal(snapshots[ts].cpu().numpy()[off:off + w.n_params], theta), f"the pull at timestamp {ts} saw other weights"
    assert np.array_equal(hip.weights().cpu().numpy(), ora.ps.theta)
    st = hip.ps.stats()
    assert st.n_reader_waits == 3 and st.n_weight_copies >= 3
    hip.close()


@pytest.mark.parametrize("P,k,own_stream", [(1, 1, False), (5, 3, True), (257, 2, False), (100_003, 18, True), (70_001, 70, False), (2_000_003, 5, True)])
def test_broadcast_writes_the_weights_of_one_timestamp_to_every_learner(hipmod, P, k, own_stream):
    """rudra_ps_broadcast_weights: one launch (two beyond 64 destinations) reads the weights once and writes k copies, on
    the server's stream or on a reader's; further updates are enqueued behind it.  Every copy equals the oracle's theta of
    that timestamp, nothing is written beyond a copy's P floats, and the final weights are the oracle's."""
    from paper_1509_04210_amd import binding as B
    w = configs.C5.scaled(n_params=P, n_pushes=9)                                # c = 1: nine updates
    learner, step = w.arrival_trace()
    hip = hipmod.HipServer(w, flags=B.FLAG_DOUBLE_BUFFER if own_stream else 0)
    ora = OracleServer(w)
    reader = torch.cuda.Stream()
    pad = 8
    dsts = [torch.full((P + 2 * pad,), 7.0, dtype=torch.float32, device="cuda") for _ in range(k)]
    torch.cuda.synchronize()
    ts_l = [0] * w.n_learners
    want = None
    for i in range(len(learner)):
        l, s = int(learner[i]), int(step[i])
        hip.push(l, s, ts_l[l])
        ora.push(l, s, ts_l[l])
        ts_l[l] = hip.pull_ts()
        if i == 3:
            ts = hip.ps.broadcast_weights([d.data_ptr() + 4 * pad for d in dsts], reader.cuda_stream if own_stream else hip.stream.cuda_stream)
            assert ts == 4 == ora.ps.ts
            want = ora.ps.theta.copy()
    hip.ps.sync()
    torch.cuda.synchronize()
    for d in dsts:
        got = d.cpu().numpy()
        assert np.array_equal(got[pad:pad + P], want)
        assert np.all(got[:pad] == 7.0) and np.all(got[pad + P:] == 7.0)
    assert np.array_equal(hip.weights().cpu().numpy(), ora.ps.theta)
    st = hip.ps.stats()
    assert st.n_weight_copies == k + 1 and st.n_reader_waits == (1 if own_stream else 0)
    with pytest.raises(B.RudraError) as e:
        hip.ps.broadcast_weights([dsts[0].data_ptr() + 4], 0)                    # a misaligned destination
    assert e.value.status == B.EINVAL
    hip.close()


@pytest.mark.parametrize("P", [1, 3, 4, 5, 255, 256, 257, 100_003])
def test_pull_copies_every_element_and_nothing_else(hipmod, P):
    """rudra_ps_pull_weights / _pull_velocity through the library's copy kernel (aligned destination) and through the
    runtime's copy (misaligned one): all P elements, and not one float beyond them."""
    w = configs.C5.scaled(n_params=P, n_pushes=7)
    learner, step = w.arrival_trace()
    hip, ora = hipmod.HipServer(w), OracleServer(w)
    replay.replay(hip, learner, step, w.n_learners)
    replay.replay(ora, learner, step, w.n_learners)
    for off in (0, 1):
        for pull, want in ((hip.ps.pull_weights, ora.ps.theta), (hip.ps.pull_velocity, ora.ps.velocity)):
            dst = torch.full((P + 9,), 7.0, dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            pull(dst.data_ptr() + 4 * (4 + off))
            hip.ps.sync()
            got = dst.cpu().numpy()
            assert np.array_equal(got[4 + off:4 + off + P], want)
            assert np.all(got[:4 + off] == 7.0) and np.all(got[4 + off + P:] == 7.0)
    hip.close()


def _copy_from_address(dst, src_ptr, n, stream):
    """hipMemcpyAsync(dst, src_ptr, 4n bytes, device to device) on `stream`."""
    import ctypes
    rt = ctypes.CDLL("libamdhip64.so")
    rt.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    assert rt.hipMemcpyAsync(dst.data_ptr(), src_ptr, 4 * n, 3, stream.cuda_stream) == 0          # 3 = device to device


def test_release_after_the_overwriting_launch_reports_it(hipmod):
    from paper_1509_04210_amd import binding as B
    w = _with(configs.C5.scaled(n_params=10_001, n_pushes=8), n_learners=2, n_split=2)      # c = 1: every push is an update
    for flags, lifetime in ((0, 1), (B.FLAG_DOUBLE_BUFFER, 2)):
        hip = hipmod.HipServer(w, flags=flags)
        reader = torch.cuda.Stream()
        _, ts, ticket = hip.ps.weights_acquire(reader.cuda_stream)
        assert ts == 0
        for k in range(lifetime):
            assert hip.push(0, k, k)[2] == 1
        assert hip.ps.weights_release(ticket, reader.cuda_stream) == B.ESTATE
        assert hip.ps.weights_release(ticket + (1 << 20), reader.cuda_stream) == B.EINVAL     # a ticket from the future
        # on the server's own stream no event is needed at all
        _, _, ticket = hip.ps.weights_acquire(hip.sh)
        assert hip.ps.weights_release(ticket, hip.sh) == B.OK
        assert hip.ps.stats().n_reader_waits == 0
        hip.close()


# ---------------------------------------------------------------- which state vector is loaded non-temporally: never changes a bit
@pytest.mark.parametrize("state_loads", [1, 2, 3])
@pytest.mark.parametrize("double_buffer", [False, True])
def test_state_load_policies_give_the_same_bits(hipmod, state_loads, double_buffer):
    """launch_state_loads is a cache hint on the loads of theta / v: results do not depend on it, one by one or in runs."""
    from paper_1509_04210_amd import binding as B
    from tests.test_gpu_parity import _compare, _run_both, _run_both_batched
    flags = B.FLAG_DOUBLE_BUFFER if double_buffer else 0
    for base, P, n in ((configs.C5, 70_003, 60), (configs.C4, 33_331, 18 * 4), (configs.C4_ADAGRAD, 20_002, 18 * 3)):
        w = base.scaled(n_params=P, n_pushes=n)
        hip, ora = _run_both(hipmod, w, flags=flags, launch_state_loads=state_loads)
        _compare(hip, ora, w)
        hip.close()
    w = configs.C5.scaled(n_params=70_003, n_pushes=90)
    hip, ora = _run_both_batched(hipmod, w, [7, 20, 50], flags=flags, launch_state_loads=state_loads)
    _compare(hip, ora, w)
    hip.close()


# ---------------------------------------------------------------- the phase-aligned kernel (opt-in): same bits as the ordinary one
@pytest.mark.parametrize("case", ["c1-sgd", "c2-momentum-decay", "c7-adagrad-decay", "c41-momentum", "c64-per-gradient-weights", "c70-fold",
                                  "double-buffer", "tree-root", "hardsync"])
def test_phased_kernel_gives_the_oracle_bits(hipmod, case):
    """launch_phased = 2: few persistent waves keep the running sums of their tiles in registers and walk the gradients in
    the outer loop; the ordinary kernel takes what is left of the vector behind the last whole pass.  Vector lengths span
    less than one wave's tiles (all ordinary), one pass with a ragged rest, and several tiles per wave."""
    from paper_1509_04210_amd import binding as B
    from tests.test_gpu_parity import _compare, _run_both
    sizes = [5_003, 6_400 * 7 + 3, 300_001, 1_000_000]       # 25 tiles of 256 parameters make one wave's pass
    base = {"c1-sgd": _with(configs.C3(30).scaled(n_pushes=40)),
            "c2-momentum-decay": _with(configs.C5.scaled(n_pushes=60), n_learners=6, n_split=3),
            "c7-adagrad-decay": _with(configs.C3(4).scaled(n_pushes=7 * 5 + 3), optimizer="adagrad", weight_decay=5e-4),
            "c41-momentum": _with(configs.C4.scaled(n_pushes=41 * 3), n_learners=41),
            "c64-per-gradient-weights": _with(configs.C3(1).scaled(n_pushes=64 * 3 + 5), n_learners=64, lr_mode="per_gradient", momentum=0.9, straggler_prob=0.3),
            "c70-fold": _with(configs.C3(1).scaled(n_pushes=70 * 3), n_learners=70, momentum=0.9, weight_decay=5e-4),
            "double-buffer": _with(configs.C4.scaled(n_pushes=18 * 5)),
            "hardsync": configs.C2.scaled(n_pushes=30 * 4)}
    if case == "tree-root":
        lam, fan_in = 12, 3
        for P in sizes[1:3]:
            w = _with(configs.C4.scaled(n_params=P, n_pushes=lam * 4), n_learners=lam)
            learner, step = w.arrival_trace()
            hip = hipmod.HipServer(w, ring=2 * fan_in + 2, avg_ring=lam // fan_in + 4, max_aggregate=fan_in, launch_phased=2)
            ora = OracleServer(w, max_aggregate=fan_in)
            lh = replay.replay_tree(hip, learner, step, lam, fan_in)
            lo = replay.replay_tree(ora, learner, step, lam, fan_in)
            for k in lo:
                assert np.array_equal(lh[k], lo[k]), k
            _compare_tree(hip, ora, w)
            assert hip.ps.stats().n_phased_launches == ora.ps.ts >= 3
            hip.close()
        return
    flags = B.FLAG_DOUBLE_BUFFER if case == "double-buffer" else 0
    for P in sizes:
        w = base[case].scaled(n_params=P)
        hip, ora = _run_both(hipmod, w, flags=flags, launch_phased=2, launch_alternate=0 if P % 2 else 2)
        _compare(hip, ora, w)
        st = hip.ps.stats()
        assert st.n_phased_launches == (st.n_updates if P >= 6_400 else 0)      # fewer than 25 whole tiles: nothing to phase
        hip.close()


def test_phased_kernel_is_not_used_with_fused_norms_or_by_default(hipmod):
    from paper_1509_04210_amd import binding as B
    from tests.test_gpu_parity import _compare, _run_both
    w = _with(configs.C4.scaled(n_params=300_001, n_pushes=45 * 2), n_learners=45)
    for kw, want in ((dict(launch_phased=2, flags=B.FLAG_STATS_NORMS), 0), (dict(), 0), (dict(launch_phased=1), 0), (dict(launch_phased=2), 2)):
        hip, ora = _run_both(hipmod, w, **kw)
        _compare(hip, ora, w)
        assert hip.ps.stats().n_phased_launches == want
        hip.close()


# ---------------------------------------------------------------- a run that diverges: overflow, infinities and NaN
def _same_bits_or_both_nan(a, b):
    """Bit-identical wherever a number (an infinity included) stands; NaN where the other has NaN.  The sign and payload of a
    NaN that an operation creates are the one thing IEEE 754 leaves to the machine, and the two machines differ there."""
    a, b = np.ascontiguousarray(a, dtype=np.float32), np.ascontiguousarray(b, dtype=np.float32)
    na, nb = np.isnan(a), np.isnan(b)
    return np.array_equal(na, nb) and np.array_equal(a.view(np.uint32)[~na], b.view(np.uint32)[~nb])


@pytest.mark.parametrize("optimizer,batched", [("sgd", False), ("adagrad", False), ("sgd", True)])
def test_a_diverging_run_overflows_like_the_oracle(hipmod, optimizer, batched):
    """Too large a rate on stale gradients makes training diverge (Sec. 5.1).  Here the numbers themselves run out
    (weights of 1e37 and gradients of 7e37 overflow in the sum of an update, in the step and in the squared-gradient sums;
    inf - inf and inf / inf then give NaN).  The kernel must produce
    infinities and NaN exactly where the CPU does, and the same bits everywhere else."""
    from tests.test_gpu_parity import _run_both, _run_both_batched
    w = _with(configs.C3(2).scaled(n_params=30_003, n_pushes=15 * 4), init_std=1e37, grad_std=7e37, alpha0=0.75,
              momentum=0.9 if optimizer == "sgd" else 0.0, weight_decay=0.0 if optimizer == "sgd" else 0.5, optimizer=optimizer,
              adagrad_eps=0.0 if optimizer == "sgd" else 1e-8)
    hip, ora = _run_both_batched(hipmod, w, [40, 15, 35]) if batched else _run_both(hipmod, w)
    theta, state = ora.ps.theta, ora.ps.velocity
    assert np.isnan(theta).mean() > 0.1 and np.isfinite(theta).mean() > 0.1                  # the case has all three kinds of
    assert np.isinf(theta).mean() > 0.1 or np.isinf(state).mean() > 0.1                      # values, each in quantity
    assert _same_bits_or_both_nan(hip.weights().cpu().numpy(), theta)
    assert _same_bits_or_both_nan(hip.velocity().cpu().numpy(), state)
    hip.close()
