"""bench.py reports `roofline.traffic` from constants measured with rocprofv3 (FETCH_SIZE / WRITE_SIZE, see
profiles/apply_update_kernel_C4_C5_72M_hbm_traffic.md).  They go stale silently when a kernel changes, so this test pins
them to the algorithmic bytes of the launches they describe: more than 1 % apart means the profile has to be taken again
(or the kernel re-reads or re-writes something)."""
import importlib.util
import os

from synth import configs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_measured_traffic_constants_match_the_algorithmic_bytes():
    b = _bench()
    for name, measured in b.MEASURED_TRAFFIC_BYTES.items():
        want = b.algorithmic_bytes_per_update(configs.ALL[name])
        assert abs(measured - want) <= 0.01 * want, (name, measured, want)
    c5 = configs.C5
    want8 = c5.n_params * (4 * 8 + 16)                       # 8 single-gradient updates in one launch: theta, v once
    assert abs(b.MEASURED_TRAFFIC_BYTES_BATCH8["C5"] - want8) <= 0.01 * want8


def test_algorithmic_bytes_per_update_formula():
    """P * (4c + 8 + 8 when there is a second state vector): the figures quoted for the two 72M workloads."""
    b = _bench()
    assert b.algorithmic_bytes_per_update(configs.C4) == 6_336_000_000          # 88 B/param
    assert b.algorithmic_bytes_per_update(configs.C5) == 1_440_000_000          # 20 B/param
    assert b.algorithmic_bytes_per_update(configs.C4_ADAGRAD) == 6_336_000_000  # AdaGrad's sums take the velocity's place
    assert b.algorithmic_bytes_per_update(configs.C1) == 131072 * 24            # no momentum: 4*4 + 8


def test_the_profile_names_the_commit_it_was_measured_at():
    text = open(os.path.join(ROOT, "profiles", "apply_update_kernel_C4_C5_72M_hbm_traffic.md")).read()
    assert "measured at commit" in text
