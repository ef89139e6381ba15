"""Do the pins bite?  Plausible mistakes are planted in COPIES of the oracle's source (a dropped term, a wrong
sign, an off-by-one, a fused operation, another reading of the momentum rule ...); each mutant is compiled and
the oracle's pin tests are run against it in a subprocess.  Every mutant must fail at least one pin, and the
unmodified copy must pass.  CPU only."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "rudra_oracle.c")).read()
PINS = ["tests/test_oracle_protocol.py", "tests/test_oracle_update.py", "tests/test_oracle_tree.py"]

MUTANTS = {
    "mean_not_divided_by_c": ("real gbar = o->acc[k] * inv_c;", "real gbar = o->acc[k];"),
    "update_sign": ("o->theta[k] = o->theta[k] - step;", "o->theta[k] = o->theta[k] + step;"),
    "momentum_sign": ("o->vel[k] = keep - step;", "o->vel[k] = keep + step;"),
    "weight_penalty_dropped": ("gbar = gbar + penalty;", "gbar = gbar;"),
    "staleness_off_by_one": ("{ return o->ts_cur - ts; }", "{ return o->ts_cur + 1 - ts; }"),
    "rate_divisor_not_clamped": ("lr = lr / (avg_sigma > 1.0 ? avg_sigma : 1.0);", "lr = lr / (avg_sigma > 0.0 ? avg_sigma : 1.0);"),
    "c_rounded_up": ("return cfg->n_learners / cfg->n_split;", "return (cfg->n_learners + cfg->n_split - 1) / cfg->n_split;"),
    "rate_outside_velocity": ("o->vel[k] = keep - step;\n      o->theta[k] = o->theta[k] + o->vel[k];",
                              "o->vel[k] = keep - gbar; (void)step;\n      o->theta[k] = o->theta[k] + lr * o->vel[k];"),
    "duplicate_check_dropped": ("if (learner >= 0 && o->seen[learner])", "if (0 && o->seen[learner])"),
    "sum_not_restarted": ("o->acc[k] = (o->count == 0) ? (real)grad[k] : o->acc[k] + (real)grad[k];",
                          "o->acc[k] = (o->n_pushes == 0) ? (real)grad[k] : o->acc[k] + (real)grad[k];"),
    "fused_multiply_add": ("o->vel[k] = keep - step;", "o->vel[k] = (real)((double)m * (double)o->vel[k] - (double)lr * (double)gbar);"),
    "per_gradient_weight_dropped": ("(real)(float)(1.0 / div) : (real)(1.0 / div)", "(real)1 : (real)1"),
    "static_rate_divides_by_c": ("lr = lr / (double)o->cfg.n_split;", "lr = lr / (double)o->c;"),
    "stale_hardsync_accepted": ("if (ts != o->ts_cur) { o->n_rejected++; return OR_EHARDSYNC_STALE; }", ""),
    "average_staleness_uses_sum": ("(double)o->sigma_sum_open / (double)o->count;", "(double)o->sigma_sum_open;"),
    "relayed_average_counts_once": ("  const real w = (real)m;", "  const real w = (real)1;"),
    "mean_over_c_not_over_collected": ("const real inv_c = (real)1 / (real)o->count;", "const real inv_c = (real)1 / (real)o->c;"),
    "leaf_relays_the_sum": ("out[i] = (float)(s * inv_k);", "out[i] = (float)s;"),
    "update_waits_for_exactly_c": ("if (o->count < o->c) return OR_OK;", "if (o->count != o->c) return OR_OK;"),
    "adagrad_accumulator_not_summed": ("o->vel[k] = o->vel[k] + sq;", "o->vel[k] = sq;"),
    "adagrad_eps_inside_the_root": ("real denom = root + (real)o->cfg.adagrad_eps;", "real denom = (real)sqrt((double)o->vel[k] + (double)o->cfg.adagrad_eps);"),
    "adagrad_penalty_after_accumulator": ("      real sq = gbar * gbar;", "      real sq = (gbar - wd * o->theta[k]) * (gbar - wd * o->theta[k]);"),
    "timestamp_in_clock_is_staleness": ("o->open_clock[o->count] = ts;", "o->open_clock[o->count] = sigma;"),
    "future_timestamp_accepted": ("  if (ts > o->ts_cur) { o->n_rejected++; return OR_EFUTURE_TS; }       /* ts_j >= ts_i */", ""),
    "mean_by_division": ("real gbar = o->acc[k] * inv_c;", "real gbar = o->acc[k] / (real)o->count; (void)inv_c;"),
    "timestamp_advances_per_gradient": ("  o->ts_cur += 1;                                  /* the timestamp counts the weight updates (Sec. 3.1) */",
                                        "  o->ts_cur += o->count;"),
    "contributors_not_forgotten_after_the_step": ("  memset(o->seen, 0, o->cfg.n_learners);", ""),
    "caller_factor_ignored": ("double lr = (double)o->cfg.alpha0 * (double)o->cfg.lr_scale;", "double lr = (double)o->cfg.alpha0;"),
    "histogram_counts_timestamps": ("  int rc = count_staleness(o, sigma);", "  int rc = count_staleness(o, ts);"),
    "gradient_norm_without_the_penalty": ("    gbar_sq += (double)gbar * (double)gbar;", "    gbar_sq += (double)(o->acc[k] * inv_c) * (double)(o->acc[k] * inv_c);"),
    "hardsync_average_may_overshoot": ("  if (o->cfg.protocol == PROTO_HARDSYNC && (uint64_t)o->count + m > o->c) { o->n_rejected++; return OR_EHARDSYNC_DUP; }", ""),
    "adagrad_root_of_the_mean_square": ("      real denom = root + (real)o->cfg.adagrad_eps;", "      real denom = root / (real)sqrt((double)(o->n_updates + 1)) + (real)o->cfg.adagrad_eps;"),
}


def _run(name, tmp):
    src = SRC
    if name != "unmodified":
        old, new = MUTANTS[name]
        assert src.count(old) == 1, f"mutant {name}: pattern occurs {src.count(old)} times"
        src = src.replace(old, new)
    c_path = os.path.join(tmp, f"{name}.c")
    with open(c_path, "w") as f:
        f.write(src)
    lib = oracle.build(force=True, src=c_path, out=os.path.join(tmp, f"lib{name}.so"))
    env = dict(os.environ, RUDRA_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=600)
    return name, r.returncode, r.stdout[-400:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    names = ["unmodified", *MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda n: _run(n, str(tmp_path)), names))
    survivors = []
    for name, rc, tail in results:
        if name == "unmodified":
            assert rc == 0, "the unmodified copy must pass its pins:\n" + tail
        elif rc == 0:
            survivors.append(name)
    assert not survivors, f"mutants no pin caught: {survivors}"
