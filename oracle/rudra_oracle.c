/*
 * Rudra parameter-server update path -- sequential CPU ORACLE.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests/, __graft_entry__.smoke()
 * and bench.py's cpu_baseline leg may build, load or call this file.  The HIP
 * library shares no code with it and neither includes the other.
 *
 * It executes the paper's parameter-server protocol literally, one message at
 * a time, on one thread (Sec. 3.2 "Parameter Server": messages are handled one
 * by one).  Nothing is blocked, fused, vectorised or reordered by hand.
 *
 * Built twice from this one source:
 *   -DORACLE_REAL=float   -DORACLE_PREFIX=oracle32_   the parity reference.  The
 *        paper stores the model in 32-bit floating point (Sec. 4.2), so state
 *        and arithmetic are IEEE binary32, every operation rounded on its own
 *        (compile with -ffp-contract=off; no fused multiply-add anywhere).
 *   -DORACLE_REAL=double  -DORACLE_PREFIX=oracle64_   the same steps in binary64;
 *        used to bound how far binary32 drifts from exact arithmetic and to
 *        compare against library routines that run in binary64.
 *
 * What the paper fixes, and where:
 *   timestamp      scalar clock, starts at 0, +1 per weight update; a gradient
 *                  carries the timestamp of the weights it was computed from
 *                  (Sec. 3.1 "Timestamp")
 *   staleness      gradient stamped i arriving when the weights are stamped j>=i
 *                  has sigma = j - i (Sec. 3.1 "sigma")
 *   vector clock   the timestamps of the gradients that trigger update i-1 -> i;
 *                  <sigma> = (i-1) - mean(i_1..i_c)  (Sec. 3.1, Eq. 2 "avg staleness")
 *   hardsync       exactly one gradient per learner per step, all lambda averaged,
 *                  so sigma = 0 for every gradient (Sec. 3.1, Eq. 3)
 *   n-softsync     update after c = floor(lambda/n) gradients, averaged
 *                  (Sec. 3.1, Eq. 5); n = lambda is the async rule (Eq. 4)
 *   sumGradients   gradients are added up as they come in (Sec. 2)
 *   applyUpdate    multiply the accumulated gradient by the learning rate and
 *                  update the weights (Sec. 2, Eq. 1c)
 *   learning rate  hardsync: alpha0 times a caller-known factor sqrt(lambda*mu/B);
 *                  softsync: alpha0 divided by the staleness,
 *                  alpha = alpha0/<sigma> = alpha0/n (Sec. 3.2, Sec. 5.1 Eq. 6)
 *   momentum 0.9, weight penalty 5e-4: named, no formula printed (Sec. 4.2).
 *   AdaGrad: named for the ImageNet 1-softsync runs (Sec. 5.5), no formula or epsilon printed.
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - the divisor of the staleness-modulated rate is max(1, <sigma>): the paper's
 *     hardsync rule divides by nothing and n >= 1, so the rate is never raised
 *     above alpha0 and <sigma> = 0 cannot divide;
 *   - the update needs c gradients or more: messages arrive one at a time, so it fires
 *     when the count reaches exactly c;
 *   - gradients are added in arrival order, the first one initialising the sum;
 *   - the average is sum * (1/c), with 1/c rounded once to the working precision;
 *   - momentum: v <- m*v - alpha*gbar ; theta <- theta + v   (rate inside the
 *     velocity, the convention of the networks the paper says it follows);
 *   - weight penalty: L2, gbar <- gbar + wd*theta before rate and momentum;
 *   - tree of servers (Sec. 3.3): a node relays (g_1+...+g_k)*(1/k) together with its constituents' timestamps;
 *     the root adds m*avg for a message standing for m gradients, fires once c or more are in and divides by the
 *     number collected (the paper says neither which timestamp a relayed average carries nor when a node relays);
 *   - per-gradient modulation (Sec. 5.1 footnote, not explored by the paper):
 *     each arriving gradient is scaled by 1/max(1, sigma_l) before it is added;
 *     the update then uses alpha0*lr_scale.
 *   - AdaGrad: the cited diagonal rule, h <- h + gbar^2, theta <- theta - alpha*gbar/(sqrt(h)+eps),
 *     the weight penalty added to gbar first, alpha the staleness-modulated rate, no momentum.
 *   PARITY UNPINNED BY THE PAPER: the momentum, weight-penalty and AdaGrad formulas, the tree's
 *   bookkeeping and the per-gradient modulation (no formula is printed); they are pinned only against
 *   library SGD / Adagrad routines and closed forms.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL float
#endif
#ifndef ORACLE_PREFIX
#define ORACLE_PREFIX oracle32_
#endif
#define OR_CAT2(a, b) a##b
#define OR_CAT(a, b) OR_CAT2(a, b)
#define FN(name) OR_CAT(ORACLE_PREFIX, name)

typedef ORACLE_REAL real;

enum { PROTO_HARDSYNC = 0, PROTO_SOFTSYNC = 1 };
enum { LR_CONST = 0, LR_STATIC_N = 1, LR_AVG_STALENESS = 2, LR_PER_GRADIENT = 3 };
enum { OPT_SGD = 0, OPT_ADAGRAD = 1 };
enum {
  OR_OK = 0,
  OR_EINVAL = -1,
  OR_EFUTURE_TS = -2,
  OR_EHARDSYNC_STALE = -3,
  OR_EHARDSYNC_DUP = -4,
  OR_ENOMEM = -5
};

typedef struct {
  uint64_t n_params;   /* P */
  uint32_t n_learners; /* lambda */
  uint32_t n_split;    /* n in [1, lambda]; ignored under hardsync */
  uint32_t c_override; /* 0 => c from the protocol */
  int32_t protocol;
  int32_t lr_mode;
  float alpha0, lr_scale, momentum, weight_decay;
  int32_t optimizer;   /* OPT_SGD (with optional momentum) or OPT_ADAGRAD */
  float adagrad_eps;   /* added to sqrt(h) */
  uint32_t max_aggregate; /* largest number of learner gradients one relayed message may stand for (0 or 1: none) */
} oracle_config;

typedef struct {
  uint64_t staleness; /* sigma of this gradient */
  uint64_t ts_after;  /* weight timestamp after this message was handled */
  uint32_t pending;   /* gradients waiting for the next update */
  int32_t applied;    /* 1 if this message triggered applyUpdate */
  float lr_used;      /* rate of the triggered update (0 if none) */
} oracle_push_result;

typedef struct {
  oracle_config cfg;
  uint32_t c;
  real *theta, *vel, *acc; /* vel: momentum velocity, or AdaGrad's sum of squared gradients h */
  uint64_t ts_cur;
  uint32_t count;
  uint64_t sigma_sum_open; /* sum of sigma over the open clock */
  uint32_t clock_cap;      /* c + max_aggregate - 1: an update can overshoot c by one message */
  uint64_t *open_clock;    /* clock_cap entries */
  uint8_t *seen;           /* hardsync: learner already contributed this step */
  /* log of every closed vector clock */
  uint64_t n_updates, cap_updates;
  uint64_t *clocks;        /* n_updates * clock_cap timestamps (the first counts[u] of each row are used) */
  uint32_t *counts;        /* gradients in each update */
  double *avg_staleness;   /* per update */
  float *lr_used;          /* per update */
  /* staleness histogram and counters */
  uint64_t *hist;
  uint64_t hist_len;
  uint64_t n_pushes, n_rejected, sigma_sum_all, sigma_max;
  double last_gbar_sq;     /* sum over k of gbar[k]^2 of the latest update, in binary64 */
} oracle_t;

static uint32_t gradients_per_update(const oracle_config *cfg) {
  if (cfg->c_override) return cfg->c_override;
  if (cfg->protocol == PROTO_HARDSYNC) return cfg->n_learners; /* Eq. 3 */
  return cfg->n_learners / cfg->n_split;                       /* Eq. 5: floor(lambda/n) */
}

uint32_t FN(gradients_per_update)(const oracle_config *cfg) { return gradients_per_update(cfg); }

void FN(destroy)(oracle_t *o) {
  if (!o) return;
  free(o->theta); free(o->vel); free(o->acc); free(o->open_clock); free(o->seen);
  free(o->clocks); free(o->counts); free(o->avg_staleness); free(o->lr_used); free(o->hist);
  free(o);
}

/* init_weights: P binary32 values (the paper's storage type), converted to the
 * working precision.  Velocity starts at zero. */
int FN(create)(const oracle_config *cfg, const float *init_weights, oracle_t **out) {
  if (!cfg || !init_weights || !out) return OR_EINVAL;
  if (cfg->n_params == 0 || cfg->n_learners == 0) return OR_EINVAL;
  if (cfg->protocol != PROTO_HARDSYNC && cfg->protocol != PROTO_SOFTSYNC) return OR_EINVAL;
  if (cfg->lr_mode < LR_CONST || cfg->lr_mode > LR_PER_GRADIENT) return OR_EINVAL;
  if (cfg->protocol == PROTO_SOFTSYNC && (cfg->n_split < 1 || cfg->n_split > cfg->n_learners))
    return OR_EINVAL;
  if (cfg->lr_mode == LR_STATIC_N && cfg->n_split < 1) return OR_EINVAL; /* alpha0/n (Eq. 6) needs n >= 1 */
  if (cfg->lr_scale == 0.0f) return OR_EINVAL;   /* the caller-known factor multiplies alpha0: 1 when there is none */
  if (gradients_per_update(cfg) == 0) return OR_EINVAL;
  if (cfg->optimizer != OPT_SGD && cfg->optimizer != OPT_ADAGRAD) return OR_EINVAL;
  if (cfg->optimizer == OPT_ADAGRAD && (cfg->momentum != 0.0f || !(cfg->adagrad_eps >= 0.0f))) return OR_EINVAL;
  oracle_t *o = (oracle_t *)calloc(1, sizeof(oracle_t));
  if (!o) return OR_ENOMEM;
  o->cfg = *cfg;
  o->c = gradients_per_update(cfg);
  uint64_t P = cfg->n_params;
  o->theta = (real *)malloc(P * sizeof(real));
  o->vel = (real *)calloc(P, sizeof(real));
  o->acc = (real *)calloc(P, sizeof(real));
  o->clock_cap = o->c + (cfg->max_aggregate > 1 ? cfg->max_aggregate - 1 : 0);
  o->open_clock = (uint64_t *)calloc(o->clock_cap, sizeof(uint64_t));
  o->seen = (uint8_t *)calloc(cfg->n_learners, 1);
  o->hist_len = 16;
  o->hist = (uint64_t *)calloc(o->hist_len, sizeof(uint64_t));
  if (!o->theta || !o->vel || !o->acc || !o->open_clock || !o->seen || !o->hist) {
    FN(destroy)(o);
    return OR_ENOMEM;
  }
  for (uint64_t k = 0; k < P; ++k) o->theta[k] = (real)init_weights[k];
  *out = o;
  return OR_OK;
}

static int log_update(oracle_t *o, double avg_sigma, float lr) {
  if (o->n_updates == o->cap_updates) {
    uint64_t cap = o->cap_updates ? 2 * o->cap_updates : 64;
    uint64_t *cl = (uint64_t *)realloc(o->clocks, cap * o->clock_cap * sizeof(uint64_t));
    if (cl) o->clocks = cl;
    uint32_t *cn = (uint32_t *)realloc(o->counts, cap * sizeof(uint32_t));
    if (cn) o->counts = cn;
    double *av = (double *)realloc(o->avg_staleness, cap * sizeof(double));
    if (av) o->avg_staleness = av;
    float *lu = (float *)realloc(o->lr_used, cap * sizeof(float));
    if (lu) o->lr_used = lu;
    if (!cl || !cn || !av || !lu) return OR_ENOMEM;
    o->cap_updates = cap;
  }
  memcpy(o->clocks + o->n_updates * o->clock_cap, o->open_clock, o->clock_cap * sizeof(uint64_t));
  o->counts[o->n_updates] = o->count;
  o->avg_staleness[o->n_updates] = avg_sigma;
  o->lr_used[o->n_updates] = lr;
  o->n_updates += 1;
  return OR_OK;
}

static int count_staleness(oracle_t *o, uint64_t sigma) {
  if (sigma >= o->hist_len) {
    uint64_t len = o->hist_len;
    while (len <= sigma) len *= 2;
    uint64_t *h = (uint64_t *)realloc(o->hist, len * sizeof(uint64_t));
    if (!h) return OR_ENOMEM;
    memset(h + o->hist_len, 0, (len - o->hist_len) * sizeof(uint64_t));
    o->hist = h;
    o->hist_len = len;
  }
  o->hist[sigma] += 1;
  return OR_OK;
}

/* applyUpdate over the whole vector, one element after the other.
 * acc holds the sum of the c gradients of this update. */
static void apply_update(oracle_t *o, real lr) {
  const uint64_t P = o->cfg.n_params;
  const real inv_c = (real)1 / (real)o->count;   /* the mean is over the gradients actually collected (= c unless a
                                                     relayed average made the count overshoot) */
  const real m = (real)o->cfg.momentum;
  const real wd = (real)o->cfg.weight_decay;
  double gbar_sq = 0.0;
  for (uint64_t k = 0; k < P; ++k) {
    real gbar = o->acc[k] * inv_c;                 /* Eq. 5: (1/c) * sum */
    if (wd != (real)0) {
      real penalty = wd * o->theta[k];             /* L2 weight penalty, Sec. 4.2 */
      gbar = gbar + penalty;
    }
    gbar_sq += (double)gbar * (double)gbar;
    if (o->cfg.optimizer == OPT_ADAGRAD) {
      /* AdaGrad (Duchi, Hazan, Singer 2011, diagonal form; named in Sec. 5.5 for the ImageNet 1-softsync runs):
       * h <- h + gbar^2 ; theta <- theta - lr * gbar / (sqrt(h) + eps).  h lives in vel[]. */
      real sq = gbar * gbar;
      o->vel[k] = o->vel[k] + sq;
      real root = (sizeof(real) == sizeof(float)) ? (real)sqrtf((float)o->vel[k]) : (real)sqrt((double)o->vel[k]);
      real denom = root + (real)o->cfg.adagrad_eps;
      real step = lr * gbar;
      real scaled = step / denom;
      o->theta[k] = o->theta[k] - scaled;
    } else if (m != (real)0) {                     /* momentum SGD, Sec. 4.2 */
      real keep = m * o->vel[k];
      real step = lr * gbar;
      o->vel[k] = keep - step;
      o->theta[k] = o->theta[k] + o->vel[k];
    } else {                                       /* Eq. 1c */
      real step = lr * gbar;
      o->theta[k] = o->theta[k] - step;
    }
  }
  o->last_gbar_sq = gbar_sq;
}

/* applyUpdate when enough gradients have been collected: rate from this update's clock, update, clock closed. */
static int maybe_update(oracle_t *o, int *applied, float *lr_used) {
  *applied = 0;
  *lr_used = 0.0f;
  if (o->count < o->c) return OR_OK;               /* fewer than c so far: wait (Sec. 3.1) */
  /* <sigma> = (i-1) - mean(i_1..i_count) with i-1 = ts_cur, i.e. mean of (ts_cur - i_k), Eq. 2 */
  const double avg_sigma = (double)o->sigma_sum_open / (double)o->count;
  double lr = (double)o->cfg.alpha0 * (double)o->cfg.lr_scale;
  if (o->cfg.lr_mode == LR_STATIC_N) lr = lr / (double)o->cfg.n_split;          /* alpha0/n */
  else if (o->cfg.lr_mode == LR_AVG_STALENESS) lr = lr / (avg_sigma > 1.0 ? avg_sigma : 1.0);
  *lr_used = (float)lr;   /* the rate is a binary32 number in both builds' logs */
  real lr_work = (sizeof(real) == sizeof(float)) ? (real)*lr_used : (real)lr;
  apply_update(o, lr_work);
  int rc = log_update(o, avg_sigma, *lr_used);
  if (rc != OR_OK) return rc;
  o->ts_cur += 1;                                  /* the timestamp counts the weight updates (Sec. 3.1) */
  o->count = 0;
  o->sigma_sum_open = 0;
  memset(o->seen, 0, o->cfg.n_learners);
  *applied = 1;
  return OR_OK;
}

/* sigma = j - i for a gradient stamped i arriving when the weights are stamped j (Sec. 3.1) */
static uint64_t staleness_of(const oracle_t *o, uint64_t ts) { return o->ts_cur - ts; }

static int note_gradient(oracle_t *o, uint64_t ts) {   /* clock, staleness statistics, count */
  const uint64_t sigma = staleness_of(o, ts);
  int rc = count_staleness(o, sigma);
  if (rc != OR_OK) return rc;
  o->open_clock[o->count] = ts;
  o->count += 1;
  o->sigma_sum_open += sigma;
  o->sigma_sum_all += sigma;
  if (sigma > o->sigma_max) o->sigma_max = sigma;
  o->n_pushes += 1;
  return OR_OK;
}

/* pushGradient as the server sees it: one gradient (P binary32 values) stamped ts
 * from learner `learner` (-1 = anonymous).  A rejected message changes nothing. */
int FN(push)(oracle_t *o, const float *grad, uint64_t ts, int32_t learner, oracle_push_result *res) {
  if (!o || !grad) return OR_EINVAL;
  if (learner < -1 || learner >= (int32_t)o->cfg.n_learners) { o->n_rejected++; return OR_EINVAL; }
  if (ts > o->ts_cur) { o->n_rejected++; return OR_EFUTURE_TS; }       /* ts_j >= ts_i */
  if (o->cfg.protocol == PROTO_HARDSYNC) {
    if (ts != o->ts_cur) { o->n_rejected++; return OR_EHARDSYNC_STALE; } /* sigma must be 0 under hardsync */
    if (learner >= 0 && o->seen[learner]) { o->n_rejected++; return OR_EHARDSYNC_DUP; } /* exactly one */
  }
  const uint64_t sigma = staleness_of(o, ts);

  /* sumGradients: every arriving gradient is added to the running sum, in arrival order */
  const uint64_t P = o->cfg.n_params;
  if (o->cfg.lr_mode == LR_PER_GRADIENT) {
    /* Sec. 5.1 footnote: a staler gradient gets a smaller rate */
    const double div = sigma > 1 ? (double)sigma : 1.0;
    const real w = (sizeof(real) == sizeof(float)) ? (real)(float)(1.0 / div) : (real)(1.0 / div);
    for (uint64_t k = 0; k < P; ++k) {
      real scaled = w * (real)grad[k];
      o->acc[k] = (o->count == 0) ? scaled : o->acc[k] + scaled;
    }
  } else {
    for (uint64_t k = 0; k < P; ++k)
      o->acc[k] = (o->count == 0) ? (real)grad[k] : o->acc[k] + (real)grad[k];
  }
  int rc = note_gradient(o, ts);
  if (rc != OR_OK) return rc;
  if (learner >= 0 && o->cfg.protocol == PROTO_HARDSYNC) o->seen[learner] = 1;

  int applied;
  float lr_used;
  rc = maybe_update(o, &applied, &lr_used);
  if (rc != OR_OK) return rc;
  if (res) {
    res->staleness = sigma;
    res->ts_after = o->ts_cur;
    res->pending = o->count;
    res->applied = applied;
    res->lr_used = lr_used;
  }
  return OR_OK;
}

/* A node of the parameter-server tree (Sec. 3.3): it averages the gradients sent by its learners and relays the
 * average to its parent.  out = (g_1 + g_2 + ... + g_k) * (1/k), added in arrival order in the working precision,
 * stored as binary32 (a relayed message is a model-sized binary32 vector like any other). */
void FN(leaf_mean)(const float *const *grads, uint32_t k, uint64_t n, float *out) {
  const real inv_k = (real)1 / (real)k;
  for (uint64_t i = 0; i < n; ++i) {
    real s = (real)grads[0][i];
    for (uint32_t l = 1; l < k; ++l) s = s + (real)grads[l][i];
    out[i] = (float)(s * inv_k);
  }
}

/* The root receiving a relayed average that stands for m learner gradients with timestamps ts[0..m-1] (reading:
 * the message carries its constituents' timestamps, so staleness, vector clock and <sigma> stay exact, Eq. 2).
 * It counts as m gradients: the sum takes m*avg, the update fires once at least c gradients are in and averages
 * over the number actually collected.  res->staleness reports the largest constituent staleness. */
int FN(push_aggregate)(oracle_t *o, const float *avg, const uint64_t *ts, uint32_t m, oracle_push_result *res) {
  if (!o || !avg || !ts || m == 0) return OR_EINVAL;
  const uint32_t max_m = o->cfg.max_aggregate > 1 ? o->cfg.max_aggregate : 1;
  if (m > max_m || o->cfg.lr_mode == LR_PER_GRADIENT) { o->n_rejected++; return OR_EINVAL; }
  /* hardsync: exactly one gradient from each of the lambda learners is averaged (Sec. 3.1, Eq. 3), so a relayed
   * average may complete the step but never overshoot it; "c or more" is the n-softsync trigger (Eq. 5) */
  if (o->cfg.protocol == PROTO_HARDSYNC && (uint64_t)o->count + m > o->c) { o->n_rejected++; return OR_EHARDSYNC_DUP; }
  for (uint32_t j = 0; j < m; ++j) {
    if (ts[j] > o->ts_cur) { o->n_rejected++; return OR_EFUTURE_TS; }
    if (o->cfg.protocol == PROTO_HARDSYNC && ts[j] != o->ts_cur) { o->n_rejected++; return OR_EHARDSYNC_STALE; }
  }
  const uint64_t P = o->cfg.n_params;
  const real w = (real)m;
  for (uint64_t k = 0; k < P; ++k) {
    real scaled = w * (real)avg[k];
    o->acc[k] = (o->count == 0) ? scaled : o->acc[k] + scaled;
  }
  uint64_t worst = 0;
  for (uint32_t j = 0; j < m; ++j) {
    if (staleness_of(o, ts[j]) > worst) worst = staleness_of(o, ts[j]);
    int rc = note_gradient(o, ts[j]);
    if (rc != OR_OK) return rc;
  }
  int applied;
  float lr_used;
  int rc = maybe_update(o, &applied, &lr_used);
  if (rc != OR_OK) return rc;
  if (res) {
    res->staleness = worst;
    res->ts_after = o->ts_cur;
    res->pending = o->count;
    res->applied = applied;
    res->lr_used = lr_used;
  }
  return OR_OK;
}

/* pullWeights: the weights and their timestamp; dst == NULL is the timestamp
 * inquiry a learner makes first (Sec. 3.2 "Learner"). dst receives binary32. */
uint64_t FN(pull)(const oracle_t *o, float *dst) {
  if (dst) for (uint64_t k = 0; k < o->cfg.n_params; ++k) dst[k] = (float)o->theta[k];
  return o->ts_cur;
}

/* raw state access for the tests (working precision) */
const real *FN(theta)(const oracle_t *o) { return o->theta; }
const real *FN(velocity)(const oracle_t *o) { return o->vel; }
uint64_t FN(n_updates)(const oracle_t *o) { return o->n_updates; }
uint64_t FN(n_pushes)(const oracle_t *o) { return o->n_pushes; }
uint64_t FN(n_rejected)(const oracle_t *o) { return o->n_rejected; }
uint32_t FN(pending)(const oracle_t *o) { return o->count; }
uint32_t FN(c)(const oracle_t *o) { return o->c; }
uint64_t FN(sigma_sum)(const oracle_t *o) { return o->sigma_sum_all; }
uint64_t FN(sigma_max)(const oracle_t *o) { return o->sigma_max; }
uint64_t FN(hist_len)(const oracle_t *o) { return o->hist_len; }
const uint64_t *FN(hist)(const oracle_t *o) { return o->hist; }
const uint64_t *FN(clocks)(const oracle_t *o) { return o->clocks; }
const uint32_t *FN(counts)(const oracle_t *o) { return o->counts; }
uint32_t FN(clock_cap)(const oracle_t *o) { return o->clock_cap; }
const double *FN(avg_staleness)(const oracle_t *o) { return o->avg_staleness; }
const float *FN(lr_log)(const oracle_t *o) { return o->lr_used; }
int FN(set_alpha0)(oracle_t *o, float alpha0) { if (!o) return OR_EINVAL; o->cfg.alpha0 = alpha0; return OR_OK; }

/* Statistics of the current state, summed in binary64 in index order:
 * out[0] = sum theta^2, out[1] = max |theta|, out[2] = sum v^2,
 * out[3] = sum gbar^2 of the latest update (gbar as multiplied by the rate). */
void FN(norms)(const oracle_t *o, double *out) {
  double s2 = 0.0, mx = 0.0, v2 = 0.0;
  for (uint64_t k = 0; k < o->cfg.n_params; ++k) {
    double t = (double)o->theta[k];
    double a = t < 0 ? -t : t;
    s2 += t * t;
    if (a > mx) mx = a;
    double v = (double)o->vel[k];
    v2 += v * v;
  }
  out[0] = s2; out[1] = mx; out[2] = v2; out[3] = o->last_gbar_sq;
}
