/*
 * rudra_ps.h -- C ABI of the MI355X (gfx950) parameter-server update path of Rudra
 * ("Model Accuracy and Runtime Tradeoff in Distributed Deep Learning: A Systematic
 * Study", arXiv 1509.04210).
 *
 * One rudra_ps_t is one parameter server: it holds the fp32 weight vector theta
 * (and the momentum velocity v) in HBM, receives pushGradient messages, and, when
 * the protocol says so, runs sumGradients + applyUpdate as ONE fused HIP kernel
 * that reads each pushed gradient once and touches each weight once.
 *
 * Conventions
 *   - "device pointer": memory of the GPU named in rudra_ps_config_t.device,
 *     accessible to kernels on rudra_ps_config_t.stream.  "host pointer": ordinary
 *     process memory.  Every pointer argument says which it is.
 *   - Every function returns RUDRA_OK (0) or a negative rudra_status code.  Nothing
 *     aborts, throws or exits.  A rejected call leaves the server unchanged.
 *   - Calls on one server are serialised by an internal mutex: the order of
 *     rudra_ps_push_gradient calls IS the arrival order of the gradients, and it
 *     fixes the order of the floating-point additions (Sec. 3.2 "Parameter Server":
 *     the server takes its messages one at a time).
 *   - All device work is enqueued on the caller's stream; push never waits for the GPU and never allocates device
 *     memory (everything is allocated by rudra_ps_create).  One exception, by request: with RUDRA_FLAG_TIME_KERNELS
 *     a push waits for the oldest timed launch once 256 timed launches are outstanding.
 */
#ifndef RUDRA_PS_H
#define RUDRA_PS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rudra_ps rudra_ps_t; /* opaque; created and destroyed by the library */

/* Synchronisation protocol (Sec. 3.1). */
enum rudra_protocol {
  RUDRA_HARDSYNC = 0, /* one gradient from each of the lambda learners per step, Eq. 3; staleness 0 */
  RUDRA_SOFTSYNC = 1  /* n-softsync: update after c = floor(lambda/n) gradients, Eq. 5; n = lambda is Async, Eq. 4 */
};

/* How the learning rate of an update is formed from alpha0 (Sec. 3.2 "Parameter Server", Sec. 5.1 Eq. 6). */
enum rudra_lr_mode {
  RUDRA_LR_CONST = 0,         /* alpha0 * lr_scale (hardsync: lr_scale = sqrt(lambda*mu/B)) */
  RUDRA_LR_STATIC_N = 1,      /* alpha0 * lr_scale / n */
  RUDRA_LR_AVG_STALENESS = 2, /* alpha0 * lr_scale / max(1, <sigma>), <sigma> of this update's vector clock */
  RUDRA_LR_PER_GRADIENT = 3   /* Sec. 5.1 footnote: gradient l is scaled by 1/max(1, sigma_l) before it is
                                 summed; the update uses alpha0 * lr_scale */
};

/* Update rule of applyUpdate. */
enum rudra_optimizer {
  RUDRA_OPT_SGD = 0,    /* Eq. 1c, with momentum and weight penalty as configured (Sec. 4.2) */
  RUDRA_OPT_ADAGRAD = 1 /* the adaptive rule the paper names for its ImageNet 1-softsync runs (Sec. 5.5): h <- h + gbar^2,
                           theta <- theta - alpha * gbar / (sqrt(h) + adagrad_eps); momentum must be 0; h takes the
                           place of the velocity (rudra_ps_pull_velocity returns it) */
};

enum rudra_flags {
  RUDRA_FLAG_STATS_NORMS = 1u,     /* every applyUpdate also reduces ||gbar||^2, ||theta||^2, ||theta||_inf, ||v||^2 */
  RUDRA_FLAG_PUSH_ACCUMULATE = 2u, /* sum each gradient into a server-owned accumulator at push time (the literal
                                      accumulate-on-arrival reading of sumGradients in Sec. 2); the caller's buffer is free again as
                                      soon as work it enqueues later on the stream runs.  Same bits as the default. */
  RUDRA_FLAG_CONTROL_ONLY = 4u,    /* timestamps, staleness, clocks and rates only: no device memory, no kernels;
                                      grad may be NULL; pulling weights is an error.  For host-side tests. */
  RUDRA_FLAG_TIME_KERNELS = 8u,    /* bracket every applyUpdate launch with HIP events; see rudra_ps_stats_t.  A measuring
                                      mode: the events live in a ring of 256, so the push that triggers a launch while 256
                                      earlier ones are still unresolved waits for the oldest of them to finish */
  RUDRA_FLAG_DOUBLE_BUFFER = 16u,  /* keep two weight buffers: update i reads one and writes the other (no extra traffic),
                                      so the weights of timestamp ts stay readable while update ts+1 runs: the
                                      computation-buffer / communication-buffer pair with a pointer swap of Sec. 3.3,
                                      on the server side.  See rudra_ps_weights_view.  Costs 4P bytes of HBM. */
  RUDRA_FLAG_CHECK_POINTERS = 32u  /* ask the HIP runtime about every pushed pointer (device memory of this device, at
                                      least 4P bytes to the end of its allocation) and reject it with EINVAL otherwise,
                                      instead of letting a kernel fault on it; a few microseconds per push */
};

enum rudra_status {
  RUDRA_OK = 0,
  RUDRA_EINVAL = -1,          /* null/unaligned pointer, n outside [1, lambda], P = 0, unknown learner, ... */
  RUDRA_EFUTURE_TS = -2,      /* gradient timestamp newer than the weights' (Sec. 3.1 requires ts_j >= ts_i) */
  RUDRA_EHARDSYNC_STALE = -3, /* hardsync gradient not computed from the current weights (staleness must be 0) */
  RUDRA_EHARDSYNC_DUP = -4,   /* hardsync: this learner already contributed to the current step */
  RUDRA_ENOMEM = -5,          /* host or device allocation failed */
  RUDRA_EHIP = -6,            /* a HIP call failed; rudra_ps_stats_t.last_hip_error has the hipError_t */
  RUDRA_ERANGE = -7,          /* requested update index not (or no longer) in the clock ring / buffer too small */
  RUDRA_ESTATE = -8           /* call not available in this mode (e.g. weights in CONTROL_ONLY mode) */
};

typedef struct {
  uint64_t n_params;     /* P, number of fp32 parameters (> 0) */
  uint32_t n_learners;   /* lambda (> 0) */
  uint32_t n_split;      /* n of n-softsync, 1..lambda; under hardsync only RUDRA_LR_STATIC_N reads it (then >= 1) */
  uint32_t c_override;   /* 0: c = lambda (hardsync) or floor(lambda/n) (softsync); else gradients per update */
  int32_t protocol;      /* enum rudra_protocol */
  int32_t lr_mode;       /* enum rudra_lr_mode */
  float alpha0;          /* base learning rate */
  float lr_scale;        /* caller-known factor, e.g. sqrt(lambda*mu/B); 1 when there is none.  0 is rejected (EINVAL):
                            a zero-initialised config would otherwise freeze the weights without a word */
  float momentum;        /* 0 = plain SGD; else v <- m v - alpha gbar, theta <- theta + v (Sec. 4.2: 0.9) */
  float weight_decay;    /* L2 penalty: gbar <- gbar + wd*theta (Sec. 4.2: 5e-4 on ImageNet) */
  int32_t optimizer;     /* enum rudra_optimizer */
  float adagrad_eps;     /* >= 0; only read when optimizer == RUDRA_OPT_ADAGRAD */
  int32_t device;        /* HIP device ordinal */
  uint32_t flags;        /* OR of enum rudra_flags */
  void* stream;          /* hipStream_t, borrowed from the caller (NULL = the device's null stream) */
  uint32_t clock_ring;   /* closed vector clocks kept for rudra_ps_vector_clock (0 = 1024); c + max_aggregate - 1 may be at
                            most 2^24 and clock_ring times that at most 2^27 timestamps (EINVAL beyond) */
  /* launch shape of the fused kernel; 0 = library default.  Results do not depend on it, except the order in
     which the optional norms are reduced. */
  uint32_t launch_block;  /* threads per workgroup: 64..1024, multiple of 64 */
  uint32_t launch_unroll; /* gradient loads issued together per lane: 1, 2, 4 or 8.  0 = library default: everything at
                             once up to 4 gradients per update, beyond that one at a time, except on short vectors (fewer
                             tiles of 64 float4 than the chip holds resident wavefronts), which take 2, 4 or 8.  Launches
                             fused by rudra_ps_push_batch: 4 or 8 = that many per round, 1 or 2 = one load ahead of the
                             arithmetic (0 = by vector length) */
  uint32_t launch_vec;    /* float4 vectors per lane per tile: 1, 2 or 4 */
  uint32_t launch_grid;   /* upper bound on workgroups (grid-stride beyond it); 0 = one tile per workgroup */
  uint32_t launch_waves_per_cu; /* cap on resident wavefronts per compute unit, 2..32 (enforced by reserving LDS per
                                   workgroup); 0 = library default.  Fewer resident waves keep fewer DRAM pages open
                                   at once; see the kernel header for the measured optimum.  The hardware hands out
                                   LDS in coarse units, so neighbouring values can give the same occupancy (measured:
                                   21..25 behave alike, 26..31 behave alike). */
  uint32_t max_aggregate;    /* largest number of learner gradients one rudra_ps_push_aggregate message may stand for
                                (0 or 1: relayed averages are not used).  An update can then collect up to
                                c + max_aggregate - 1 gradients. */
  uint32_t launch_alternate; /* 1: successive updates walk the vector in opposite directions, so the theta/v lines
                                written last are the first read next (memory-side cache reuse); 2: always forward;
                                0 = library default (alternate) */
  uint32_t launch_state_loads; /* which state vector the update kernel reads with non-temporal loads: 1 neither, 2 the
                                velocity / AdaGrad sums, 3 the weights; 0 = library default (by c and by
                                RUDRA_FLAG_DOUBLE_BUFFER, see the kernel header for the measurements).  Takes effect in the
                                default launch shape (launch_vec 1, launch_unroll 1 or 4). */
  uint32_t launch_phased;      /* 2: run single-update launches through the phase-aligned kernel (few persistent waves keep
                                the running sums of their tiles in registers and the whole chip streams through one gradient
                                at a time; not with RUDRA_FLAG_STATS_NORMS, not for launches fused by rudra_ps_push_batch).
                                Same results to the bit.  0 or 1: off (the default): measured +1 to +6 % for 54-64 gradients
                                per update on vectors of 72M parameters and more, slower everywhere else. */
} rudra_ps_config_t;

typedef struct {
  uint64_t staleness; /* sigma = (weight timestamp at arrival) - ts, Sec. 3.1 */
  uint64_t ts_after;  /* weight timestamp after this message was handled */
  uint32_t pending;   /* gradients now waiting for the next update */
  int32_t applied;    /* 1 if this push completed a set of c gradients and applyUpdate was enqueued */
  float lr_used;      /* learning rate of that update (0 when applied == 0) */
} rudra_push_result_t;

typedef struct {
  uint64_t ts_cur;          /* current weight timestamp = number of updates so far */
  uint64_t n_pushes;        /* accepted gradients */
  uint64_t n_updates;
  uint64_t n_rejected;
  uint64_t sigma_sum;       /* over all accepted gradients */
  uint64_t sigma_max;
  uint64_t hist_len;        /* sigma_max + 1 once a gradient has arrived (see rudra_ps_staleness_hist) */
  uint64_t bytes_absorbed;  /* n_pushes * 4 * P */
  double sigma_mean;        /* sigma_sum / n_pushes */
  double last_avg_staleness; /* <sigma> of the latest update, Sec. 3.1 Eq. 2 */
  double theta_sq, theta_inf, v_sq, gbar_sq; /* state after / averaged gradient of the latest update; only with
                                                RUDRA_FLAG_STATS_NORMS and n_updates > 0 (norms_valid = 1) */
  double kernel_ms;         /* RUDRA_FLAG_TIME_KERNELS: summed device time of the applyUpdate launches ... */
  uint64_t kernel_launches; /* ... and how many launches that covers */
  uint32_t pending;         /* gradients received since the latest update */
  uint32_t c;               /* gradients per update */
  float last_lr;
  int32_t norms_valid;
  int32_t last_hip_error;   /* hipError_t of the latest failed HIP call, 0 if none */
  uint32_t reserved;
  uint64_t n_weight_copies; /* copies of the weights handed out: rudra_ps_pull_weights / _pull_weights_on calls that copied,
                               k per rudra_ps_broadcast_weights ... */
  uint64_t n_ts_inquiries;  /* ... and those that only asked for the timestamp (Sec. 3.2 "Learner": a learner asks first
                               and skips the transfer when nothing changed) */
  uint64_t n_weight_views;  /* rudra_ps_weights_view calls */
  uint64_t n_apply_launches;  /* applyUpdate kernel launches: equals n_updates unless rudra_ps_push_batch fused some */
  uint64_t n_batched_updates; /* updates that shared a launch with at least one other update */
  uint64_t n_weight_acquires; /* rudra_ps_weights_acquire calls */
  uint64_t n_reader_waits;    /* reader events that applyUpdate launches were made to wait for (rudra_ps_weights_release) */
  uint64_t n_phased_launches; /* updates that ran through the phase-aligned kernel (see launch_phased) */
} rudra_ps_stats_t;

/* Create a server.  init_weights: DEVICE pointer to P floats (checked with the HIP runtime), copied (the caller keeps its buffer); in
 * CONTROL_ONLY mode it is ignored and may be NULL.  theta, v and any scratch are allocated with hipMalloc and
 * owned by the library until rudra_ps_destroy.  Timestamp starts at 0 (Sec. 3.1), v at 0.
 * Errors: EINVAL (bad config / null), ENOMEM, EHIP. */
int rudra_ps_create(const rudra_ps_config_t* config, const float* init_weights, rudra_ps_t** out);

/* Wait for the stream, free everything.  NULL is allowed. */
int rudra_ps_destroy(rudra_ps_t* ps);

/* pushGradient as the server receives it (Sec. 2, Sec. 3.2): one gradient of P floats plus the timestamp of the
 * weights it was computed from.  Computes its staleness, appends ts to the open vector clock and, on the c-th
 * gradient, enqueues sumGradients+applyUpdate (Eq. 3 / Eq. 5 with the rate of the configured mode) and advances
 * the weight timestamp by one.
 *   grad     DEVICE pointer, P contiguous floats, 16-byte aligned.  BORROWED: unless PUSH_ACCUMULATE is set the
 *            buffer must stay allocated and unmodified until the update that consumes it has run; work enqueued
 *            on the same stream after the push that returned applied = 1 is safe, as is anything after
 *            rudra_ps_sync.
 *   ts       timestamp the learner obtained from rudra_ps_pull_weights
 *   learner  0..lambda-1, or -1 for anonymous (no duplicate check under hardsync)
 *   out      HOST pointer, may be NULL
 * Errors: EINVAL, EFUTURE_TS, EHARDSYNC_STALE, EHARDSYNC_DUP, EHIP; ENOMEM if the staleness histogram cannot grow to
 * this gradient's staleness (the message is then rejected like any other). */
int rudra_ps_push_gradient(rudra_ps_t* ps, const float* grad, uint64_t ts, int32_t learner, rudra_push_result_t* out);

/* A run of n pushGradient messages handled in one call: the gradients that queued up at the server while it was
 * busy (Sec. 3.2: learners send with blocking calls and the server takes the messages one at a time).  Message i is
 * (grads[i], ts[i], learners[i]); the protocol state (staleness, vector clocks, rates, timestamps, statistics, rejections)
 * is exactly what n calls of rudra_ps_push_gradient in this order would leave, and so are theta and v, bit for bit.
 * What differs is the device work: consecutive updates completed inside the call are applied by ONE launch that
 * keeps theta and v in registers from update to update (up to 64 updates / 64 gradients per launch), so u updates of c
 * gradients move P*(4uc + 16) bytes instead of u*P*(4c + 16).  The weights of the timestamps in between are never
 * stored: nothing can pull them, because no other call on this server runs inside this one.  This is the batching
 * of per-gradient updates that small models and lambda-softsync (c = 1) need, where one launch per update is bound by
 * launch latency or by re-reading theta and v.
 *   grads    HOST array of n DEVICE pointers (each P floats, 16-byte aligned, borrowed as in rudra_ps_push_gradient;
 *            safe to reuse after work enqueued on the stream after this call)
 *   ts       HOST array of n timestamps;  learners: HOST array of n learner ids, or NULL (all anonymous)
 *   out      HOST array of n results, or NULL;  n_handled: HOST pointer, or NULL
 * The first rejected message stops the call: messages before it are handled (and their updates enqueued), it and
 * the rest are not; its status is returned and *n_handled = its index (n when all were handled).
 * With RUDRA_FLAG_PUSH_ACCUMULATE the call is the plain loop (the accumulator cannot be shared between updates). */
int rudra_ps_push_batch(rudra_ps_t* ps, const float* const* grads, const uint64_t* ts, const int32_t* learners, uint32_t n,
                        rudra_push_result_t* out, uint32_t* n_handled);

/* The root of a parameter-server tree (Sec. 3.3) receiving what a node relays: avg = the average of m learner
 * gradients (see rudra_ps_leaf_mean), with the m timestamps of those gradients (HOST pointer ts) so that staleness,
 * vector clock and <sigma> stay exact.  It counts as m gradients: the running sum takes m*avg, applyUpdate fires once
 * c or more gradients are in (Sec. 3.1) and averages over the number collected.  The paper does not
 * say which timestamp a relayed average carries nor when a node relays: this is this library's reading.
 * avg: DEVICE pointer, borrowed like a pushed gradient.  out->staleness = the largest constituent staleness.
 * Under hardsync exactly lambda gradients make a step (Eq. 3): a message that would carry the count past lambda is
 * rejected with EHARDSYNC_DUP (some learner would be counted twice).
 * Errors: EINVAL (m = 0, m > max_aggregate, RUDRA_LR_PER_GRADIENT, bad pointer), EFUTURE_TS, EHARDSYNC_STALE,
 * EHARDSYNC_DUP, EHIP. */
int rudra_ps_push_aggregate(rudra_ps_t* ps, const float* avg, const uint64_t* ts, uint32_t m, rudra_push_result_t* out);

/* The arithmetic of a non-root node of the tree (Sec. 3.3: it averages the gradients sent from its learners and relays
 * the average): out[i] = (g_1[i] + ... + g_k[i]) * (1/k), added in the order given.  grads: HOST array of k DEVICE
 * pointers (P floats each, 16-byte aligned, read once); out: DEVICE pointer to P floats; enqueued on `stream` of
 * `device`.  Stateless: which gradients form a group, and their timestamps, are the caller's (the transport's). */
int rudra_ps_leaf_mean(const float* const* grads, uint32_t k, uint64_t n_params, float* out, int32_t device, void* stream);

/* pullWeights (Sec. 2, Sec. 3.2 "Learner"): the weights and their timestamp.  dst: DEVICE pointer to P floats
 * receiving a copy enqueued on the stream after all updates so far (the library's own copy kernel when dst is 16-byte
 * aligned, else the runtime's device-to-device copy), or NULL for the timestamp inquiry a learner makes first to skip the
 * transfer.  ts_out: HOST pointer, may be NULL. */
int rudra_ps_pull_weights(rudra_ps_t* ps, float* dst, uint64_t* ts_out);

/* Zero-copy pullWeights: a DEVICE pointer to the P weights of the current timestamp (HOST pointers theta_out, ts_out
 * receive it and the timestamp).  The weights are produced by work already enqueued on the server's stream: read them
 * on that stream, or after an event recorded on it.  With RUDRA_FLAG_DOUBLE_BUFFER the contents stay unchanged until the
 * SECOND applyUpdate launch after this call is enqueued (the next launch only reads this buffer; a launch is one
 * update, or the updates rudra_ps_push_batch fused); without it, only until the next update is enqueued.  Read-only
 * for the caller. */
int rudra_ps_weights_view(rudra_ps_t* ps, const float** theta_out, uint64_t* ts_out);

/* The same view for a reader on ANOTHER stream, with the ordering made explicit: the communication-buffer side of the
 * computation/communication buffer pair of Sec. 3.3 (a learner's pull thread copies weights while the computation goes on).
 *   rudra_ps_weights_acquire  makes `reader_stream` (hipStream_t of the same device; may be NULL = null stream) wait
 *       for the work on the server's stream that produces the weights of the current timestamp, and returns their
 *       DEVICE pointer, the timestamp and a ticket.  The caller then enqueues its reads (copies, kernels) on
 *       reader_stream.
 *   rudra_ps_weights_release  announces that all those reads have been enqueued on reader_stream: the applyUpdate
 *       launch that overwrites this buffer is made to wait (on the device; no host call blocks) until they are done.
 * The buffer is overwritten by the FIRST applyUpdate launch enqueued after the acquire, or, with
 * RUDRA_FLAG_DOUBLE_BUFFER, by the SECOND (the first only reads it), so with two buffers the reads overlap the next update
 * instead of delaying it.  Release must come before that launch is enqueued; if it comes too late it returns ESTATE and
 * the reads may have seen a torn buffer (the caller should acquire again).  A ticket that is never released
 * protects nothing.  theta_out, ts_out (may be NULL), ticket_out: HOST pointers.
 * Errors: EINVAL, ESTATE (CONTROL_ONLY; release too late), ENOMEM, EHIP. */
int rudra_ps_weights_acquire(rudra_ps_t* ps, void* reader_stream, const float** theta_out, uint64_t* ts_out, uint64_t* ticket_out);
int rudra_ps_weights_release(rudra_ps_t* ps, uint64_t ticket, void* reader_stream);

/* pullWeights on the READER's stream (Sec. 3.3: the learner's pull thread fetches the weights while the computation goes
 * on): acquire, copy and release in one call.  reader_stream (hipStream_t of the same device, may be NULL = null stream)
 * waits for the work that produces the current weights, the copy into dst (DEVICE pointer, P floats) runs there, and the
 * applyUpdate launch that next writes the buffer the copy reads waits for it on the device: with
 * RUDRA_FLAG_DOUBLE_BUFFER that is the second launch from now, so the copy overlaps the next update; without the flag it
 * is the next launch.  No host call blocks.  Given the server's own stream it is rudra_ps_pull_weights.  Counted in
 * n_weight_copies.  ts_out: HOST pointer, may be NULL.  Errors: EINVAL, ESTATE (CONTROL_ONLY), ENOMEM, EHIP. */
int rudra_ps_pull_weights_on(rudra_ps_t* ps, float* dst, void* reader_stream, uint64_t* ts_out);

/* pullWeights for k learners at once: the broadcast of the new weights that ends a hardsync step (Sec. 3.1: every learner
 * gets the updated weights before the next step) and the weight broadcast of Rudra-adv* (Sec. 3.3).  One launch reads the
 * weights once and writes the k copies, P * (4 + 4k) bytes instead of the P * 8k of k pulls (more than 64 destinations go
 * out as several launches).  dsts: HOST array of k DEVICE pointers (P floats each, 16-byte aligned, distinct, not
 * overlapping).  Stream and ordering exactly as rudra_ps_pull_weights_on (give the server's own stream to queue it
 * between the updates).  Counted as k weight copies.  ts_out: HOST pointer, may be NULL.
 * Errors: EINVAL (null or misaligned destination, k = 0), ESTATE (CONTROL_ONLY), ENOMEM, EHIP. */
int rudra_ps_broadcast_weights(rudra_ps_t* ps, float* const* dsts, uint32_t k, void* reader_stream, uint64_t* ts_out);

/* The launch shape the next single-update launch (batched = 0) or batched launch (batched != 0) would use: workgroups,
 * threads per workgroup, tiles of the vector (more than the workgroups when the grid is capped: grid-stride), LDS
 * bytes reserved per workgroup as the occupancy cap.  Pure host arithmetic (works in CONTROL_ONLY mode): grid * block
 * always stays below 2^32, the most one HIP launch takes.  HOST pointers, each may be NULL. */
int rudra_ps_launch_shape(rudra_ps_t* ps, int32_t batched, uint32_t* grid_out, uint32_t* block_out, uint64_t* ntiles_out,
                          uint32_t* lds_bytes_out);

/* Copy of the second state vector (the momentum velocity v, or AdaGrad's h) to dst (DEVICE pointer to P floats),
 * enqueued on the stream.  ESTATE when the update rule keeps none (plain SGD, momentum = 0). */
int rudra_ps_pull_velocity(rudra_ps_t* ps, float* dst);

/* Counters and staleness statistics the server records (Sec. 3.2: it records the vector clock of each update to
 * track the average staleness).  out: HOST pointer.  Waits for the stream only if norms or kernel times are on. */
int rudra_ps_stats(rudra_ps_t* ps, rudra_ps_stats_t* out);

/* Staleness histogram (the distribution shown with the lambda-softsync measurement, Sec. 5.1): out[s] = number of
 * accepted gradients with staleness s.  out: HOST pointer to cap entries; n_out: entries that exist. Copies
 * min(cap, n) entries; ERANGE if cap < n (n_out is still set). */
int rudra_ps_staleness_hist(rudra_ps_t* ps, uint64_t* out, uint64_t cap, uint64_t* n_out);

/* Vector clock of update `update_idx` (0-based: the update advancing timestamp update_idx -> update_idx+1): the c
 * gradient timestamps in arrival order (n_out of them: c, or up to c + max_aggregate - 1), its <sigma> (Eq. 2) and its learning rate.  HOST pointers; avg_sigma_out and
 * lr_out may be NULL.  ERANGE if the update has not happened, has left the ring, or cap < n_out. */
int rudra_ps_vector_clock(rudra_ps_t* ps, uint64_t update_idx, uint64_t* ts_out, uint32_t cap, uint32_t* n_out,
                          double* avg_sigma_out, float* lr_out);

/* FOR CALLERS THAT CANNOT ALLOCATE (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): one sumGradients + applyUpdate with the fused norms, the update that the c-th rudra_ps_push_gradient
 * triggers on a server with RUDRA_FLAG_STATS_NORMS, as a stateless call on the caller's own vectors.  It calls no
 * hipMalloc / hipFree and no allocating routine: the per-workgroup norm slots that the server path keeps in
 * hipMalloc'ed memory live in a fixed array in the library's device image (4 MiB per GPU, held until the process
 * ends), and the slots are combined by a small second launch instead of on the host.
 *   grads      HOST array of c DEVICE pointers (P floats each, 16-byte aligned, read once), summed in the order given
 *   theta      DEVICE pointer, P floats, 16-byte aligned: weights, updated in place
 *   state      DEVICE pointer, P floats, 16-byte aligned: velocity (momentum != 0) or AdaGrad's h, updated in place;
 *              may be NULL for plain SGD
 *   lr         the rate of this update (the caller's: this call keeps no timestamps and computes no staleness)
 *   optimizer  enum rudra_optimizer; momentum, weight_decay, adagrad_eps as in rudra_ps_config_t
 *   norms_out  DEVICE pointer to 4 doubles, 8-byte aligned: sum gbar^2, sum theta^2, sum state^2, max |theta| after
 *              the update, valid once the work enqueued on `stream` has run
 * Arithmetic and bits of theta and state are those of the server path.  Limits: c <= 64 and P <= 134 217 728
 * (one norm slot per 1024-parameter tile); beyond either the call returns ERANGE and does nothing.
 * The first call on a device looks up that device's copy of the array (one hipGetSymbolAddress, no allocation): a caller
 * that records a HIP graph makes one call outside the capture first.
 * All calls on one GPU share that GPU's slot array: calls whose device work can overlap (different streams without
 * ordering between them) race on it and must be serialised by the caller; nothing in it needs clearing between calls.
 * Errors: EINVAL (null / misaligned pointer, c = 0, P = 0, bad optimizer or device), ERANGE, EHIP. */
int rudra_ps_apply_update_noalloc(const float* const* grads, uint32_t c, uint64_t n_params, float* theta, float* state,
                                  float lr, float momentum, float weight_decay, int32_t optimizer, float adagrad_eps,
                                  double* norms_out, int32_t device, void* stream);

/* Learning-rate schedule hook (Sec. 4.2: alpha0 is divided by 10 after given epochs; epochs are the caller's). */
int rudra_ps_set_lr(rudra_ps_t* ps, float alpha0);

/* Wait until everything enqueued so far has run. */
int rudra_ps_sync(rudra_ps_t* ps);

/* Static description of a status code. */
const char* rudra_ps_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* RUDRA_PS_H */
