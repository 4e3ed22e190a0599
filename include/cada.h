/*
 * cada.h - C ABI of the CADA (Communication-Adaptive Distributed Adam) hot path
 *          for all M simulated workers on one AMD MI355X (gfx950).
 *
 * One call to cada_step() is one iteration k of the paper's Algorithm 1:
 *   - every worker m evaluates its minibatch stochastic gradient at theta^k and at
 *     its reference point on the SAME samples (CADA1: the snapshot theta-tilde,
 *     refreshed when k mod D == 0; CADA2: theta^{k - tau_m^k}, the iterate of its
 *     last upload);
 *   - the squared norm of the rule's left-hand side (Section 2.2, condition
 *     (workerrule1) for CADA1, (workerrule2) for CADA2) is compared with
 *         (c / d_max) * sum_{d=1..d_max} |theta^{k+1-d} - theta^{k-d}|^2 ;
 *     a worker uploads iff the condition is violated or tau_m^k >= D;
 *   - uploading workers refresh their stored gradient (tau_m <- 1), the others
 *     keep the stale one (tau_m <- tau_m + 1);
 *   - the server forms nabla^k = (1/M) sum_m (stored gradient of m) and applies
 *     equations (CADA-1)-(CADA-3) of Section 1.2:
 *         h <- beta1 h + (1-beta1) nabla,  v <- beta2 vhat + (1-beta2) nabla^2,
 *         vhat <- max(v, vhat),  theta <- theta - alpha * h / sqrt(eps + vhat),
 *     and records |theta^{k+1}-theta^k|^2 among the last d_max squared steps.
 *
 * Conventions
 *   - Pointers marked DEVICE are HIP device pointers owned by the caller; HOST
 *     pointers are ordinary host memory and are only read during the call.
 *   - The library never allocates or frees device memory: all state lives in the
 *     caller's workspace (size from cada_workspace_bytes()).
 *   - cada_init / cada_step / cada_run enqueue work on the given stream and never
 *     synchronise the host.  X, y, idx, replay and the workspace must stay valid
 *     until that work has completed.
 *   - Every function returns 0 on success or a negative CADA_E* code; the text of
 *     the last error on the calling thread is available from cada_last_error().
 *     Nothing aborts or throws across this boundary.
 */
#ifndef CADA_H
#define CADA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cada_ctx cada_ctx; /* opaque, host memory owned by the library */

enum {
  CADA_RULE_ALWAYS = 0, /* every worker uploads every iteration: the distributed Adam/AMSGrad baseline (Section 4) */
  CADA_RULE_CADA1 = 1,  /* condition (workerrule1), Section 2.2 */
  CADA_RULE_CADA2 = 2,  /* condition (workerrule2), Section 2.2 */
  CADA_RULE_LAG = 3     /* stochastic LAG, condition (LAGrule), Section 2.1: left-hand side
                           |fresh gradient - stored gradient|^2, one gradient evaluation per iteration */
};
enum {
  CADA_SERVER_AMSGRAD = 0, /* equations (CADA-1)-(CADA-3) */
  CADA_SERVER_SGD = 1      /* theta <- theta - alpha * nabla, the update stochastic LAG follows (Section 2.1);
                              h, v, vhat stay at their initial zeros */
};
enum { CADA_MODEL_LOGREG = 0, CADA_MODEL_MLP = 1 };
enum {
  CADA_PATH_AUTO = 0,        /* single pass where it applies (p >= 8192, a multiple of 4), whole steps for small
                                workloads (at most 64 workers of at most 64 rows whose minibatch and the server's
                                vectors fit one workgroup's LDS), two passes otherwise */
  CADA_PATH_TWO_PASS = 1,    /* two streaming passes over the minibatch rows (any shape) */
  CADA_PATH_SINGLE_PASS = 2, /* one pass: the rows stay in registers/LDS between the two products */
  CADA_PATH_WHOLE_STEPS = 3  /* whole iterations in one launch, one workgroup per worker, whenever the shape allows it,
                                also where separate kernels would be faster for one run: cada_run_replicas needs it */
};
enum {
  CADA_GEMM_FP32 = 0, /* not implemented for the MLP model: cada_workspace_bytes/cada_init refuse it (CADA_EUNSUPPORTED) */
  CADA_GEMM_BF16 = 1  /* bf16 MFMA products of split (hi + lo) operands, float32 accumulation; the MLP model
                         supports at most 32 classes (width of the last layer) */
};

/* How the server keeps the workers' last uploaded (stale) stochastic gradients, the terms that the aggregate of
 * (CADA-1) sums (Section 1.2). */
enum {
  CADA_STORE_F32 = 0, /* float32: the aggregate is the sum of the gradients as computed */
  CADA_STORE_BF16 = 1 /* bf16 (MLP model with the CADA1, CADA2 or always-upload rule): every gradient is rounded to
                         nearest-even when its worker writes it, so each term of the aggregate carries a relative
                         error of at most 2^-9 (the rule's left-hand side is formed before the rounding and does not
                         change); halves the bytes that the weight-gradient kernels write and the server reads.
                         cada_copy_stored_gradients returns the rounded values, cada_set_state rounds what it is given */
};

enum {
  CADA_OK = 0,
  CADA_EINVAL = -1,     /* bad argument (message says which) */
  CADA_EWORKSPACE = -2, /* workspace too small or misaligned */
  CADA_EHIP = -3,       /* a HIP call failed */
  CADA_EUNSUPPORTED = -4
};

#define CADA_REPLAY_FREE 255 /* replay byte that leaves the decision to the rule */
#define CADA_MAX_LAYERS 8
#define CADA_MAX_B 4096      /* minibatch rows per worker */
#define CADA_MAX_DMAX 1024

/* Problem statement of Section 1 (M workers, theta in R^p, local data per worker)
 * plus the inputs of Algorithm 1 (alpha, c, D) and of the rules (d_max). */
typedef struct cada_config {
  int32_t M;                 /* workers */
  int64_t p;                 /* parameters; checked against the model */
  int32_t model;             /* CADA_MODEL_* */
  int32_t n_layers;          /* LOGREG: 1 ; MLP: number of weight layers L */
  const int32_t *layer_dims; /* HOST [n_layers+1]; LOGREG: {p, 1}; MLP: {d0,...,dL} */
  int32_t B;                 /* minibatch rows per worker per step, 1..CADA_MAX_B */
  const int64_t *n_samples;  /* HOST [M]; worker m owns rows [off_m, off_m+N_m) of X,
                                off_m = N_0 + ... + N_{m-1} */
  const float *X;            /* DEVICE, row-major [sum N_m, d0] float32, read-only */
  const void *y;             /* DEVICE [sum N_m]: float32 +1/-1 (LOGREG), int32 class (MLP) */
  double alpha, beta1, beta2, eps; /* (CADA-1)-(CADA-3); constant stepsize.  Doubles so that
                                1-beta1 and 1-beta2 are formed before rounding to float32
                                (1.0f-0.999f is off by 1.3e-5 relative) */
  double lambda_l2;          /* LOGREG: (lambda/2)|theta|^2 is part of the loss */
  double c;                  /* threshold constant of the rules, >= 0 */
  int32_t d_max;             /* squared steps averaged on the right-hand side */
  int32_t D;                 /* max delay (forced upload) and CADA1 snapshot period */
  int32_t rule;              /* CADA_RULE_* */
  int32_t gemm_dtype;        /* MLP contractions: CADA_GEMM_* (LOGREG ignores it) */
  int32_t server;            /* CADA_SERVER_* */
  int64_t alpha_K0;          /* 0: constant stepsize alpha; K0 > 0: alpha_k = alpha K0/(k + K0), the
                                decaying stepsize 2/(mu (k + K0)) of Theorem 2 with alpha = 2/(mu K0) */
  int64_t trace_steps;       /* steps of per-step trace to keep (0 = none) */
  int32_t path;              /* LOGREG: which kernels compute the gradients and the rule's left-hand side, CADA_PATH_*.
                                A request the shape does not allow falls back to the library's own choice;
                                cada_profile_phase_name() tells which kernels a context runs.  MLP ignores it */
  int32_t single_pass_rows;  /* CADA_PATH_SINGLE_PASS tuning: 0 = the library picks (two minibatch rows per iteration
                                when B is even), 1 = one row per iteration */
  int32_t single_pass_clusters; /* 0 = as many workgroup clusters as the device holds; n > 0: at most n (fewer,
                                longer-lived clusters: every cluster then changes worker in mid-stream) */
  int32_t plain_launch;      /* 1 = launch the single-pass and the whole-step kernel as ordinary grids instead of cooperatively (for
                                profilers that cannot trace cooperative dispatches; the device must be otherwise idle;
                                every wait in the kernel is bounded and reports through error_flags bit 1) */
  int32_t two_pass_group;    /* CADA_PATH_TWO_PASS tuning: workers per pair of launches, 0 = all */
  int32_t gradient_store;    /* CADA_STORE_*; anything but CADA_STORE_F32 on a model or rule that does not support it is
                                refused (CADA_EUNSUPPORTED) */
  void *workspace;           /* DEVICE, 256-byte aligned, caller-owned */
  size_t workspace_bytes;
  void *stream;              /* hipStream_t; NULL = the default stream */
} cada_config;

/* Device pointers into the workspace (valid until cada_destroy, contents change
 * with every step) and host-side counters. */
typedef struct cada_state {
  const float *theta, *h, *v, *vhat, *nabla; /* DEVICE [p] */
  const float *theta_lo;                     /* DEVICE [p]: the iterate is theta + theta_lo, a
                                                two-float sum (|theta_lo| <= ulp(theta)/2) */
  const int32_t *tau;                        /* DEVICE [M], tau_m^k for the next step */
  const float *ring;                         /* DEVICE [d_max], slot j mod d_max = |theta^{j+1}-theta^j|^2 */
  const uint8_t *mask;                       /* DEVICE [M], uploads of the last step */
  const float *lhs;                          /* DEVICE [M], rule left-hand sides of the last step */
  const uint64_t *uploads_total;             /* DEVICE [1], sum of all masks so far */
  const uint32_t *error_flags;               /* DEVICE [1]; bit 0: a minibatch index was out of range (clamped);
                                                bit 1: a bounded wait among workgroups gave up (the single-pass and the
                                                whole-iteration logistic kernels; results of that step are invalid);
                                                bit 2: cada_set_state was given a delay outside [1, D] (clamped);
                                                bit 3: a replay mask kept a CADA2 worker silent for more than D
                                                iterations, so its reference point theta^{k - tau_m} was no longer
                                                retained and theta^{k - D} was used instead */
  int64_t k;                                 /* steps enqueued so far */
  int64_t trace_steps;                       /* capacity of the trace */
  const uint8_t *trace_mask;                 /* DEVICE [trace_steps, M] applied masks */
  const uint8_t *trace_own_mask;             /* DEVICE [trace_steps, M] the rule's own decision */
  const float *trace_lhs;                    /* DEVICE [trace_steps, M] */
  const float *trace_rhs;                    /* DEVICE [trace_steps] */
  const int32_t *trace_tau;                  /* DEVICE [trace_steps, M] tau_m^k before the step */
} cada_state;

/* Bytes of device workspace cada_init needs for this configuration (only the
 * shape fields, rule, model, gemm_dtype, gradient_store, D, d_max and trace_steps are read).
 * Returns 0 and sets the error text if the configuration is invalid. */
size_t cada_workspace_bytes(const cada_config *cfg);

/* Validates cfg, lays the state out in cfg->workspace and enqueues its
 * initialisation: theta <- theta0 (DEVICE [p]), h = v = vhat = 0, stored
 * gradients 0, tau_m = D (so every worker uploads at k = 0), all squared steps 0
 * (theta^{-D} = ... = theta^0, supplement "Supporting Lemmas").  *out receives the
 * context.  theta0 may be released once the stream has passed this call. */
int cada_init(const cada_config *cfg, const float *theta0, cada_ctx **out);

/* One iteration of Algorithm 1.  idx: DEVICE int32 [M, B], worker-local row ids
 * in [0, N_m) (duplicates allowed; out-of-range ids are clamped and flagged).
 * replay: DEVICE uint8 [M] or NULL; 0 / 1 force "skip" / "upload" for that
 * worker, CADA_REPLAY_FREE leaves the decision to the rule.  The rule's own
 * decision is always evaluated and traced. */
int cada_step(cada_ctx *ctx, const int32_t *idx, const uint8_t *replay);

/* n_steps iterations back to back: idx_sched DEVICE int32 [n_steps, M, B],
 * replay_sched DEVICE uint8 [n_steps, M] or NULL. */
int cada_run(cada_ctx *ctx, const int32_t *idx_sched, const uint8_t *replay_sched, int64_t n_steps);

/* Independent runs side by side (the simulations of Section 4 average several Monte-Carlo runs):
 * the n_replicas contexts, all with the same M, p, B and rule, initialised with path = CADA_PATH_WHOLE_STEPS on
 * the same stream, advance n_steps iterations each in ONE launch (one workgroup per worker and
 * replica), with their own data, iterates, schedules and decisions.  ctxs, idx_scheds,
 * replay_scheds: HOST arrays of n_replicas entries; idx_scheds[r] DEVICE int32 [n_steps, M, B],
 * replay_scheds NULL or replay_scheds[r] DEVICE uint8 [n_steps, M] or NULL.  At most
 * CADA_MAX_REPLICAS contexts and n_replicas * M workgroups no more than the device's CUs; each
 * context ends exactly where n_steps calls of cada_step would have left it. */
#define CADA_MAX_REPLICAS 16
int cada_run_replicas(cada_ctx *const *ctxs, int32_t n_replicas, const int32_t *const *idx_scheds,
                      const uint8_t *const *replay_scheds, int64_t n_steps);

/* Fills *out with device pointers and host counters.  Enqueues one small kernel on the context's
 * stream (it adds the last step's partial sums of |theta^{k+1} - theta^k|^2 into its ring slot, which
 * the next step would otherwise do) and does not synchronise: read the device memory after
 * synchronising the stream. */
int cada_get_state(cada_ctx *ctx, cada_state *out);

/* Enqueues a copy of the M stored (possibly stale) gradients, one row per
 * worker, into out (DEVICE float32 [M, p]). */
int cada_copy_stored_gradients(cada_ctx *ctx, float *out);

/* The state of Algorithm 1 before iteration k as explicit arrays: the iterate and the moments of
 * equations (CADA-1)-(CADA-3), the stored stale gradients nabla l(theta-hat_m; xi-hat_m) that
 * nabla^k sums (Section 1.2), each worker's reference point (CADA2: theta-hat_m = theta^{k - tau_m},
 * the iterate of its last upload; CADA1: the snapshot theta-tilde and the stored innovations
 * delta-tilde_m^{k - tau_m} of condition (workerrule1)), the delays tau_m^k and the last d_max
 * squared steps of the rules' right-hand side.  Every pointer is DEVICE memory owned by the caller,
 * float32 unless stated, read by kernels that cada_set_state enqueues on the context's stream (no
 * host synchronisation; the arrays may be released once the stream has passed the call). */
typedef struct cada_state_in {
  int64_t k;                       /* the iteration the next cada_step performs, >= 0 */
  const float *theta;              /* [p] */
  const float *theta_lo;           /* [p] or NULL (zeros): the iterate is theta + theta_lo */
  const float *h, *vhat;           /* [p]; v is an output of a step, not state */
  const float *stored_gradients;   /* [M, p] */
  const float *reference;          /* CADA2: [M, p], row m = theta^{k - tau_m}; workers with equal tau_m must
                                      hold equal rows (they uploaded at the same iteration).  CADA1: [p], the
                                      snapshot.  Other rules: ignored, may be NULL */
  const float *reference_lo;       /* same shape, or NULL (zeros): low parts as for theta_lo */
  const float *stored_innovations; /* CADA1: [M, p]; other rules: ignored, may be NULL */
  const int32_t *tau;              /* int32 [M], each in [1, D]; a value outside sets bit 2 of error_flags and is clamped */
  const float *ring;               /* [d_max], slot j mod d_max = |theta^{j+1} - theta^j|^2 for the last d_max j < k */
  uint64_t uploads_total;          /* uploads counted so far */
} cada_state_in;

/* Replaces the context's state by *in and sets its step counter to in->k, so that the following
 * steps continue Algorithm 1 from that state (resume from arrays that another implementation, or
 * cada_get_state / cada_copy_stored_gradients of another context, produced).  The per-step trace
 * keeps what it holds; steps k >= trace_steps are not traced.  Returns CADA_EINVAL (and changes
 * nothing) if a required pointer is NULL or k < 0. */
int cada_set_state(cada_ctx *ctx, const cada_state_in *in);

/* Evaluation on all the data at the current iterate (the y-axes of the figures of Section 4):
 * out[0] = L(theta) = (1/M) sum_m L_m(theta), L_m the mean loss over worker m's N_m samples
 * (problem (1), Section 1; plus (lambda/2)|theta|^2 for the logistic model), out[1] = the
 * fraction of correctly classified samples, averaged over the workers in the same way.
 * out: DEVICE double[2], written by kernels enqueued on the context's stream (no host
 * synchronisation).  Not part of an iteration: the optimiser state is not touched; the MLP
 * variant runs the forward contractions in chunks of B rows per worker and overwrites the
 * activation buffers of the last step. */
int cada_eval(cada_ctx *ctx, double *out);

/* cada_eval for callers that cannot allocate device memory or hand over a workspace sized for it:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same result as cada_eval (bit for bit), but the per-block partial sums and the
 * per-worker means live in a fixed array inside the library (2.1 MB per GPU, held until the
 * process ends) instead of in the context's workspace.  Logistic model only, at most
 * CADA_EVAL_NOALLOC_MAX_M workers: more workers return CADA_EINVAL, the MLP model
 * CADA_EUNSUPPORTED, and nothing is launched.  The call allocates and frees nothing, records no
 * memset, and does not synchronise.  All calls on one GPU share the array: calls that may overlap
 * on that GPU (different streams) race; calls on one stream are safe.  out: DEVICE double[2]. */
#define CADA_EVAL_NOALLOC_MAX_M 256
int cada_eval_noalloc(cada_ctx *ctx, double *out);

/* Checkpoint / resume.  A checkpoint is the whole workspace (iterate, moments, stored
 * gradients, reference points, delays, ring, trace, ...) plus the host-side counters, as one
 * opaque block of cada_checkpoint_bytes(ctx) bytes of DEVICE memory owned by the caller.
 * cada_checkpoint_save enqueues the copy on the context's stream and then waits for it (this
 * call synchronises the stream).  cada_checkpoint_load validates the block against the
 * context (same configuration: shapes, rule, model, workspace size), restores the state and
 * the step counter, and also waits for the stream; on a mismatch it returns CADA_EINVAL and
 * changes nothing.  A block saved by one context can be loaded into another context created
 * with an equal configuration (the data X, y are not part of it). */
size_t cada_checkpoint_bytes(cada_ctx *ctx);
int cada_checkpoint_save(cada_ctx *ctx, void *dst);
int cada_checkpoint_load(cada_ctx *ctx, const void *src);

/* Measurement hooks (not part of the method).  cada_profile_begin creates HIP events
 * for up to max_steps steps; while profiling, every step records an event on the
 * context's stream before and after each of its phases (a phase is one kernel, or one
 * group of kernels, named by cada_profile_phase_name).  cada_profile_end waits for
 * the last recorded event (this one call does synchronise the host), writes the
 * summed duration of each phase in milliseconds into ms_out (HOST, n_out doubles,
 * n_out >= cada_profile_phases(ctx)), the number of profiled steps into *steps_out,
 * and destroys the events. */
int cada_profile_phases(cada_ctx *ctx);
const char *cada_profile_phase_name(cada_ctx *ctx, int phase);
int cada_profile_begin(cada_ctx *ctx, int64_t max_steps);
int cada_profile_end(cada_ctx *ctx, double *ms_out, int n_out, int64_t *steps_out);

/* Frees the host context.  Device memory is the caller's. */
void cada_destroy(cada_ctx *ctx);

/* Text of the last error on this thread ("" if none). */
const char *cada_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CADA_H */
