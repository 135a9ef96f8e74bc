/* Adaptive control of speculative decoding and of draft training (host-only C library, no GPU calls).
 *
 * Two independent parts, both from the paper's Section 4:
 *   1. the batch-size-aware speedup model (Eq. 1-5 with the profiled latencies of Appendix Table 5):
 *      decides whether speculation pays at the current batch size and acceptance rate;
 *   2. the training controller (Algorithm 1, Eq. 6): two exponential moving averages of the acceptance
 *      rate detect a distribution shift, switch signal collection on, ask for a training round when
 *      enough samples are stored, and gate the deployment of the retrained draft.
 * All pointers are HOST pointers.  Nothing here allocates; the caller owns every struct and array.
 * Functions returning double return NaN on invalid arguments; functions returning int return a
 * TIDE_CTRL_* code (< 0) on invalid arguments.  Thread-safety: none needed for the pure functions; a
 * controller struct must not be used from two threads at once. */
#ifndef TIDE_CONTROL_H_
#define TIDE_CONTROL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIDE_CTRL_OK 0
#define TIDE_CTRL_ERR_NULL (-1)
#define TIDE_CTRL_ERR_ARG (-2)

/* ---- speedup model ------------------------------------------------------------------------------ */

/* Eq. 2: expected number of tokens produced per speculation step, (1 - alpha^(gamma+1)) / (1 - alpha),
 * evaluated as the geometric sum 1 + alpha + ... + alpha^gamma (exact also at alpha = 1).
 * alpha in [0,1], gamma >= 0; otherwise NaN. */
double tide_expected_accept_length(double alpha, int gamma);

/* Eq. 3: per-token latency with speculation, (gamma * D_b + T_verify) / E[l]; D_b = draft latency for the
 * batch, T_verify = target latency for b*(gamma+1) tokens.  Same unit as the inputs. */
double tide_sd_latency(double alpha, int gamma, double d_b, double t_verify);

/* Eq. 1: theoretical speedup E[l] / (c*gamma + 1), c = draft/target latency ratio. */
double tide_theoretical_speedup(double alpha, int gamma, double c);

/* Eq. 4: speedup T(b) / SD(b) from the three measured latencies. */
double tide_speedup(double alpha, int gamma, double d_b, double t_b, double t_verify);

/* Profiled latencies (Appendix Table 5): T(n) at n_points increasing token counts n[i], and the
 * batch-independent draft latency D_0.  Arrays are caller-owned and only read. */
typedef struct {
  int32_t n_points;       /* >= 1 */
  const int32_t *n;       /* strictly increasing, n[0] >= 1 */
  const double *t;        /* T(n[i]) > 0, same unit as d0 */
  double d0;              /* D_0 > 0 */
} tide_latency_profile;

/* T(n): the profiled value at a profiled n, linear interpolation in n between neighbouring profiled
 * points (the paper profiles a grid of batch sizes and does not say how it reads between them), NaN
 * outside [n[0], n[n_points-1]] or for an invalid profile. */
double tide_profile_latency(const tide_latency_profile *p, double n_tokens);

/* Eq. 5: practical speedup E[l] / (c(b)*gamma + beta(b)) with c(b) = D_0 / T(b) and
 * beta(b) = T(b*(gamma+1)) / T(b).  NaN when b or b*(gamma+1) is outside the profiled range. */
double tide_practical_speedup(const tide_latency_profile *p, double alpha, int gamma, int32_t batch);

/* Smallest acceptance rate at which Eq. 5 reaches 1 (speculation breaks even) for this batch size:
 * the root of E[l](alpha) = c(b)*gamma + beta(b), found by bisection to 1e-12.  Returns a value > 1
 * (exactly 2.0) when even alpha = 1 does not break even, NaN outside the profiled range. */
double tide_min_acceptance(const tide_latency_profile *p, int gamma, int32_t batch);

/* 1 when Eq. 5 predicts a speedup above `margin` (use 1.0 for break-even), else 0 (also outside the
 * profiled range: without a latency estimate speculation stays off); < 0 on invalid arguments. */
int tide_should_speculate(const tide_latency_profile *p, double alpha, int gamma, int32_t batch,
                          double margin);

/* ---- training controller (Algorithm 1) ------------------------------------------------------------ */

typedef struct {
  double lambda_short, lambda_long;   /* EMA decay rates of Eq. 6, both in [0,1), lambda_short < lambda_long */
  double epsilon;                     /* shift threshold: collect when short < long - epsilon; >= 0 */
  int32_t n_init;                     /* requests averaged to initialise both EMAs; >= 1 */
  int32_t n_threshold;                /* stored samples that trigger a training round; >= 2 */
  double train_fraction;              /* share of the stored samples (the oldest) used as D_train; in (0,1) */
} tide_controller_params;

typedef struct {
  tide_controller_params prm;
  int64_t n_seen;                     /* acceptance rates observed so far */
  double init_sum;                    /* running sum during the first n_init observations */
  double ema_short, ema_long;         /* valid once n_seen >= n_init */
  int32_t collection_enabled;
  int32_t n_stored;                   /* samples stored since the last training round */
  int32_t n_train;                    /* floor(n_threshold * train_fraction), at least 1, at most n_threshold-1 */
  double train_alpha_sum;             /* sum of alpha over the first n_train stored samples */
  int32_t awaiting_result;            /* a training round was requested and its result not yet reported */
} tide_controller;

/* bits of the value returned by tide_controller_observe */
#define TIDE_CTRL_STORE 1             /* store this request's (hidden states, alpha) as a training signal */
#define TIDE_CTRL_TRAIN 2             /* n_threshold samples are stored: split, train, evaluate, then report */

/* what tide_controller_report returns */
#define TIDE_CTRL_DEPLOY 1            /* alpha_eval > alpha_train: the new draft replaces the old one */
#define TIDE_CTRL_STOP_COLLECTING 2   /* alpha_eval < alpha_train: keep the old draft, collection off */
#define TIDE_CTRL_KEEP 3              /* equal: nothing changes */

int tide_controller_init(tide_controller *c, const tide_controller_params *prm);

/* One served request with measured acceptance rate alpha in [0,1].  The first n_init calls only
 * accumulate the initial average (they are not stored and do not move the EMAs); from then on each call
 * updates both EMAs, may switch collection on, and returns the TIDE_CTRL_STORE / TIDE_CTRL_TRAIN bits.
 * While a training round is outstanding (TIDE_CTRL_TRAIN returned, tide_controller_report not yet
 * called) the EMAs keep moving but nothing is stored. */
int tide_controller_observe(tide_controller *c, double alpha);

/* Mean alpha over D_train (the first n_train stored samples); NaN when none is stored. */
double tide_controller_train_alpha(const tide_controller *c);

/* Result of the training round: alpha_eval = acceptance (top-1 agreement) of the retrained draft on
 * D_eval.  Applies the deploy gate, clears the stored-sample counters, and returns one of
 * TIDE_CTRL_DEPLOY / TIDE_CTRL_STOP_COLLECTING / TIDE_CTRL_KEEP (< 0 when no round is outstanding). */
int tide_controller_report(tide_controller *c, double alpha_eval);

#ifdef __cplusplus
}
#endif
#endif  /* TIDE_CONTROL_H_ */
