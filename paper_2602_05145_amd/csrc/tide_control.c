/* Host-only adaptive control: speedup model (Eq. 1-5) and training controller (Algorithm 1, Eq. 6). */
#include "../../include/tide_control.h"

#include <math.h>
#include <string.h>

static int alpha_gamma_ok(double alpha, int gamma) { return alpha >= 0.0 && alpha <= 1.0 && gamma >= 0; }

double tide_expected_accept_length(double alpha, int gamma) {
  if (!alpha_gamma_ok(alpha, gamma)) return NAN;
  /* Horner form of 1 + alpha + ... + alpha^gamma */
  double s = 1.0;
  for (int i = 0; i < gamma; ++i) s = 1.0 + alpha * s;
  return s;
}

double tide_sd_latency(double alpha, int gamma, double d_b, double t_verify) {
  if (!alpha_gamma_ok(alpha, gamma) || !(d_b >= 0.0) || !(t_verify > 0.0)) return NAN;
  return ((double)gamma * d_b + t_verify) / tide_expected_accept_length(alpha, gamma);
}

double tide_theoretical_speedup(double alpha, int gamma, double c) {
  if (!alpha_gamma_ok(alpha, gamma) || !(c >= 0.0)) return NAN;
  return tide_expected_accept_length(alpha, gamma) / (c * (double)gamma + 1.0);
}

double tide_speedup(double alpha, int gamma, double d_b, double t_b, double t_verify) {
  if (!(t_b > 0.0)) return NAN;
  const double sd = tide_sd_latency(alpha, gamma, d_b, t_verify);
  return isnan(sd) ? NAN : t_b / sd;
}

static int profile_ok(const tide_latency_profile *p) {
  if (!p || !p->n || !p->t || p->n_points < 1 || !(p->d0 > 0.0) || p->n[0] < 1) return 0;
  for (int i = 0; i < p->n_points; ++i) {
    if (!(p->t[i] > 0.0)) return 0;
    if (i > 0 && p->n[i] <= p->n[i - 1]) return 0;
  }
  return 1;
}

double tide_profile_latency(const tide_latency_profile *p, double x) {
  if (!profile_ok(p) || isnan(x)) return NAN;
  const int m = p->n_points;
  if (x < (double)p->n[0] || x > (double)p->n[m - 1]) return NAN;
  for (int i = 0; i < m; ++i) {
    if (x == (double)p->n[i]) return p->t[i];
    if (x < (double)p->n[i]) {
      const double x0 = (double)p->n[i - 1], x1 = (double)p->n[i];
      return p->t[i - 1] + (p->t[i] - p->t[i - 1]) * ((x - x0) / (x1 - x0));
    }
  }
  return NAN;
}

/* c(b)*gamma + beta(b): the denominator of Eq. 5 */
static double practical_denominator(const tide_latency_profile *p, int gamma, int32_t batch) {
  if (gamma < 0 || batch < 1) return NAN;
  const double tb = tide_profile_latency(p, (double)batch);
  const double tv = tide_profile_latency(p, (double)batch * (double)(gamma + 1));
  if (isnan(tb) || isnan(tv)) return NAN;
  return (p->d0 / tb) * (double)gamma + tv / tb;
}

double tide_practical_speedup(const tide_latency_profile *p, double alpha, int gamma, int32_t batch) {
  if (!alpha_gamma_ok(alpha, gamma)) return NAN;
  const double den = practical_denominator(p, gamma, batch);
  return isnan(den) ? NAN : tide_expected_accept_length(alpha, gamma) / den;
}

double tide_min_acceptance(const tide_latency_profile *p, int gamma, int32_t batch) {
  const double den = practical_denominator(p, gamma, batch);
  if (isnan(den)) return NAN;
  if (den <= 1.0) return 0.0;                    /* E[l](0) = 1 already breaks even */
  if (den > (double)(gamma + 1)) return 2.0;     /* E[l](1) = gamma + 1 is not enough */
  double lo = 0.0, hi = 1.0;                     /* E[l] is increasing in alpha */
  for (int it = 0; it < 200 && hi - lo > 1e-12; ++it) {
    const double mid = 0.5 * (lo + hi);
    if (tide_expected_accept_length(mid, gamma) < den) lo = mid; else hi = mid;
  }
  return hi;
}

int tide_should_speculate(const tide_latency_profile *p, double alpha, int gamma, int32_t batch, double margin) {
  if (!p) return TIDE_CTRL_ERR_NULL;
  if (!profile_ok(p) || !alpha_gamma_ok(alpha, gamma) || batch < 1 || !(margin > 0.0)) return TIDE_CTRL_ERR_ARG;
  const double s = tide_practical_speedup(p, alpha, gamma, batch);
  return (!isnan(s) && s > margin) ? 1 : 0;
}

int tide_controller_init(tide_controller *c, const tide_controller_params *prm) {
  if (!c || !prm) return TIDE_CTRL_ERR_NULL;
  if (!(prm->lambda_short >= 0.0 && prm->lambda_short < 1.0) || !(prm->lambda_long >= 0.0 && prm->lambda_long < 1.0) ||
      !(prm->lambda_short < prm->lambda_long) || !(prm->epsilon >= 0.0) || prm->n_init < 1 || prm->n_threshold < 2 ||
      !(prm->train_fraction > 0.0 && prm->train_fraction < 1.0))
    return TIDE_CTRL_ERR_ARG;
  memset(c, 0, sizeof(*c));
  c->prm = *prm;
  int32_t nt = (int32_t)floor((double)prm->n_threshold * prm->train_fraction);
  if (nt < 1) nt = 1;
  if (nt > prm->n_threshold - 1) nt = prm->n_threshold - 1;
  c->n_train = nt;
  return TIDE_CTRL_OK;
}

int tide_controller_observe(tide_controller *c, double alpha) {
  if (!c) return TIDE_CTRL_ERR_NULL;
  if (!(alpha >= 0.0 && alpha <= 1.0)) return TIDE_CTRL_ERR_ARG;
  c->n_seen += 1;
  if (c->n_seen <= c->prm.n_init) {
    c->init_sum += alpha;
    if (c->n_seen == c->prm.n_init) c->ema_short = c->ema_long = c->init_sum / (double)c->prm.n_init;
    return 0;
  }
  c->ema_short = c->prm.lambda_short * c->ema_short + (1.0 - c->prm.lambda_short) * alpha;
  c->ema_long = c->prm.lambda_long * c->ema_long + (1.0 - c->prm.lambda_long) * alpha;
  if (c->ema_short < c->ema_long - c->prm.epsilon) c->collection_enabled = 1;
  int flags = 0;
  if (c->collection_enabled && !c->awaiting_result) {
    flags |= TIDE_CTRL_STORE;
    if (c->n_stored < c->n_train) c->train_alpha_sum += alpha;
    c->n_stored += 1;
    if (c->n_stored >= c->prm.n_threshold) {
      flags |= TIDE_CTRL_TRAIN;
      c->awaiting_result = 1;
    }
  }
  return flags;
}

double tide_controller_train_alpha(const tide_controller *c) {
  if (!c || c->n_stored < 1) return NAN;
  const int32_t k = c->n_stored < c->n_train ? c->n_stored : c->n_train;
  return c->train_alpha_sum / (double)k;
}

int tide_controller_report(tide_controller *c, double alpha_eval) {
  if (!c) return TIDE_CTRL_ERR_NULL;
  if (!c->awaiting_result || !(alpha_eval >= 0.0 && alpha_eval <= 1.0)) return TIDE_CTRL_ERR_ARG;
  const double alpha_train = tide_controller_train_alpha(c);
  int decision = TIDE_CTRL_KEEP;
  if (alpha_eval > alpha_train) decision = TIDE_CTRL_DEPLOY;
  else if (alpha_eval < alpha_train) { decision = TIDE_CTRL_STOP_COLLECTING; c->collection_enabled = 0; }
  c->n_stored = 0;
  c->train_alpha_sum = 0.0;
  c->awaiting_result = 0;
  return decision;
}
