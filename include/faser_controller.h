/*
 * faser_controller -- the host-side controller of FASER (arXiv 2604.20503) that feeds the
 * verification kernels: per-request speculative lengths (Sec. 3.1: cost objective, Eqs. 1-2, and
 * the GP-LCB search, Eqs. 3-4), the pruning trigger of token-wise early exit (Sec. 3.2, Eqs. 5-10),
 * the frontier chunk-size rule (Sec. 3.3) and the latency models of offline profiling with their
 * least-squares fit (Sec. 3.4, Eqs. 11-14).
 *
 * Everything here is scalar host arithmetic in double precision: EVERY pointer is HOST memory, no
 * call touches the GPU or a stream.  Functions return FSR_OK or a negative FSR_E* code of
 * faser_verify.h; fsr_last_error() describes the last failure.  A controller object is not
 * thread-safe; different objects are independent.
 *
 * What the paper leaves open is fixed here (and can be changed through the configuration): the
 * candidate set S, epsilon, beta_n, the Gaussian-process kernel and the window length.
 */
#ifndef FASER_CONTROLLER_H
#define FASER_CONTROLLER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FSR_CTL_MAX_LENGTHS 16

typedef struct fsr_ctl fsr_ctl; /* opaque controller state */

typedef struct fsr_ctl_config {
    int32_t n_lengths;                    /* |S|, 1 .. FSR_CTL_MAX_LENGTHS */
    int32_t lengths[FSR_CTL_MAX_LENGTHS]; /* the candidate speculative lengths S, strictly increasing, >= 1 */
    int32_t window;                       /* observations kept per (context, request): the sliding window (>= 1) */
    int32_t reserved;                     /* 0 */
    double eps;                           /* epsilon of Eqs. 1 and 4 (> 0) */
    double beta;                          /* > 0: constant beta_n of Eq. 3; <= 0: beta_n = 2 ln(|S| n^2 pi^2 / (6 delta)),
                                             n = observations in the window + 1 */
    double delta;                         /* in (0, 1); used only when beta <= 0 */
    double length_scale;                  /* squared-exponential kernel on s: k(s, s') = signal_var exp(-(s-s')^2 / (2 l^2)) */
    double signal_var;                    /* in units of the window's variance of the observed costs (they are standardised) */
    double noise_var;                     /* observation noise variance, same units (> 0) */
} fsr_ctl_config;

/* Fills cfg with the defaults: S = {2, 4, 6, 8, 10}, window 32, eps 1e-6, beta 2, delta 0.1,
 * length scale 2, signal variance 1, noise variance 0.1. */
int fsr_ctl_default_config(fsr_ctl_config* cfg);
int fsr_ctl_create(const fsr_ctl_config* cfg, fsr_ctl** out);
void fsr_ctl_destroy(fsr_ctl* ctl);

/* Sec. 3.1: one request's outcome in one verification step run under serving context `context` (the
 * caller's bucket of batch size b and compute share r): it drafted s tokens (s in S), n_accepted of
 * them were accepted (0 .. s), and the step took `latency` (any unit, > 0; batch-level, the same value
 * for every request of the step).  Enters a_obs = n_accepted / s, the latency and the realised cost of
 * Eq. 4, latency / (s a_obs + eps), into the window of (context, request), dropping its oldest entry
 * when the window is full. */
int fsr_ctl_observe(fsr_ctl* ctl, int32_t context, int64_t request, int32_t s, int32_t n_accepted, double latency);
/* Drops every window of `request` (it left the batch). */
int fsr_ctl_forget(fsr_ctl* ctl, int64_t request);

/* Eq. 1 for every candidate s (arrays of n_lengths doubles, any may be NULL): a_hat = mean accepted
 * fraction of this request's window entries with that s, T_hat = mean latency of the context's
 * entries (all requests) with that s, J = T_hat / (s a_hat + eps).  Candidates without an observation
 * give NaN. */
int fsr_ctl_estimates(fsr_ctl* ctl, int32_t context, int64_t request, double* a_hat, double* T_hat, double* J);
/* Eq. 2: the observed candidate with the smallest J (the smaller s on ties); FSR_ESHAPE if none is observed. */
int fsr_ctl_best_length(fsr_ctl* ctl, int32_t context, int64_t request, int32_t* s_out);

/* Eqs. 3-4: Gaussian-process posterior of the cost over S from the realised costs in the window of
 * (context, request), standardised by the window's mean and standard deviation (constant prior mean =
 * window mean); mu and sigma (n_lengths doubles each, either may be NULL) come back in the cost's own
 * unit.  With an empty window mu = 0 and sigma = sqrt(signal_var). */
int fsr_ctl_posterior(fsr_ctl* ctl, int32_t context, int64_t request, double* mu, double* sigma);
/* Eq. 3: argmin over S of mu - sqrt(beta_n) sigma (the smaller s on ties). */
int fsr_ctl_choose(fsr_ctl* ctl, int32_t context, int64_t request, int32_t* s_out);

/* ---- Sec. 3.2, Eqs. 5-10: should the estimator's mask be applied after layer `layer`? ---- */
/* Eqs. 5-6: expected number of drafted tokens in rejected suffixes, sum_i s_i (1 - a_hat_i). */
int fsr_expected_rejected(int32_t n, const int32_t* s, const double* a_hat, double* k_rej);
/* Eqs. 7-10 with the three times already evaluated at (b, r, k_rej): the estimator's latency eats
 * dL = L T_ee / T_t layers, L_r' = max(L - layer - dL, 0), T_save = L_r' / L * T_t; *prune = 1 iff
 * T_save > T_pr.  T_save_out may be NULL. */
int fsr_prune_trigger(int32_t L, int32_t layer, double T_t, double T_ee, double T_pr, double* T_save_out, int32_t* prune);

/* ---- Sec. 3.4, Eqs. 11-14: latency models ---- */
enum {
    FSR_LAT_DRAFT = 0,  /* Eq. 11: x = r,     base = alpha b + beta s + c */
    FSR_LAT_TARGET = 1, /* Eq. 12: x = 1 - r, base = (alpha b + beta) s + c   (beta is the paper's lambda_p) */
    FSR_LAT_EXIT = 2,   /* Eq. 13: x = 1 - r, base = alpha b s + beta */
    FSR_LAT_PRUNE = 3,  /* Eq. 14: x = r,     base = alpha b s + beta */
    FSR_LAT_KV = 4      /* not in the paper: x = 1 - r, base = alpha b s + beta b + c.  Eq. 12's base has no term in b
                           alone, which the target's GEMMs do not need but its attention does: reading the
                           cached K/V costs time proportional to b whatever s is */
};
/* T = (a1 - g1 x) base for x <= knee, (a2 - g2 x) base for x > knee, x the share of the compute
 * units the model's side owns (r is the drafter's share). */
typedef struct fsr_latency_model {
    int32_t form;
    int32_t reserved;
    double a1, g1, a2, g2, knee;
    double alpha, beta, c; /* c unused by FSR_LAT_EXIT / FSR_LAT_PRUNE */
} fsr_latency_model;
int fsr_latency_eval(const fsr_latency_model* m, double b, double s, double r, double* T);
/* Least-squares fit to n profiled points (b[j], s[j], r[j]) -> T[j]: for every candidate knee (between
 * consecutive distinct shares, or none) the two linear factors are fitted in turn (each a linear
 * least-squares problem given the other) until the residual stops falling; the best knee wins.  The
 * product leaves one scale free: it is fixed by a1 = 1.  rms_out (nullable) = root mean square residual. */
int fsr_latency_fit(int32_t form, int32_t n, const double* b, const double* s, const double* r, const double* T,
                    fsr_latency_model* out, double* rms_out);

/* ---- Sec. 3.3: frontier chunk size ---- */
/* Among the candidate chunk sizes (n_candidates values, each 1 .. s) picks the one that minimises
 * T_q(s_c; b, r) + ceil(s / s_c) T_p(s_c; b, r) and returns it if that time is below T_hat (the
 * observed latency of unchunked verification of s tokens); otherwise *s_c = 0: overlap is not worth it.
 * draft and target are Eq. 11 / Eq. 12 models (the target's share is 1 - r inside Eq. 12). */
int fsr_chunk_size(const fsr_latency_model* draft, const fsr_latency_model* target, double b, double r, int32_t s,
                   double T_hat, int32_t n_candidates, const int32_t* candidates, int32_t* s_c, double* T_chunked);

#ifdef __cplusplus
}
#endif
#endif
