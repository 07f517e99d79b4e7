// Host-side controller (no device code): per-request speculative lengths (Sec. 3.1, Eqs. 1-4), the
// pruning trigger (Sec. 3.2, Eqs. 5-10), the frontier chunk-size rule (Sec. 3.3) and the latency
// models with their fit (Sec. 3.4, Eqs. 11-14).  Plain double-precision arithmetic on small data.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <deque>
#include <limits>
#include <map>
#include <new>
#include <vector>

#include "../../include/faser_controller.h"
#include "common.hpp"

namespace {

struct Obs {
    int s;
    double a;  // accepted fraction
    double T;  // step latency
    double J;  // realised cost, Eq. 4
};
using Window = std::deque<Obs>;

}  // namespace

struct fsr_ctl {
    fsr_ctl_config cfg;
    std::map<int32_t, std::map<int64_t, Window>> contexts;

    int index_of(int s) const {
        for (int k = 0; k < cfg.n_lengths; ++k)
            if (cfg.lengths[k] == s) return k;
        return -1;
    }
    const Window* find(int32_t context, int64_t request) const {
        auto c = contexts.find(context);
        if (c == contexts.end()) return nullptr;
        auto w = c->second.find(request);
        return w == c->second.end() ? nullptr : &w->second;
    }
};

namespace {

using fsr::fail;
constexpr double kNaN = std::numeric_limits<double>::quiet_NaN();

// Solves the symmetric positive definite system A x = y in place (A is n x n row-major, destroyed).
// Cholesky; returns false if a pivot is not positive.
bool solve_spd(std::vector<double>& A, std::vector<double>& y, int n) {
    for (int j = 0; j < n; ++j) {
        double d = A[j * n + j];
        for (int k = 0; k < j; ++k) d -= A[j * n + k] * A[j * n + k];
        if (!(d > 0.0)) return false;
        d = std::sqrt(d);
        A[j * n + j] = d;
        for (int i = j + 1; i < n; ++i) {
            double v = A[i * n + j];
            for (int k = 0; k < j; ++k) v -= A[i * n + k] * A[j * n + k];
            A[i * n + j] = v / d;
        }
    }
    for (int i = 0; i < n; ++i) {  // L z = y
        double v = y[i];
        for (int k = 0; k < i; ++k) v -= A[i * n + k] * y[k];
        y[i] = v / A[i * n + i];
    }
    for (int i = n - 1; i >= 0; --i) {  // L^T x = z
        double v = y[i];
        for (int k = i + 1; k < n; ++k) v -= A[k * n + i] * y[k];
        y[i] = v / A[i * n + i];
    }
    return true;
}

// Linear least squares min |F theta - t|^2 by the normal equations (p <= 4 columns, well scaled by the
// caller); a tiny ridge keeps a rank-deficient design (one share only, say) solvable.
bool least_squares(const std::vector<double>& F, const std::vector<double>& t, int n, int p, double* theta) {
    std::vector<double> A(p * p, 0.0), y(p, 0.0);
    for (int j = 0; j < n; ++j)
        for (int u = 0; u < p; ++u) {
            y[u] += F[j * p + u] * t[j];
            for (int v = 0; v < p; ++v) A[u * p + v] += F[j * p + u] * F[j * p + v];
        }
    double tr = 0.0;
    for (int u = 0; u < p; ++u) tr += A[u * p + u];
    for (int u = 0; u < p; ++u) A[u * p + u] += 1e-12 * (tr > 0.0 ? tr / p : 1.0);
    if (!solve_spd(A, y, p)) return false;
    for (int u = 0; u < p; ++u) theta[u] = y[u];
    return true;
}

int base_terms(int form) { return form == FSR_LAT_EXIT || form == FSR_LAT_PRUNE ? 2 : 3; }
void base_features(int form, double b, double s, double* phi) {
    switch (form) {
        case FSR_LAT_DRAFT: phi[0] = b; phi[1] = s; phi[2] = 1.0; break;
        case FSR_LAT_TARGET: phi[0] = b * s; phi[1] = s; phi[2] = 1.0; break;
        case FSR_LAT_KV: phi[0] = b * s; phi[1] = b; phi[2] = 1.0; break;
        default: phi[0] = b * s; phi[1] = 1.0; break;
    }
}
double share_of(int form, double r) { return form == FSR_LAT_DRAFT || form == FSR_LAT_PRUNE ? r : 1.0 - r; }
bool form_ok(int form) { return form >= FSR_LAT_DRAFT && form <= FSR_LAT_KV; }

double eval_model(const fsr_latency_model& m, double b, double s, double r) {
    double phi[3];
    base_features(m.form, b, s, phi);
    const double base = base_terms(m.form) == 3 ? m.alpha * phi[0] + m.beta * phi[1] + m.c * phi[2] : m.alpha * phi[0] + m.beta * phi[1];
    const double x = share_of(m.form, r);
    return (x <= m.knee ? m.a1 - m.g1 * x : m.a2 - m.g2 * x) * base;
}

// Window statistics of the realised costs.
void cost_scale(const Window& w, double& mean, double& scale) {
    mean = 0.0;
    for (const Obs& o : w) mean += o.J;
    mean /= (double)w.size();
    double var = 0.0;
    for (const Obs& o : w) var += (o.J - mean) * (o.J - mean);
    var /= (double)w.size();
    scale = var > 0.0 ? std::sqrt(var) : (std::fabs(mean) > 0.0 ? std::fabs(mean) : 1.0);
}

// Gaussian-process posterior over the candidate set (Eq. 3's mu and sigma) in the cost's unit.
int posterior(const fsr_ctl* ctl, const Window* w, double* mu, double* sigma) {
    const fsr_ctl_config& c = ctl->cfg;
    const int m = c.n_lengths;
    auto kern = [&](double s0, double s1) {
        const double d = s0 - s1;
        return c.signal_var * std::exp(-d * d / (2.0 * c.length_scale * c.length_scale));
    };
    if (!w || w->empty()) {
        for (int k = 0; k < m; ++k) {
            if (mu) mu[k] = 0.0;
            if (sigma) sigma[k] = std::sqrt(c.signal_var);
        }
        return FSR_OK;
    }
    const int n = (int)w->size();
    double mean, scale;
    cost_scale(*w, mean, scale);
    std::vector<double> K(n * n), y(n);
    for (int i = 0; i < n; ++i) {
        y[i] = ((*w)[i].J - mean) / scale;
        for (int j = 0; j < n; ++j) K[i * n + j] = kern((*w)[i].s, (*w)[j].s) + (i == j ? c.noise_var : 0.0);
    }
    // alpha = (K + noise I)^-1 y; the variance needs (K + noise I)^-1 k_* for every candidate
    std::vector<double> Kc = K, alpha = y;
    if (!solve_spd(Kc, alpha, n)) return fail(FSR_EINVAL, "fsr_ctl_posterior: kernel matrix not positive definite");
    for (int k = 0; k < m; ++k) {
        std::vector<double> ks(n), v;
        for (int i = 0; i < n; ++i) ks[i] = kern(c.lengths[k], (*w)[i].s);
        double mk = 0.0;
        for (int i = 0; i < n; ++i) mk += ks[i] * alpha[i];
        Kc = K;
        v = ks;
        if (!solve_spd(Kc, v, n)) return fail(FSR_EINVAL, "fsr_ctl_posterior: kernel matrix not positive definite");
        double var = kern(c.lengths[k], c.lengths[k]);
        for (int i = 0; i < n; ++i) var -= ks[i] * v[i];
        if (mu) mu[k] = mean + scale * mk;
        if (sigma) sigma[k] = scale * std::sqrt(std::max(var, 0.0));
    }
    return FSR_OK;
}

bool config_ok(const fsr_ctl_config& c) {
    if (c.n_lengths < 1 || c.n_lengths > FSR_CTL_MAX_LENGTHS || c.window < 1 || c.reserved != 0) return false;
    for (int k = 0; k < c.n_lengths; ++k)
        if (c.lengths[k] < 1 || (k > 0 && c.lengths[k] <= c.lengths[k - 1])) return false;
    if (!(c.eps > 0.0) || !(c.length_scale > 0.0) || !(c.signal_var > 0.0) || !(c.noise_var > 0.0)) return false;
    if (!(c.beta > 0.0) && !(c.delta > 0.0 && c.delta < 1.0)) return false;
    return true;
}

}  // namespace

extern "C" int fsr_ctl_default_config(fsr_ctl_config* cfg) {
    if (!cfg) return fail(FSR_EINVAL, "fsr_ctl_default_config: cfg is null");
    *cfg = fsr_ctl_config{};
    cfg->n_lengths = 5;
    for (int k = 0; k < 5; ++k) cfg->lengths[k] = 2 * (k + 1);
    cfg->window = 32;
    cfg->eps = 1e-6;
    cfg->beta = 2.0;
    cfg->delta = 0.1;
    cfg->length_scale = 2.0;
    cfg->signal_var = 1.0;
    cfg->noise_var = 0.1;
    return FSR_OK;
}

extern "C" int fsr_ctl_create(const fsr_ctl_config* cfg, fsr_ctl** out) {
    if (!cfg || !out) return fail(FSR_EINVAL, "fsr_ctl_create: null argument");
    if (!config_ok(*cfg)) return fail(FSR_EINVAL, "fsr_ctl_create: invalid configuration");
    fsr_ctl* ctl = new (std::nothrow) fsr_ctl();
    if (!ctl) return fail(FSR_EINVAL, "fsr_ctl_create: out of memory");
    ctl->cfg = *cfg;
    *out = ctl;
    return FSR_OK;
}

extern "C" void fsr_ctl_destroy(fsr_ctl* ctl) { delete ctl; }

extern "C" int fsr_ctl_observe(fsr_ctl* ctl, int32_t context, int64_t request, int32_t s, int32_t n_accepted, double latency) {
    if (!ctl) return fail(FSR_EINVAL, "fsr_ctl_observe: ctl is null");
    if (ctl->index_of(s) < 0) return fail(FSR_EINVAL, "fsr_ctl_observe: s=%d is not a candidate length", s);
    if (n_accepted < 0 || n_accepted > s || !(latency > 0.0) || !std::isfinite(latency))
        return fail(FSR_EINVAL, "fsr_ctl_observe: n_accepted=%d of s=%d, latency=%g", n_accepted, s, latency);
    Window& w = ctl->contexts[context][request];
    Obs o;
    o.s = s;
    o.a = (double)n_accepted / (double)s;
    o.T = latency;
    o.J = latency / ((double)s * o.a + ctl->cfg.eps);
    w.push_back(o);
    while ((int)w.size() > ctl->cfg.window) w.pop_front();
    return FSR_OK;
}

extern "C" int fsr_ctl_forget(fsr_ctl* ctl, int64_t request) {
    if (!ctl) return fail(FSR_EINVAL, "fsr_ctl_forget: ctl is null");
    for (auto& c : ctl->contexts) c.second.erase(request);
    return FSR_OK;
}

extern "C" int fsr_ctl_estimates(fsr_ctl* ctl, int32_t context, int64_t request, double* a_hat, double* T_hat, double* J) {
    if (!ctl) return fail(FSR_EINVAL, "fsr_ctl_estimates: ctl is null");
    const int m = ctl->cfg.n_lengths;
    std::vector<double> a_sum(m, 0.0), t_sum(m, 0.0);
    std::vector<int> a_cnt(m, 0), t_cnt(m, 0);
    if (const Window* w = ctl->find(context, request))
        for (const Obs& o : *w) {
            const int k = ctl->index_of(o.s);
            a_sum[k] += o.a;
            ++a_cnt[k];
        }
    auto c = ctl->contexts.find(context);
    if (c != ctl->contexts.end())
        for (const auto& rw : c->second)
            for (const Obs& o : rw.second) {
                const int k = ctl->index_of(o.s);
                t_sum[k] += o.T;
                ++t_cnt[k];
            }
    for (int k = 0; k < m; ++k) {
        const double a = a_cnt[k] ? a_sum[k] / a_cnt[k] : kNaN;
        const double t = t_cnt[k] ? t_sum[k] / t_cnt[k] : kNaN;
        if (a_hat) a_hat[k] = a;
        if (T_hat) T_hat[k] = t;
        if (J) J[k] = t / ((double)ctl->cfg.lengths[k] * a + ctl->cfg.eps);
    }
    return FSR_OK;
}

extern "C" int fsr_ctl_best_length(fsr_ctl* ctl, int32_t context, int64_t request, int32_t* s_out) {
    if (!ctl || !s_out) return fail(FSR_EINVAL, "fsr_ctl_best_length: null argument");
    double J[FSR_CTL_MAX_LENGTHS];
    const int rc = fsr_ctl_estimates(ctl, context, request, nullptr, nullptr, J);
    if (rc != FSR_OK) return rc;
    int best = -1;
    for (int k = 0; k < ctl->cfg.n_lengths; ++k)
        if (!std::isnan(J[k]) && (best < 0 || J[k] < J[best])) best = k;
    if (best < 0) return fail(FSR_ESHAPE, "fsr_ctl_best_length: no candidate length observed yet");
    *s_out = ctl->cfg.lengths[best];
    return FSR_OK;
}

extern "C" int fsr_ctl_posterior(fsr_ctl* ctl, int32_t context, int64_t request, double* mu, double* sigma) {
    if (!ctl) return fail(FSR_EINVAL, "fsr_ctl_posterior: ctl is null");
    return posterior(ctl, ctl->find(context, request), mu, sigma);
}

extern "C" int fsr_ctl_choose(fsr_ctl* ctl, int32_t context, int64_t request, int32_t* s_out) {
    if (!ctl || !s_out) return fail(FSR_EINVAL, "fsr_ctl_choose: null argument");
    double mu[FSR_CTL_MAX_LENGTHS], sigma[FSR_CTL_MAX_LENGTHS];
    const Window* w = ctl->find(context, request);
    const int rc = posterior(ctl, w, mu, sigma);
    if (rc != FSR_OK) return rc;
    const fsr_ctl_config& c = ctl->cfg;
    const double n = (double)(w ? w->size() : 0) + 1.0;
    const double pi = 3.14159265358979323846;
    const double beta = c.beta > 0.0 ? c.beta : 2.0 * std::log(c.n_lengths * n * n * pi * pi / (6.0 * c.delta));
    int best = 0;
    double best_v = 0.0;
    for (int k = 0; k < c.n_lengths; ++k) {
        const double v = mu[k] - std::sqrt(std::max(beta, 0.0)) * sigma[k];
        if (k == 0 || v < best_v) {
            best = k;
            best_v = v;
        }
    }
    *s_out = c.lengths[best];
    return FSR_OK;
}

extern "C" int fsr_expected_rejected(int32_t n, const int32_t* s, const double* a_hat, double* k_rej) {
    if (n < 0 || !k_rej || (n > 0 && (!s || !a_hat))) return fail(FSR_EINVAL, "fsr_expected_rejected: bad argument");
    double sum = 0.0;
    for (int i = 0; i < n; ++i) {
        if (s[i] < 0 || !(a_hat[i] >= 0.0 && a_hat[i] <= 1.0))
            return fail(FSR_EINVAL, "fsr_expected_rejected: request %d has s=%d a_hat=%g", i, s[i], a_hat[i]);
        sum += (double)s[i] * (1.0 - a_hat[i]);
    }
    *k_rej = sum;
    return FSR_OK;
}

extern "C" int fsr_prune_trigger(int32_t L, int32_t layer, double T_t, double T_ee, double T_pr, double* T_save_out, int32_t* prune) {
    if (!prune) return fail(FSR_EINVAL, "fsr_prune_trigger: prune is null");
    if (L < 1 || layer < 0 || layer > L || !(T_t > 0.0) || !(T_ee >= 0.0) || !(T_pr >= 0.0))
        return fail(FSR_EINVAL, "fsr_prune_trigger: L=%d layer=%d T_t=%g T_ee=%g T_pr=%g", L, layer, T_t, T_ee, T_pr);
    const double dL = (double)L * T_ee / T_t;                      // Eq. 7
    const double left = std::max((double)(L - layer) - dL, 0.0);   // Eq. 8
    const double T_save = left / (double)L * T_t;                  // Eq. 9
    if (T_save_out) *T_save_out = T_save;
    *prune = T_save > T_pr ? 1 : 0;                                // Eq. 10
    return FSR_OK;
}

extern "C" int fsr_latency_eval(const fsr_latency_model* m, double b, double s, double r, double* T) {
    if (!m || !T) return fail(FSR_EINVAL, "fsr_latency_eval: null argument");
    if (!form_ok(m->form)) return fail(FSR_EINVAL, "fsr_latency_eval: form=%d", m->form);
    *T = eval_model(*m, b, s, r);
    return FSR_OK;
}

extern "C" int fsr_latency_fit(int32_t form, int32_t n, const double* b, const double* s, const double* r, const double* T,
                               fsr_latency_model* out, double* rms_out) {
    if (!form_ok(form)) return fail(FSR_EINVAL, "fsr_latency_fit: form=%d", form);
    if (!b || !s || !r || !T || !out) return fail(FSR_EINVAL, "fsr_latency_fit: null argument");
    const int p = base_terms(form);
    if (n < p + 2) return fail(FSR_ESHAPE, "fsr_latency_fit: %d points cannot determine the model", n);
    std::vector<double> x(n), phi(n * 3);
    for (int j = 0; j < n; ++j) {
        x[j] = share_of(form, r[j]);
        base_features(form, b[j], s[j], &phi[j * 3]);
    }
    // candidate knees: none (one piece), or between consecutive distinct shares with at least two
    // distinct shares on either side (a piece is a line in x)
    std::vector<double> xs(x);
    std::sort(xs.begin(), xs.end());
    xs.erase(std::unique(xs.begin(), xs.end()), xs.end());
    std::vector<double> knees;
    knees.push_back(xs.back());  // every point in the first piece
    for (size_t k = 1; k + 2 < xs.size(); ++k) knees.push_back(0.5 * (xs[k] + xs[k + 1]));

    std::vector<double> t(T, T + n), F(n * 4), theta(4), base(n), fac(n);
    double best_sse = std::numeric_limits<double>::infinity();
    fsr_latency_model best{};
    for (double knee : knees) {
        // start: the base alone (factor 1)
        std::vector<double> Fb(n * p);
        for (int j = 0; j < n; ++j)
            for (int u = 0; u < p; ++u) Fb[j * p + u] = phi[j * 3 + u];
        double th_b[3] = {0, 0, 0}, th_f[4] = {1, 0, 1, 0};
        if (!least_squares(Fb, t, n, p, th_b)) continue;
        double sse = std::numeric_limits<double>::infinity();
        const bool one_piece = knee >= xs.back();
        for (int it = 0; it < 200; ++it) {
            for (int j = 0; j < n; ++j) {
                base[j] = 0.0;
                for (int u = 0; u < p; ++u) base[j] += th_b[u] * phi[j * 3 + u];
            }
            // factor given the base: T ~ (a_k - g_k x) base, linear in (a1, g1, a2, g2)
            const int pf = one_piece ? 2 : 4;
            std::vector<double> Ff(n * pf, 0.0);
            for (int j = 0; j < n; ++j) {
                const int piece = (!one_piece && x[j] > knee) ? 1 : 0;
                Ff[j * pf + 2 * piece] = base[j];
                Ff[j * pf + 2 * piece + 1] = -x[j] * base[j];
            }
            double th[4] = {1, 0, 1, 0};
            if (!least_squares(Ff, t, n, pf, th)) break;
            th_f[0] = th[0]; th_f[1] = th[1];
            th_f[2] = one_piece ? th[0] : th[2];
            th_f[3] = one_piece ? th[1] : th[3];
            // base given the factor
            for (int j = 0; j < n; ++j) {
                const bool second = !one_piece && x[j] > knee;
                fac[j] = second ? th_f[2] - th_f[3] * x[j] : th_f[0] - th_f[1] * x[j];
                for (int u = 0; u < p; ++u) Fb[j * p + u] = fac[j] * phi[j * 3 + u];
            }
            if (!least_squares(Fb, t, n, p, th_b)) break;
            double e = 0.0;
            for (int j = 0; j < n; ++j) {
                double bj = 0.0;
                for (int u = 0; u < p; ++u) bj += th_b[u] * phi[j * 3 + u];
                const double d = fac[j] * bj - t[j];
                e += d * d;
            }
            const bool done = !(e < sse * (1.0 - 1e-12));
            sse = std::min(sse, e);
            if (done) break;
        }
        if (sse < best_sse && th_f[0] != 0.0) {
            best_sse = sse;
            // the free scale: a1 = 1
            const double k = th_f[0];
            best.form = form;
            best.reserved = 0;
            best.a1 = 1.0; best.g1 = th_f[1] / k; best.a2 = th_f[2] / k; best.g2 = th_f[3] / k;
            best.knee = knee;
            best.alpha = th_b[0] * k; best.beta = th_b[1] * k; best.c = p == 3 ? th_b[2] * k : 0.0;
        }
    }
    if (!std::isfinite(best_sse)) return fail(FSR_ESHAPE, "fsr_latency_fit: the points do not determine a model");
    *out = best;
    if (rms_out) *rms_out = std::sqrt(best_sse / n);
    return FSR_OK;
}

extern "C" int fsr_chunk_size(const fsr_latency_model* draft, const fsr_latency_model* target, double b, double r, int32_t s,
                              double T_hat, int32_t n_candidates, const int32_t* candidates, int32_t* s_c, double* T_chunked) {
    if (!draft || !target || !s_c || n_candidates < 0 || (n_candidates > 0 && !candidates))
        return fail(FSR_EINVAL, "fsr_chunk_size: null argument");
    if (draft->form != FSR_LAT_DRAFT || target->form != FSR_LAT_TARGET) return fail(FSR_EINVAL, "fsr_chunk_size: wrong model forms");
    if (s < 1 || !(T_hat > 0.0)) return fail(FSR_EINVAL, "fsr_chunk_size: s=%d T_hat=%g", s, T_hat);
    int best = 0;
    double best_t = std::numeric_limits<double>::infinity();
    for (int k = 0; k < n_candidates; ++k) {
        const int sc = candidates[k];
        if (sc < 1 || sc > s) return fail(FSR_EINVAL, "fsr_chunk_size: candidate %d outside 1..%d", sc, s);
        const int chunks = (s + sc - 1) / sc;
        const double t = eval_model(*draft, b, sc, r) + chunks * eval_model(*target, b, sc, r);
        if (t < best_t) {
            best_t = t;
            best = sc;
        }
    }
    const bool worth = best > 0 && best_t < T_hat;
    *s_c = worth ? best : 0;
    if (T_chunked) *T_chunked = best > 0 ? best_t : kNaN;
    return FSR_OK;
}
