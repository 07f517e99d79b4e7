"""Oracle of the host controller: TEST INFRASTRUCTURE ONLY (tests/ may import it; the product never does).

Plain numpy / scipy, float64, written from the paper: the cost objective and its minimiser (Sec. 3.1,
Eqs. 1-2), the GP-LCB step (Eqs. 3-4), the pruning trigger (Sec. 3.2, Eqs. 5-10), the chunk-size rule
(Sec. 3.3) and the latency models with a general-purpose non-linear least-squares fit (Sec. 3.4,
Eqs. 11-14).  Shares no code with the C++ controller.

Readings of what the paper leaves open (the product makes the same ones): the window
keeps the last W outcomes of a (context, request) pair; a_hat_i(s) averages that request's accepted
fractions at s, T_hat(s) the latencies of every request of the context at s; the Gaussian process has a
squared-exponential kernel on s, a constant prior mean equal to the window mean of the realised costs,
and works on costs standardised by the window's standard deviation (population form; |mean| or 1 when
it is zero); s / s_c of the chunk rule is rounded up.
"""
from __future__ import annotations

import math
from collections import defaultdict, deque

import numpy as np
from scipy.optimize import least_squares

DRAFT, TARGET, EXIT, PRUNE, KV = 0, 1, 2, 3, 4  # KV: this build's attention-only form, base = alpha b s + beta b + c


class Controller:
    def __init__(self, lengths=(2, 4, 6, 8, 10), window=32, eps=1e-6, beta=2.0, delta=0.1, length_scale=2.0,
                 signal_var=1.0, noise_var=0.1):
        self.lengths = list(lengths)
        self.window, self.eps, self.beta, self.delta = window, eps, beta, delta
        self.length_scale, self.signal_var, self.noise_var = length_scale, signal_var, noise_var
        self.obs = defaultdict(lambda: defaultdict(lambda: deque(maxlen=window)))  # context -> request -> (s, a, T, J)

    def observe(self, context, request, s, n_accepted, latency):
        a = n_accepted / s
        self.obs[context][request].append((s, a, latency, latency / (s * a + self.eps)))  # Eq. 4

    def forget(self, request):
        for c in self.obs.values():
            c.pop(request, None)

    def estimates(self, context, request):
        """Eq. 1 for every candidate length: (a_hat, T_hat, J), NaN where nothing was observed."""
        a_hat, T_hat, J = [], [], []
        mine = list(self.obs[context].get(request, ()))
        everyone = [o for w in self.obs[context].values() for o in w]
        for s in self.lengths:
            a = [o[1] for o in mine if o[0] == s]
            t = [o[2] for o in everyone if o[0] == s]
            a_hat.append(float(np.mean(a)) if a else math.nan)
            T_hat.append(float(np.mean(t)) if t else math.nan)
            J.append(T_hat[-1] / (s * a_hat[-1] + self.eps))
        return np.array(a_hat), np.array(T_hat), np.array(J)

    def best_length(self, context, request):
        """Eq. 2 over the observed candidates; None if there is none."""
        J = self.estimates(context, request)[2]
        if np.all(np.isnan(J)):
            return None
        return self.lengths[int(np.nanargmin(J))]

    def posterior(self, context, request):
        """mu, sigma of the Gaussian process over the candidate lengths (Eq. 3's ingredients)."""
        w = list(self.obs[context].get(request, ()))
        S = np.array(self.lengths, dtype=np.float64)
        kern = lambda x, y: self.signal_var * np.exp(-(x[:, None] - y[None, :]) ** 2 / (2 * self.length_scale ** 2))
        if not w:
            return np.zeros(len(S)), np.full(len(S), math.sqrt(self.signal_var))
        xs = np.array([o[0] for o in w], dtype=np.float64)
        y = np.array([o[3] for o in w], dtype=np.float64)
        mean, std = y.mean(), y.std()
        scale = std if std > 0 else (abs(mean) if abs(mean) > 0 else 1.0)
        K = kern(xs, xs) + self.noise_var * np.eye(len(xs))
        Ks = kern(S, xs)
        mu = Ks @ np.linalg.solve(K, (y - mean) / scale)
        var = self.signal_var - np.einsum("ij,ji->i", Ks, np.linalg.solve(K, Ks.T))
        return mean + scale * mu, scale * np.sqrt(np.maximum(var, 0.0))

    def choose(self, context, request):
        """Eq. 3: argmin of mu - sqrt(beta_n) sigma."""
        mu, sigma = self.posterior(context, request)
        n = len(self.obs[context].get(request, ())) + 1
        beta = self.beta if self.beta > 0 else 2 * math.log(len(self.lengths) * n * n * math.pi ** 2 / (6 * self.delta))
        return self.lengths[int(np.argmin(mu - math.sqrt(max(beta, 0.0)) * sigma))]


def expected_rejected(s, a_hat):
    """Eqs. 5-6."""
    return float(np.sum(np.asarray(s, dtype=np.float64) * (1.0 - np.asarray(a_hat, dtype=np.float64))))


def prune_trigger(L, layer, T_t, T_ee, T_pr):
    """Eqs. 7-10: (T_save, prune?)."""
    dL = L * T_ee / T_t
    left = max((L - layer) - dL, 0.0)
    T_save = left / L * T_t
    return T_save, T_save > T_pr


def latency(form, params, b, s, r):
    """Eqs. 11-14.  params = (a1, g1, a2, g2, knee, alpha, beta, c)."""
    a1, g1, a2, g2, knee, alpha, beta, c = params
    b, s, r = np.asarray(b, dtype=np.float64), np.asarray(s, dtype=np.float64), np.asarray(r, dtype=np.float64)
    x = r if form in (DRAFT, PRUNE) else 1.0 - r
    if form == DRAFT:
        base = alpha * b + beta * s + c
    elif form == TARGET:
        base = (alpha * b + beta) * s + c
    elif form == KV:
        base = alpha * b * s + beta * b + c
    else:
        base = alpha * b * s + beta
    return np.where(x <= knee, a1 - g1 * x, a2 - g2 * x) * base


def fit_latency(form, b, s, r, T, starts=6, seed=0):
    """Non-linear least squares of Eqs. 11-14 with a general-purpose solver (Levenberg-Marquardt-like
    trust region), every candidate knee, several starts.  Returns (params with a1 = 1, rms)."""
    b, s, r, T = (np.asarray(v, dtype=np.float64) for v in (b, s, r, T))
    x = r if form in (DRAFT, PRUNE) else 1.0 - r
    xs = np.unique(x)
    knees = [xs[-1]] + [0.5 * (xs[k] + xs[k + 1]) for k in range(1, len(xs) - 2)]
    rng = np.random.default_rng(seed)
    best = None
    for knee in knees:
        one = knee >= xs[-1]

        with_c = form in (DRAFT, TARGET, KV)  # the other two forms have no constant term

        def unpack(v):
            v = list(v) + ([] if with_c else [0.0])
            if one:
                g1, alpha, beta, c = v
                return (1.0, g1, 1.0, g1, knee, alpha, beta, c)
            g1, a2, g2, alpha, beta, c = v
            return (1.0, g1, a2, g2, knee, alpha, beta, c)

        resid = lambda v: latency(form, unpack(v), b, s, r) - T
        scale = float(np.mean(T))
        for k in range(starts):
            jitter = rng.uniform(0.5, 1.5, size=3) if k else np.ones(3)
            tail = [scale * 0.01 * jitter[0], scale * 0.01 * jitter[1]] + ([scale * jitter[2]] if with_c else [])
            v0 = ([0.1 * k] if one else [0.1 * k, 1.0, 0.1 * k]) + tail
            sol = least_squares(resid, v0, method="trf", x_scale="jac", xtol=1e-15, ftol=1e-15, gtol=1e-15, max_nfev=4000)
            sse = float(np.sum(sol.fun ** 2))
            if best is None or sse < best[1]:
                best = (unpack(sol.x), sse)
    return best[0], math.sqrt(best[1] / len(T))


def chunk_size(draft_params, target_params, b, r, s, T_hat, candidates):
    """Sec. 3.3: the candidate minimising T_q(s_c) + ceil(s / s_c) T_p(s_c), if below T_hat; else 0."""
    times = [float(latency(DRAFT, draft_params, b, sc, r)) + math.ceil(s / sc) * float(latency(TARGET, target_params, b, sc, r))
             for sc in candidates]
    if not times:
        return 0, math.nan
    k = int(np.argmin(times))
    return (candidates[k] if times[k] < T_hat else 0), times[k]
