"""Host controller (Sec. 3.1 Eqs. 1-4, Sec. 3.2 Eqs. 5-10, Sec. 3.3 chunk rule, Sec. 3.4 Eqs. 11-14).

First the oracle is pinned to values worked out by hand and to closed forms; then the C++ controller is
compared with the oracle on seeded random histories.  No GPU."""
import math
import os

import numpy as np
import pytest

from oracle import controller as oc


@pytest.fixture(scope="module")
def ctl():
    from paper_2604_20503_amd import binding, controller
    if not os.path.exists(binding.library_path()):
        from paper_2604_20503_amd.build import build
        build()
    return controller


# ------------------------------------------------------------------ pins of the oracle
def test_oracle_objective_by_hand():
    """Eq. 1 / Eq. 2 / Eq. 4 on numbers small enough to do on paper."""
    c = oc.Controller(lengths=(2, 4, 8), window=8, eps=0.5)
    c.observe(0, 7, 4, 2, 10.0)    # a = 0.5, J = 10 / (4 * 0.5 + 0.5) = 4
    c.observe(0, 7, 4, 4, 14.0)    # a = 1.0, J = 14 / 4.5
    c.observe(0, 7, 8, 2, 20.0)    # a = 0.25
    c.observe(0, 9, 4, 0, 18.0)    # another request of the same context: only T_hat(4) sees it
    a_hat, T_hat, J = c.estimates(0, 7)
    assert math.isnan(a_hat[0]) and math.isnan(T_hat[0]) and math.isnan(J[0])
    assert a_hat[1] == 0.75 and T_hat[1] == 14.0 and J[1] == 14.0 / (4 * 0.75 + 0.5)
    assert a_hat[2] == 0.25 and T_hat[2] == 20.0 and J[2] == 20.0 / (8 * 0.25 + 0.5)
    assert c.best_length(0, 7) == 4          # 4.0 < 8.0
    assert [o[3] for o in c.obs[0][7]] == [4.0, 14.0 / 4.5, 8.0]
    assert c.best_length(1, 7) is None       # other context: nothing observed
    # the window forgets: after 8 more outcomes at s = 2 nothing of s = 4 or 8 is left for request 7
    for _ in range(8):
        c.observe(0, 7, 2, 1, 6.0)
    a_hat, T_hat, J = c.estimates(0, 7)
    assert a_hat[0] == 0.5 and math.isnan(a_hat[1]) and T_hat[1] == 18.0 and math.isnan(T_hat[2])


def test_oracle_gp_closed_forms():
    """One observation: mu(s0) = y0 exactly when centred (prior mean = window mean), and
    sigma^2(s0) = sf - sf^2 / (sf + sn) in standardised units; far away the prior comes back.
    Two observations at one s: the 2x2 system solved by hand."""
    c = oc.Controller(lengths=(2, 4, 6, 30), length_scale=1.0, signal_var=1.5, noise_var=0.25)
    c.observe(0, 1, 4, 2, 9.0)
    y0 = 9.0 / (2 + 1e-6)
    mu, sigma = c.posterior(0, 1)
    assert np.allclose(mu, y0)                               # centred observation: posterior mean = window mean
    scale = y0                                               # zero variance -> |mean|
    assert math.isclose(sigma[1], scale * math.sqrt(1.5 - 1.5 ** 2 / 1.75), rel_tol=1e-12)
    k = 1.5 * math.exp(-2.0)                                 # k(2, 4) with l = 1
    assert math.isclose(sigma[0], scale * math.sqrt(1.5 - k * k / 1.75), rel_tol=1e-12)
    assert math.isclose(sigma[3], scale * math.sqrt(1.5), rel_tol=1e-9)
    # two observations at the same s: y = +-1 after standardising, K = [[sf+sn, sf], [sf, sf+sn]]
    c = oc.Controller(lengths=(4, 6), length_scale=1.0, signal_var=1.0, noise_var=0.5, eps=1e-12)
    c.observe(0, 1, 4, 4, 8.0)    # J = 2
    c.observe(0, 1, 4, 4, 16.0)   # J = 4
    mu, sigma = c.posterior(0, 1)
    assert math.isclose(mu[0], 3.0, rel_tol=1e-12)           # symmetric: the mean of the two
    # K^-1 [1,1]^T = [1,1]/(2 sf + sn) -> var = sf - 2 sf^2 / (2 sf + sn)
    assert math.isclose(sigma[0], 1.0 * math.sqrt(1.0 - 2.0 / 2.5), rel_tol=1e-12)
    # Eq. 3: an unexplored length with a large sigma wins once beta is large, loses when beta -> 0
    c = oc.Controller(lengths=(2, 10), length_scale=1.0, beta=1e-9)
    c.observe(0, 1, 2, 2, 4.0); c.observe(0, 1, 2, 1, 4.0); c.observe(0, 1, 10, 1, 9.0)
    assert c.choose(0, 1) == 2
    c.beta = 0.0   # schedule: beta_n = 2 ln(|S| n^2 pi^2 / (6 delta))
    mu, sigma = c.posterior(0, 1)
    beta = 2 * math.log(2 * 16 * math.pi ** 2 / 0.6)
    assert c.choose(0, 1) == (2, 10)[int(np.argmin(mu - math.sqrt(beta) * sigma))]
    # empty window: prior, ties go to the smallest candidate
    assert oc.Controller().choose(3, 3) == 2


def test_oracle_trigger_by_hand():
    """Eqs. 5-10 with L = 32, after layer 8."""
    assert oc.expected_rejected([4, 8, 2], [0.5, 0.25, 1.0]) == 4 * 0.5 + 8 * 0.75
    # dL = 32 * 0.5 / 4 = 4 layers; L_r' = 32 - 8 - 4 = 20; T_save = 20 / 32 * 4 = 2.5
    T_save, prune = oc.prune_trigger(32, 8, 4.0, 0.5, 2.4)
    assert T_save == 2.5 and prune
    assert not oc.prune_trigger(32, 8, 4.0, 0.5, 2.5)[1]            # strict inequality
    assert oc.prune_trigger(32, 30, 4.0, 0.5, 0.0) == (0.0, False)   # estimator slower than what is left


def test_oracle_latency_models_by_hand():
    """Eqs. 11-14: the share each form sees and the piece each share falls into."""
    p = (1.0, 0.5, 0.8, 0.2, 0.4, 2.0, 3.0, 5.0)   # a1 g1 a2 g2 knee alpha beta c
    assert oc.latency(oc.DRAFT, p, 4, 2, 0.25) == (1.0 - 0.5 * 0.25) * (2 * 4 + 3 * 2 + 5)
    assert oc.latency(oc.DRAFT, p, 4, 2, 0.5) == (0.8 - 0.2 * 0.5) * (2 * 4 + 3 * 2 + 5)
    assert oc.latency(oc.TARGET, p, 4, 2, 0.75) == (1.0 - 0.5 * 0.25) * ((2 * 4 + 3) * 2 + 5)   # its share is 1 - r
    assert oc.latency(oc.TARGET, p, 4, 2, 0.25) == (0.8 - 0.2 * 0.75) * ((2 * 4 + 3) * 2 + 5)
    assert oc.latency(oc.EXIT, p, 4, 2, 0.75) == (1.0 - 0.5 * 0.25) * (2 * 8 + 3)
    assert oc.latency(oc.PRUNE, p, 4, 2, 0.75) == (0.8 - 0.2 * 0.75) * (2 * 8 + 3)
    assert oc.latency(oc.DRAFT, p, 4, 2, 0.4) == (1.0 - 0.5 * 0.4) * 19    # the knee itself belongs to the first piece
    assert oc.latency(oc.KV, p, 4, 2, 0.75) == (1.0 - 0.5 * 0.25) * (2 * 8 + 3 * 4 + 5)


def planted(form, rng, n=60, noise=0.0):
    p = (1.0, 0.6, 0.7, 0.15, 0.45, 0.03, 0.2, 1.5 if form in (oc.DRAFT, oc.TARGET, oc.KV) else 0.0)
    b = rng.choice([8, 16, 64, 128, 256], size=n).astype(np.float64)
    s = rng.choice([2, 4, 6, 8, 10], size=n).astype(np.float64)
    r = rng.choice([0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9], size=n)
    T = oc.latency(form, p, b, s, r)
    return p, b, s, r, T * (1.0 + noise * rng.standard_normal(n))


@pytest.mark.parametrize("form", [oc.DRAFT, oc.TARGET, oc.EXIT, oc.PRUNE, oc.KV])
def test_oracle_fit_recovers_planted_model(form):
    rng = np.random.default_rng(form)
    p, b, s, r, T = planted(form, rng)
    q, rms = oc.fit_latency(form, b, s, r, T)
    assert rms < 1e-8 * T.mean()
    bb, ss, rr = np.meshgrid([10.0, 100.0], [3.0, 7.0], [0.15, 0.45, 0.85], indexing="ij")
    assert np.allclose(oc.latency(form, q, bb, ss, rr), oc.latency(form, p, bb, ss, rr), rtol=1e-6)


def test_oracle_chunk_rule_by_hand():
    d = (1.0, 0.0, 1.0, 0.0, 1.0, 0.0, 1.0, 0.0)    # T_q = s
    t = (1.0, 0.0, 1.0, 0.0, 1.0, 0.0, 2.0, 3.0)    # T_p = 2 s + 3
    # s = 8: s_c = 2 -> 2 + 4 * 7 = 30; s_c = 4 -> 4 + 2 * 11 = 26; s_c = 3 -> 3 + 3 * 9 = 30 (s / s_c rounded up)
    assert oc.chunk_size(d, t, 16, 0.25, 8, 27.0, [2, 3, 4]) == (4, 26.0)
    assert oc.chunk_size(d, t, 16, 0.25, 8, 26.0, [2, 3, 4]) == (0, 26.0)   # not strictly below: no overlap
    assert oc.chunk_size(d, t, 16, 0.25, 8, 26.0, [])[0] == 0


# ------------------------------------------------------------------ C++ controller vs the oracle
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("beta", [2.0, 0.0])
def test_controller_matches_oracle_on_random_histories(ctl, seed, beta):
    rng = np.random.default_rng(seed)
    lengths = (2, 4, 6, 8, 10) if seed != 2 else (1, 3, 4, 9)
    kw = dict(window=6 + seed, eps=1e-3, beta=beta, delta=0.2, length_scale=1.5 + seed, signal_var=1.0 + 0.5 * seed, noise_var=0.05 * (seed + 1))
    ref = oc.Controller(lengths=lengths, **kw)
    dut = ctl.Controller(lengths=lengths, **kw)
    for step in range(120):
        context, request = int(rng.integers(0, 2)), int(rng.integers(0, 3)) + (1 << 40)
        # follow the controller's own choice most of the time, as the serving loop would
        s_ref, s_dut = ref.choose(context, request), dut.choose(context, request)
        assert s_ref == s_dut, (step, s_ref, s_dut)
        s = s_ref if rng.random() < 0.7 else int(rng.choice(lengths))
        n_acc = int(rng.integers(0, s + 1))
        lat = float(1.0 + 0.3 * s + rng.random())
        ref.observe(context, request, s, n_acc, lat)
        dut.observe(context, request, s, n_acc, lat)
        if step % 7 == 0:
            for got, want in zip(dut.estimates(context, request), ref.estimates(context, request)):
                assert np.allclose(got, want, rtol=1e-13, atol=0, equal_nan=True)
            mu, sigma = dut.posterior(context, request)
            mu_r, sigma_r = ref.posterior(context, request)
            assert np.allclose(mu, mu_r, rtol=1e-9, atol=1e-12) and np.allclose(sigma, sigma_r, rtol=1e-7, atol=1e-10)
            assert dut.best_length(context, request) == ref.best_length(context, request)
        if step == 60:
            ref.forget((1 << 40) + 1)
            dut.forget((1 << 40) + 1)
    dut.close()


def test_controller_trigger_models_and_chunks_match_oracle(ctl):
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(0, 9))
        s = rng.integers(0, 11, size=n)
        a = rng.random(n)
        assert math.isclose(ctl.expected_rejected(list(s), list(a)), oc.expected_rejected(s, a), rel_tol=1e-14, abs_tol=0)
        L = int(rng.integers(1, 81)); layer = int(rng.integers(0, L + 1))
        T_t, T_ee, T_pr = float(rng.random() * 10 + 0.1), float(rng.random()), float(rng.random() * 3)
        got, want = ctl.prune_trigger(L, layer, T_t, T_ee, T_pr), oc.prune_trigger(L, layer, T_t, T_ee, T_pr)
        assert got[1] == want[1] and math.isclose(got[0], want[0], rel_tol=1e-14, abs_tol=0)
        form = int(rng.integers(0, 5))
        p = tuple(float(v) for v in rng.random(8))
        m = ctl.latency_model(form, *p)
        b_, s_, r_ = float(rng.integers(1, 300)), float(rng.integers(1, 12)), float(rng.random())
        assert math.isclose(ctl.latency_eval(m, b_, s_, r_), float(oc.latency(form, p, b_, s_, r_)), rel_tol=1e-14)
        pd, pt = tuple(float(v) for v in rng.random(8)), tuple(float(v) for v in rng.random(8))
        S = int(rng.integers(1, 13))
        cands = sorted(set(int(v) for v in rng.integers(1, S + 1, size=4)))
        T_hat = float(rng.random() * 40)
        got = ctl.chunk_size(ctl.latency_model(0, *pd), ctl.latency_model(1, *pt), b_, r_, S, T_hat, cands)
        want = oc.chunk_size(pd, pt, b_, r_, S, T_hat, cands)
        assert got[0] == want[0] and math.isclose(got[1], want[1], rel_tol=1e-13)


@pytest.mark.parametrize("form", [oc.DRAFT, oc.TARGET, oc.EXIT, oc.PRUNE, oc.KV])
@pytest.mark.parametrize("noise", [0.0, 0.03])
def test_controller_fit_matches_oracle_fit(ctl, form, noise):
    rng = np.random.default_rng(10 + form)
    p, b, s, r, T = planted(form, rng, n=80, noise=noise)
    model, rms = ctl.latency_fit(form, list(b), list(s), list(r), list(T))
    q, rms_ref = oc.fit_latency(form, b, s, r, T)
    assert model.a1 == 1.0
    if noise == 0.0:
        assert rms < 1e-7 * T.mean() and math.isclose(model.knee, 0.45, abs_tol=0.051)
        bb, ss, rr = np.meshgrid([10.0, 100.0], [3.0, 7.0], [0.15, 0.45, 0.85], indexing="ij")
        got = np.array([ctl.latency_eval(model, float(x), float(y), float(z)) for x, y, z in zip(bb.ravel(), ss.ravel(), rr.ravel())])
        assert np.allclose(got, oc.latency(form, p, bb, ss, rr).ravel(), rtol=1e-6)
    else:
        # both are local searches of the same least-squares problem: neither may be noticeably worse
        assert rms <= rms_ref * 1.02 and rms_ref <= rms * 1.02, (rms, rms_ref)
        assert math.isclose(rms, float(np.sqrt(np.mean((np.array([ctl.latency_eval(model, *v) for v in zip(b, s, r)]) - T) ** 2))), rel_tol=1e-9)


def test_controller_rejects_bad_arguments(ctl):
    from paper_2604_20503_amd.binding import FsrError
    with pytest.raises(FsrError):
        ctl.Controller(lengths=(4, 2))            # not increasing
    with pytest.raises(FsrError):
        ctl.Controller(window=0)
    c = ctl.Controller()
    with pytest.raises(FsrError):
        c.observe(0, 1, 3, 1, 1.0)                # 3 is not a candidate
    with pytest.raises(FsrError):
        c.observe(0, 1, 4, 5, 1.0)                # more accepted than drafted
    with pytest.raises(FsrError):
        c.best_length(0, 1)                       # nothing observed
    with pytest.raises(FsrError):
        ctl.prune_trigger(0, 0, 1.0, 0.1, 0.1)
    with pytest.raises(FsrError):
        ctl.latency_fit(0, [1.0] * 3, [1.0] * 3, [0.5] * 3, [1.0] * 3)
    with pytest.raises(FsrError):
        ctl.chunk_size(ctl.latency_model(1, 1, 0, 1, 0, 1, 0, 1, 0), ctl.latency_model(1, 1, 0, 1, 0, 1, 0, 1, 0), 1, 0.5, 4, 1.0, [2])


def test_oracle_gp_against_sklearn():
    """The oracle's Gaussian-process posterior (Eq. 3's mu and sigma) against scikit-learn's regressor with the same
    fixed kernel: an independent implementation of the same textbook formulas."""
    from sklearn.gaussian_process import GaussianProcessRegressor
    from sklearn.gaussian_process.kernels import RBF, ConstantKernel
    rng = np.random.default_rng(8)
    lengths = (2, 3, 4, 6, 8, 10, 12)
    c = oc.Controller(lengths=lengths, window=40, eps=1e-3, length_scale=1.7, signal_var=1.3, noise_var=0.07)
    for _ in range(25):
        s = int(rng.choice(lengths))
        c.observe(0, 5, s, int(rng.integers(0, s + 1)), float(1.0 + 0.2 * s + rng.random()))
    mu, sigma = c.posterior(0, 5)
    w = list(c.obs[0][5])
    X = np.array([[o[0]] for o in w], dtype=np.float64)
    y = np.array([o[3] for o in w])
    mean, scale = y.mean(), y.std()
    gp = GaussianProcessRegressor(kernel=ConstantKernel(1.3, "fixed") * RBF(1.7, "fixed"), alpha=0.07, optimizer=None,
                                  normalize_y=False).fit(X, (y - mean) / scale)
    pm, ps = gp.predict(np.array(lengths, dtype=np.float64)[:, None], return_std=True)
    assert np.allclose(mu, mean + scale * pm, rtol=1e-9, atol=1e-12)
    assert np.allclose(sigma, scale * ps, rtol=1e-6, atol=1e-9)
