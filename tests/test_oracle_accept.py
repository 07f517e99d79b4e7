"""Pins of the accept/reject oracle (Sec. 2.1: accept until the first mismatch, resample the
mismatched token from the target; Sec. 3.3: recovery token) against closed forms, exact
rational brute force, the output-distribution theorem and library routines."""
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax

import workloads


def _probs(rng, n, V, sigma=2.0):
    return workloads.softmax_rows_f32(rng.standard_normal((n, V)).astype(np.float32) * np.float32(sigma))


def exact_reference(p_rows, q_rows, toks, u_acc, u_s, has_bonus):
    """Independent definition in exact rational arithmetic (python Fractions) for one request."""
    F = lambda x: Fraction(float(x))
    d = len(toks)
    n = 0
    while n < d and F(u_acc[n]) * F(q_rows[n][toks[n]]) < F(p_rows[n][toks[n]]):
        n += 1
    if n < d:
        r = [max(F(a) - F(b), Fraction(0)) for a, b in zip(p_rows[n], q_rows[n])]
        if sum(r) == 0:
            r = [F(a) for a in p_rows[n]]
    elif has_bonus:
        r = [F(a) for a in p_rows[d]]
    else:
        return n, list(toks[:n])
    R = sum(r)
    c = Fraction(0)
    tok = None
    for v, m in enumerate(r):
        c += m
        if m > 0 and c > F(u_s) * R:
            tok = v
            break
    if tok is None:
        tok = max(v for v, m in enumerate(r) if m > 0)
    return n, list(toks[:n]) + [tok]


def _dyadic(rng, n, V):
    """Rows of multiples of 1/16 summing to 1 (many exact zeros and exact CDF ties with a k/16 uniform grid)."""
    out = np.zeros((n, V), np.float32)
    for r in range(n):
        out[r] = np.bincount(rng.integers(0, V, size=16), minlength=V) / 16.0
    return out


@pytest.mark.parametrize("dyadic", [False, True])
@pytest.mark.parametrize("V", [2, 5, 8])
def test_bruteforce_tiny_vocab_exact_rational(oracle, V, dyadic):
    rng = np.random.default_rng(100 + V)
    B = 200
    spec = rng.integers(0, 4, size=B).astype(np.int32)
    bonus = rng.integers(0, 2, size=B).astype(np.int32)
    bonus[spec == 0] = 1
    cu_d = workloads.exclusive_offsets(spec)
    cu_t = workloads.exclusive_offsets(spec + bonus)
    p = _probs(rng, int(cu_t[-1]), V)
    q = _probs(rng, int(cu_d[-1]), V)
    # sprinkle exact zeros and exact ties to exercise the edge rules
    p[rng.random(p.shape) < 0.15] = 0.0
    q[rng.random(q.shape) < 0.15] = 0.0
    p[:, 0] += (p.sum(axis=1) == 0)
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    grid = np.linspace(0, 1, 17, endpoint=False).astype(np.float32)
    if dyadic:  # u * R lands exactly on cumulative sums: pins the strict comparisons
        p, q = _dyadic(rng, int(cu_t[-1]), V), _dyadic(rng, int(cu_d[-1]), V)
        grid = (np.arange(16) / 16.0).astype(np.float32)
    u_acc = rng.choice(grid, size=int(cu_d[-1])).astype(np.float32)
    u_s = rng.choice(grid, size=B).astype(np.float32)
    r = oracle.spec_accept(p, q, toks, u_acc, u_s, cu_t, cu_d, S_max=3)
    for i in range(B):
        d = int(spec[i])
        n, em = exact_reference(p[cu_t[i]: cu_t[i + 1]], q[cu_d[i]: cu_d[i + 1]], toks[cu_d[i]: cu_d[i + 1]],
                                u_acc[cu_d[i]: cu_d[i + 1]], u_s[i], bool(bonus[i]))
        assert r["accepted_len"][i] == n, i
        assert r["n_emitted"][i] == len(em), i
        assert list(r["emitted"][i, : len(em)]) == em, i
        assert (r["emitted"][i, len(em):] == -1).all()


def test_draft_equals_target_accepts_everything(oracle):
    b = workloads.make_batch(1, with_kv=False, draft_mode="equal")
    r = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                           S_max=b.S_max)
    assert np.array_equal(r["accepted_len"], b.spec_lens)
    assert np.array_equal(r["n_emitted"], b.spec_lens + 1)
    for i in range(b.B):
        s = int(b.spec_lens[i])
        assert list(r["emitted"][i, :s]) == list(b.draft_tokens[b.cu_d[i]: b.cu_d[i + 1]])
        prow = b.p_target[b.cu_q[i] + s].astype(np.float64)
        c = np.cumsum(prow)
        assert r["emitted"][i, s] == np.searchsorted(c, float(b.u_sample[i]) * c[-1], side="right")


def test_spec_len_zero_is_inverse_cdf_sampling(oracle):
    rng = np.random.default_rng(5)
    B, V = 64, 1000
    p = _probs(rng, B, V)
    u = rng.random(B, dtype=np.float32)
    cu_t = np.arange(B + 1, dtype=np.int32)
    cu_d = np.zeros(B + 1, np.int32)
    r = oracle.spec_accept(p, np.zeros((0, V), np.float32), np.zeros(0, np.int32), np.zeros(0, np.float32), u,
                           cu_t, cu_d, S_max=0)
    c = np.cumsum(p.astype(np.float64), axis=1)
    ref = [np.searchsorted(c[i], float(u[i]) * c[i, -1], side="right") for i in range(B)]
    assert list(r["emitted"][:, 0]) == ref
    assert (r["accepted_len"] == 0).all() and (r["n_emitted"] == 1).all()
    # the reported CDF interval brackets u
    assert ((r["cdf_lo"] <= u) & (u < r["cdf_hi"])).all()


def test_output_distribution_theorem_chi_square(oracle):
    """First emitted token ~ p_0 when the draft is drawn from q_0 (speculative sampling)."""
    rng = np.random.default_rng(11)
    V, n = 60, 400_000
    p = _probs(rng, 1, V, sigma=1.5)
    q = _probs(rng, 1, V, sigma=1.5)
    cq = np.cumsum(q[0].astype(np.float64))
    toks = np.minimum(np.searchsorted(cq, rng.random(n) * cq[-1], side="right"), V - 1).astype(np.int32)
    u_acc = rng.random(n, dtype=np.float32)
    u_s = rng.random(n, dtype=np.float32)
    # the target row is shared through t_rows; draft rows are replicated per slab of requests
    first = np.empty(n, np.int64)
    slab = 20_000
    qs = np.repeat(q, slab, axis=0)
    for a in range(0, n, slab):
        m = min(slab, n - a)
        cu_s = np.arange(m + 1, dtype=np.int32)
        rr = oracle.spec_accept(p, qs[:m], toks[a: a + m], u_acc[a: a + m], u_s[a: a + m], cu_s, cu_s, S_max=1,
                                t_rows=np.zeros(m, np.int32))
        first[a: a + m] = rr["emitted"][:, 0]
        assert (rr["n_emitted"] == 1).all()
        acc = rr["accepted_len"] if a == 0 else np.concatenate([acc, rr["accepted_len"]])
    obs = np.bincount(first, minlength=V).astype(np.float64)
    exp = p[0].astype(np.float64) / p[0].astype(np.float64).sum() * n
    keep = exp >= 5
    obs_p = np.append(obs[keep], obs[~keep].sum())
    exp_p = np.append(exp[keep], exp[~keep].sum())
    if exp_p[-1] == 0:
        obs_p, exp_p = obs_p[:-1], exp_p[:-1]
    chi2, pval = stats.chisquare(obs_p, exp_p)
    assert pval > 0.01, (chi2, pval)
    # closed form: P(accept at position 0) = sum_v min(p, q) = 1 - TV(p, q)
    alpha = np.minimum(p[0].astype(np.float64), q[0].astype(np.float64)).sum()
    rate = acc.mean()
    assert abs(rate - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / n), (rate, alpha)
    # a wrong residual (e.g. q - p) or a non-strict/inverted test would fail the chi-square above;
    # check the test has power: the draft-token histogram itself is far from p
    chi2_q, pval_q = stats.chisquare(np.bincount(toks, minlength=V)[keep], exp[keep] * (np.bincount(toks, minlength=V)[keep].sum() / exp[keep].sum()))
    assert pval_q < 1e-6


def test_expected_accepted_length_iid_rows(oracle):
    rng = np.random.default_rng(21)
    V, d, n = 40, 4, 60_000
    p = _probs(rng, d + 1, V, sigma=1.0)
    q = _probs(rng, d, V, sigma=1.0)
    alphas = np.minimum(p[:d].astype(np.float64), q.astype(np.float64)).sum(axis=1)
    expect = sum(np.prod(alphas[: k + 1]) for k in range(d))
    toks = np.empty((n, d), np.int32)
    for k in range(d):
        cq = np.cumsum(q[k].astype(np.float64))
        toks[:, k] = np.minimum(np.searchsorted(cq, rng.random(n) * cq[-1], side="right"), V - 1)
    cu_d = (np.arange(n + 1) * d).astype(np.int32)
    cu_t = (np.arange(n + 1) * (d + 1)).astype(np.int32)
    t_rows = np.tile(np.arange(d + 1, dtype=np.int32), n)
    q_rep = np.tile(q, (n, 1))
    r = oracle.spec_accept(p, q_rep, toks.reshape(-1), rng.random(n * d, dtype=np.float32),
                           rng.random(n, dtype=np.float32), cu_t, cu_d, S_max=d, t_rows=t_rows)
    mean = r["accepted_len"].mean()
    var = r["accepted_len"].var()
    assert abs(mean - expect) < 4 * np.sqrt(var / n), (mean, expect)
    assert (r["n_emitted"] == r["accepted_len"] + 1).all()


def test_point_mass_cases(oracle):
    V = 16
    rng = np.random.default_rng(3)
    p = _probs(rng, 2, V)
    p[0, 5] = 0.0
    q = np.zeros((1, V), np.float32)
    q[0, 5] = 1.0
    cu_t, cu_d = np.array([0, 2], np.int32), np.array([0, 1], np.int32)
    for u_a in (0.0, 0.3, 0.999):
        for u_s in (0.0, 0.25, 0.5, 0.999):
            r = oracle.spec_accept(p, q, np.array([5], np.int32), np.array([u_a], np.float32),
                                   np.array([u_s], np.float32), cu_t, cu_d, S_max=1)
            assert r["accepted_len"][0] == 0 and r["n_emitted"][0] == 1
            c = np.cumsum(p[0].astype(np.float64))  # residual = p since q is zero wherever p > 0
            assert r["emitted"][0, 0] == np.searchsorted(c, float(np.float32(u_s)) * c[-1], side="right")
    # target one-hot: whatever the draft, the token emitted at that position is the target's token
    p1 = np.zeros((2, V), np.float32)
    p1[0, 9] = 1.0
    p1[1, 2] = 1.0
    qd = _probs(rng, 1, V)
    for x in range(V):
        r = oracle.spec_accept(p1, qd, np.array([x], np.int32), np.array([0.5], np.float32),
                               np.array([0.7], np.float32), cu_t, cu_d, S_max=1)
        assert r["emitted"][0, 0] == 9
        assert r["accepted_len"][0] == (1 if x == 9 else 0)
        if x == 9:
            assert r["emitted"][0, 1] == 2 and r["n_emitted"][0] == 2
    # accept predicate edges: p >= q > 0 always accepts (u < 1); p = 0 always rejects, also when q = 0
    pe = np.full((2, V), 1.0 / V, np.float32)
    qe = pe[:1].copy()
    r = oracle.spec_accept(pe, qe, np.array([3], np.int32), np.array([np.nextafter(np.float32(1), np.float32(0))]),
                           np.array([0.1], np.float32), cu_t, cu_d, S_max=1)
    assert r["accepted_len"][0] == 1
    pz, qz = pe.copy(), qe.copy()
    pz[0, 3] = 0.0
    qz[0, 3] = 0.0
    r = oracle.spec_accept(pz, qz, np.array([3], np.int32), np.array([0.0], np.float32),
                           np.array([0.1], np.float32), cu_t, cu_d, S_max=1)
    assert r["accepted_len"][0] == 0 and r["emitted"][0, 0] != 3


def test_no_bonus_row_emits_only_accepted_drafts(oracle):
    b = workloads.make_batch(1, with_kv=False, draft_mode="equal")
    # drop the bonus row of every request: target rows = draft rows
    t_rows = np.concatenate([np.arange(b.cu_q[i], b.cu_q[i] + b.spec_lens[i]) for i in range(b.B)]).astype(np.int32)
    r = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_d, b.cu_d,
                           S_max=b.S_max, t_rows=t_rows)
    assert np.array_equal(r["accepted_len"], b.spec_lens)
    assert np.array_equal(r["n_emitted"], b.spec_lens)
    assert np.isnan(r["cdf_lo"]).all()


def test_logits_mode_matches_library_softmax(oracle):
    rng = np.random.default_rng(8)
    B, V, T = 40, 300, 0.8
    spec = rng.integers(0, 5, size=B).astype(np.int32)
    cu_d = workloads.exclusive_offsets(spec)
    cu_t = workloads.exclusive_offsets(spec + 1)
    z_t = (rng.standard_normal((int(cu_t[-1]), V)) * 2).astype(np.float32)
    z_d = np.empty((int(cu_d[-1]), V), np.float32)
    for i in range(B):
        z_d[cu_d[i]: cu_d[i + 1]] = z_t[cu_t[i]: cu_t[i] + spec[i]] + rng.standard_normal((spec[i], V)).astype(np.float32) * 0.5
    p_t = softmax(z_t.astype(np.float64) / T, axis=1)
    p_d = softmax(z_d.astype(np.float64) / T, axis=1)
    toks = np.array([rng.choice(V, p=p_d[r]) for r in range(p_d.shape[0])], np.int32)
    u_a = rng.random(int(cu_d[-1]), dtype=np.float32)
    u_s = rng.random(B, dtype=np.float32)
    r = oracle.spec_accept(z_t, z_d, toks, u_a, u_s, cu_t, cu_d, S_max=4, mode=oracle.LOGITS, temperature=T)
    n_rej = 0
    for i in range(B):
        d = int(spec[i])
        n = 0
        while n < d and float(u_a[cu_d[i] + n]) * p_d[cu_d[i] + n, toks[cu_d[i] + n]] < p_t[cu_t[i] + n, toks[cu_d[i] + n]]:
            n += 1
        res = np.maximum(p_t[cu_t[i] + n] - p_d[cu_d[i] + n], 0) if n < d else p_t[cu_t[i] + d]
        n_rej += n < d
        c = np.cumsum(res)
        tok = int(np.searchsorted(c, float(u_s[i]) * c[-1], side="right"))
        assert r["accepted_len"][i] == n
        assert r["emitted"][i, n] == tok, (i, r["emitted"][i], tok)
    assert 0 < n_rej < B


@pytest.mark.parametrize("mode", ["probs", "logits"])
def test_bf16_rows_equal_their_widened_fp32_rows(oracle, mode):
    """Rows given as bf16 bit patterns are read as the fp32 values with the same leading bits: the
    result must be that of the (separately pinned) fp32 path on the widened rows."""
    b = workloads.make_batch(1, rep=17, keep_logits=True, draft_mode="noise")
    src_t, src_d = (b.p_target, b.p_draft) if mode == "probs" else (b.z_target, b.z_draft)
    bits_t, bits_d = workloads.f32_to_bf16_bits(src_t), workloads.f32_to_bf16_bits(src_d)
    wide_t, wide_d = workloads.bf16_bits_to_f32(bits_t), workloads.bf16_bits_to_f32(bits_d)
    kw = dict(S_max=b.S_max, mode=oracle.PROBS if mode == "probs" else oracle.LOGITS, temperature=0.8)
    ref = oracle.spec_accept(wide_t, wide_d, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, **kw)
    got = oracle.spec_accept(bits_t, bits_d, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, dtype="bf16", **kw)
    for k in ("accepted_len", "n_emitted", "emitted"):
        assert np.array_equal(ref[k], got[k]), k
    assert np.array_equal(ref["cdf_lo"], got["cdf_lo"], equal_nan=True)


def test_neighbour_tokens_of_the_drawn_token(oracle):
    """tok_below / tok_above: nearest positive-mass ids around the drawn token, written out by hand on
    rows with zero-mass gaps (bonus draw from p, so the mass row is the target row itself)."""
    p = np.array([[0.25, 0.0, 0.25, 0.0, 0.5, 0.0],      # u = 0.3  -> token 2, neighbours 0 and 4
                  [0.0, 0.5, 0.0, 0.0, 0.5, 0.0],        # u = 0.1  -> token 1, nothing below, 4 above
                  [0.0, 0.5, 0.0, 0.0, 0.5, 0.0],        # u = 0.9  -> token 4, 1 below, nothing above
                  [0.0, 0.0, 1.0, 0.0, 0.0, 0.0]], np.float32)   # one-hot: no neighbours
    u = np.array([0.3, 0.1, 0.9, 0.5], np.float32)
    cu_t = np.arange(5, dtype=np.int32)
    cu_d = np.zeros(5, np.int32)
    r = oracle.spec_accept(p, np.zeros((0, 6), np.float32), np.zeros(0, np.int32), np.zeros(0, np.float32), u, cu_t, cu_d,
                           S_max=0)
    assert r["emitted"][:, 0].tolist() == [2, 1, 4, 2]
    assert r["tok_below"].tolist() == [0, -1, 1, -1]
    assert r["tok_above"].tolist() == [4, 4, -1, -1]
    # brute force on random sparse rows
    rng = np.random.default_rng(5)
    for _ in range(50):
        V = int(rng.integers(2, 12))
        row = rng.random(V) * (rng.random(V) < 0.6)
        if row.sum() == 0:
            row[rng.integers(V)] = 1.0
        row = (row / row.sum()).astype(np.float32)[None]
        uu = np.array([rng.random()], np.float32)
        r = oracle.spec_accept(row, np.zeros((0, V), np.float32), np.zeros(0, np.int32), np.zeros(0, np.float32), uu,
                               np.array([0, 1], np.int32), np.zeros(2, np.int32), S_max=0)
        t = int(r["emitted"][0, 0])
        pos = np.flatnonzero(row[0] > 0)
        k = int(np.searchsorted(pos, t))
        assert pos[k] == t
        assert r["tok_below"][0] == (pos[k - 1] if k > 0 else -1)
        assert r["tok_above"][0] == (pos[k + 1] if k + 1 < len(pos) else -1)
