"""Pins of the oracle's greedy (temperature 0) verification against things other than itself:
numpy's arg-max, the already pinned probabilistic rule on one-hot target rows (which it must
equal), the low-temperature limit of the LOGITS mode, ties, and hand-made cases."""
import numpy as np
import pytest

import workloads


def _layout(spec):
    spec = np.asarray(spec, np.int32)
    return workloads.exclusive_offsets(spec + 1), workloads.exclusive_offsets(spec)


def _python_greedy(z, toks, cu_t, cu_d, S_max):
    """The rule spelled with numpy's argmax (first maximum), in python loops."""
    B = len(cu_t) - 1
    em = np.full((B, S_max + 1), -1, np.int32)
    acc, nem = np.zeros(B, np.int32), np.zeros(B, np.int32)
    for i in range(B):
        d, t = cu_d[i + 1] - cu_d[i], cu_t[i + 1] - cu_t[i]
        n = 0
        while n < d and toks[cu_d[i] + n] == int(np.argmax(z[cu_t[i] + n])):
            em[i, n] = toks[cu_d[i] + n]
            n += 1
        acc[i] = n
        if n < d or t == d + 1:
            em[i, n] = int(np.argmax(z[cu_t[i] + n]))
            nem[i] = n + 1
        else:
            nem[i] = n
    return acc, nem, em


def test_matches_numpy_argmax_on_random_rows_with_planted_matches(oracle):
    rng = np.random.default_rng(2)
    V = 500
    spec = [0, 1, 4, 8, 3, 6]
    cu_t, cu_d = _layout(spec)
    z = rng.standard_normal((int(cu_t[-1]), V)).astype(np.float32)
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    # make runs of matching drafts of different lengths: all of request 2, first 3 of request 3, none of 4
    for i, upto in ((2, 4), (3, 3), (5, 5)):
        for j in range(upto):
            toks[cu_d[i] + j] = int(np.argmax(z[cu_t[i] + j]))
    r = oracle.greedy_accept(z, toks, cu_t, cu_d, S_max=8)
    acc, nem, em = _python_greedy(z, toks, cu_t, cu_d, 8)
    assert np.array_equal(r["accepted_len"], acc) and np.array_equal(r["n_emitted"], nem)
    assert np.array_equal(r["emitted"], em)
    assert list(acc[[2, 3, 5]]) == [4, 3, 5] and nem[2] == 5 and nem[0] == 1


def test_equals_probabilistic_rule_on_one_hot_targets(oracle):
    """With the target row replaced by the one-hot distribution of its arg-max, speculative sampling
    accepts exactly the drafts equal to that token and resamples exactly that token, whatever the
    uniforms and the draft distribution are: the greedy rule must give the same result."""
    b = workloads.make_batch(1, rep=8, keep_logits=True, draft_mode="noise")
    hot = np.zeros_like(b.p_target)
    hot[np.arange(b.N), np.argmax(b.z_target, axis=1)] = 1.0
    prob = oracle.spec_accept(hot, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, S_max=b.S_max)
    gr = oracle.greedy_accept(b.z_target, b.draft_tokens, b.cu_q, b.cu_d, S_max=b.S_max)
    for k in ("accepted_len", "n_emitted", "emitted"):
        assert np.array_equal(prob[k], gr[k]), k
    assert gr["accepted_len"].sum() > 0 and (gr["accepted_len"] < b.spec_lens).any()


def test_is_the_low_temperature_limit_of_logits_mode(oracle):
    b = workloads.make_batch(1, rep=9, keep_logits=True, draft_mode="noise")
    cold = oracle.spec_accept(b.z_target, b.z_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                              S_max=b.S_max, mode=oracle.LOGITS, temperature=1e-4)
    # at this temperature the draft rows are one-hot too; a draft is then its own row's arg-max with
    # probability one under the draft's own sampling, but here drafts were drawn at temperature 1, so
    # compare only the target-side outcome: accepted run and the token taken from the target
    gr = oracle.greedy_accept(b.z_target, b.draft_tokens, b.cu_q, b.cu_d, S_max=b.S_max)
    assert np.array_equal(cold["accepted_len"], gr["accepted_len"])
    assert np.array_equal(cold["emitted"], gr["emitted"])


def test_ties_go_to_the_lowest_id_and_hand_cases(oracle):
    V = 6
    # request 0: 2 drafts; request 1: 1 draft, no bonus row; request 2: no drafts (plain decode)
    cu_t = np.array([0, 3, 4, 5], np.int32)
    cu_d = np.array([0, 2, 3, 3], np.int32)
    z = np.array([[1, 5, 5, 0, 5, 2],      # arg-max 1 (tie 1,2,4 -> lowest)
                  [0, 0, 0, 0, 0, 0],      # all equal -> 0
                  [3, 1, 2, 9, 9, 0],      # bonus row: 3
                  [0, 7, 1, 1, 1, 1],      # request 1 row 0: 1
                  [2, 2, 8, 8, 1, 8]],     # request 2: 2
                 np.float32)
    toks = np.array([1, 0, 1], np.int32)
    r = oracle.greedy_accept(z, toks, cu_t, cu_d, S_max=2)
    assert list(r["accepted_len"]) == [2, 1, 0]
    assert r["emitted"].tolist() == [[1, 0, 3], [1, -1, -1], [2, -1, -1]]
    assert list(r["n_emitted"]) == [3, 1, 1]
    toks2 = np.array([2, 0, 4], np.int32)   # a tied but not-lowest id does not match
    r2 = oracle.greedy_accept(z, toks2, cu_t, cu_d, S_max=2)
    assert list(r2["accepted_len"]) == [0, 0, 0]
    assert r2["emitted"].tolist() == [[1, -1, -1], [1, -1, -1], [2, -1, -1]]


def test_row_maps_and_chunked_equals_one_shot(oracle):
    """Frontier chunks with greedy verification emit what the one-shot call emits (Sec. 3.3)."""
    b = workloads.make_batch(5, rep=4, B=20, V=64, with_kv=False, keep_logits=True)
    # plant long matching runs so that several chunks are needed
    for i in range(b.B):
        for j in range(int(b.spec_lens[i]) - (i % 3)):
            b.draft_tokens[b.cu_d[i] + j] = int(np.argmax(b.z_target[b.cu_q[i] + j]))
    one = oracle.greedy_accept(b.z_target, b.draft_tokens, b.cu_q, b.cu_d, S_max=b.S_max)
    b.p_target = b.z_target
    chunks = workloads.chunk_plan(5, b.spec_lens, s_c=2)
    ch = oracle.verify_chunked(b, chunks, with_attention=False, mode=oracle.GREEDY)
    assert np.array_equal(ch["accepted_len"], one["accepted_len"])
    assert np.array_equal(ch["emitted"], one["emitted"])
    perm = np.random.default_rng(0).permutation(b.N).astype(np.int32)
    inv = np.argsort(perm).astype(np.int32)
    mapped = oracle.greedy_accept(b.z_target[perm], b.draft_tokens, b.cu_q, b.cu_d, S_max=b.S_max, t_rows=inv)
    assert np.array_equal(mapped["emitted"], one["emitted"])


def test_nan_scores_never_win(oracle):
    """A NaN score counts as minus infinity: it loses to every number, ties with -inf resolve to the lowest id,
    a row of NaN alone yields token 0."""
    nan, inf = np.nan, np.inf
    z = np.array([[nan, 1.0, 3.0, nan, 3.0],      # NaN in front must not shadow the maximum: 2
                  [nan, nan, nan, nan, nan],      # 0
                  [-inf, nan, -inf, nan, -inf],   # all equal after the rule: 0
                  [nan, -inf, -5.0, nan, -inf],   # 2
                  [2.0, nan, 2.0, 1.0, nan]], np.float32)   # 0
    cu_t = np.arange(6, dtype=np.int32)
    cu_d = np.zeros(6, np.int32)
    r = oracle.greedy_accept(z, np.zeros(0, np.int32), cu_t, cu_d, S_max=0)
    assert r["emitted"][:, 0].tolist() == [2, 0, 0, 2, 0]
    # the same rows as drafts' targets: a draft equal to that arg-max is accepted, any other is not
    toks = np.array([2, 1, 0, 2, 4], np.int32)
    r = oracle.greedy_accept(np.concatenate([z, z[:0]]), toks, cu_t, np.arange(6, dtype=np.int32), S_max=1)
    assert r["accepted_len"].tolist() == [1, 0, 1, 1, 0]
    assert np.array_equal(np.nanargmax(np.where(np.isnan(z[[0, 3, 4]]), -inf, z[[0, 3, 4]]), axis=1), [2, 2, 0])
