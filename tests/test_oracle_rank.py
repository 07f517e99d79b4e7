"""Pins of the oracle's early-exit rank check (Sec. 3.2: a draft outside the Top-K set of the
intermediate logits is a pruning candidate; Sec. 4: only "do at least K tokens exceed the draft's
score" is checked) against things other than itself: closed forms on permutations, numpy's sort
and partition routines, tie cases, and the composition with pruning and restoring."""
import numpy as np
import pytest

import workloads


def _layout(spec, q_lens=None):
    spec = np.asarray(spec, np.int32)
    q = spec + 1 if q_lens is None else np.asarray(q_lens, np.int32)
    return workloads.exclusive_offsets(q), workloads.exclusive_offsets(spec)


def test_permutation_rows_have_closed_form_ranks(oracle):
    """A row that is a permutation of 0..V-1 ranks the token holding value x at V-1-x exactly;
    a draft passes iff that is below K (so rank K-1 passes and rank K does not)."""
    rng = np.random.default_rng(7)
    V, K = 97, 10
    spec = [3, 0, 5, 1]
    cu_q, cu_d = _layout(spec)
    N, N_d = int(cu_q[-1]), int(cu_d[-1])
    z = np.stack([rng.permutation(V) for _ in range(N)]).astype(np.float32)
    toks = rng.integers(0, V, size=N_d).astype(np.int32)
    # plant the boundary: one draft at rank exactly K-1, one at rank exactly K
    row0, row1 = int(cu_q[0]), int(cu_q[0]) + 1
    toks[cu_d[0]] = int(np.where(z[row0] == V - 1 - (K - 1))[0][0])
    toks[cu_d[0] + 1] = int(np.where(z[row1] == V - 1 - K)[0][0])
    r = oracle.topk_rank_check(z, toks, cu_q, cu_d, K=K)
    for i, s in enumerate(spec):
        assert r["keep"][cu_q[i]] == 1
        for j in range(s):
            want = V - 1 - int(z[cu_q[i] + j, toks[cu_d[i] + j]])
            assert r["rank"][cu_d[i] + j] == want
            assert r["keep"][cu_q[i] + j + 1] == (1 if want < K else 0)
    assert r["rank"][cu_d[0]] == K - 1 and r["keep"][cu_q[0] + 1] == 1
    assert r["rank"][cu_d[0] + 1] == K and r["keep"][cu_q[0] + 2] == 0


@pytest.mark.parametrize("K", [1, 10, 64])
def test_matches_numpy_sort_and_partition(oracle, K):
    """Continuous scores (no ties): the rank is the draft's position in numpy's descending sort,
    and passing is membership in numpy's Top-K partition."""
    b = workloads.make_batch(1, rep=3, keep_logits=True)
    z = b.z_target
    r = oracle.topk_rank_check(z, b.draft_tokens, b.cu_q, b.cu_d, K=K)
    for i in range(b.B):
        for j in range(int(b.spec_lens[i])):
            row, tok = int(b.cu_q[i]) + j, int(b.draft_tokens[b.cu_d[i] + j])
            order = np.argsort(-z[row].astype(np.float64), kind="stable")
            assert r["rank"][b.cu_d[i] + j] == int(np.where(order == tok)[0][0])
            topk = set(np.argpartition(-z[row], K - 1)[:K].tolist())
            assert bool(r["keep"][row + 1]) == (tok in topk)


def test_ties_count_strictly_greater_scores_only(oracle):
    """bf16 scores full of ties: rank = V - (number of scores <= the draft's), from numpy's sorted
    search; all-equal rows give rank 0 and pass for every K >= 1; K = 0 passes nothing."""
    rng = np.random.default_rng(11)
    V = 300
    spec = [4, 2, 6]
    cu_q, cu_d = _layout(spec)
    N, N_d = int(cu_q[-1]), int(cu_d[-1])
    vals = rng.integers(-3, 4, size=(N, V)).astype(np.float32) * 0.5       # 7 distinct values per row
    vals[2] = 1.25                                                           # an all-equal row
    bits = workloads.f32_to_bf16_bits(vals)
    toks = rng.integers(0, V, size=N_d).astype(np.int32)
    r = oracle.topk_rank_check(bits, toks, cu_q, cu_d, K=5, dtype="bf16")
    wide = workloads.bf16_bits_to_f32(bits)
    for i, s in enumerate(spec):
        for j in range(s):
            row = int(cu_q[i]) + j
            srt = np.sort(wide[row])
            want = V - int(np.searchsorted(srt, wide[row, toks[cu_d[i] + j]], side="right"))
            assert r["rank"][cu_d[i] + j] == want
    assert r["rank"][cu_d[0] + 2] == 0 and r["keep"][cu_q[0] + 3] == 1   # row 2 is request 0's third row
    r0 = oracle.topk_rank_check(bits, toks, cu_q, cu_d, K=0, dtype="bf16")
    for i, s in enumerate(spec):
        assert r0["keep"][cu_q[i]] == 1 and not r0["keep"][cu_q[i] + 1: cu_q[i + 1]].any()
    rV = oracle.topk_rank_check(bits, toks, cu_q, cu_d, K=V, dtype="bf16")
    assert rV["keep"].all()


def test_compacted_layout_and_invalid_tokens(oracle):
    """Fewer active rows than drafts + 1 (rows already pruned): only drafts that still have a row
    are ranked, the others report -1; an out-of-range draft id never passes."""
    rng = np.random.default_rng(5)
    V = 50
    spec = [4, 3, 0, 2]
    q_lens = [2, 4, 1, 0]                      # request 0 pruned to 2 rows, request 3 to none
    cu_q, cu_d = _layout(spec, q_lens)
    z = rng.standard_normal((int(cu_q[-1]), V)).astype(np.float32)
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    toks[cu_d[1] + 1] = V + 3
    r = oracle.topk_rank_check(z, toks, cu_q, cu_d, K=V)
    assert list(r["rank"][cu_d[0]:cu_d[1]] >= 0) == [True, True, False, False]
    assert (r["rank"][cu_d[3]:cu_d[4]] == -1).all()
    assert r["rank"][cu_d[1] + 1] == V and r["keep"][cu_q[1] + 2] == 0
    assert r["keep"][cu_q[0]] == 1 and r["keep"][cu_q[0] + 1] == 1 and len(r["keep"]) == int(cu_q[-1])


def test_check_prune_restore_composition(oracle):
    """Rank check -> suffix-closing compaction -> restore (Sec. 3.2 workflow figure: pruned tokens
    come back as rows with no values): a row has a value iff every draft up to its input passed."""
    rng = np.random.default_rng(21)
    V, K = 40, 6
    spec = [3, 3, 3]
    cu_q, cu_d = _layout(spec)
    N = int(cu_q[-1])
    z = np.stack([rng.permutation(V) for _ in range(N)]).astype(np.float32)
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    r = oracle.topk_rank_check(z, toks, cu_q, cu_d, K=K)
    passed = r["rank"] < K
    pc = oracle.prune_compact(r["keep"], cu_q, suffix_close=True, payload=z)
    restored, has = oracle.prune_restore(pc["payload"], pc["dst_row"])
    for i in range(3):
        alive = True
        assert has[cu_q[i]] == 1
        for j in range(3):
            alive = alive and bool(passed[cu_d[i] + j])
            assert has[cu_q[i] + j + 1] == (1 if alive else 0)
    assert np.array_equal(restored[has == 1], z[has == 1]) and not restored[has == 0].any()
