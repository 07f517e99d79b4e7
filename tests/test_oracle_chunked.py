"""Frontier (chunked) verification: Sec. 3.3 says chunking changes the schedule, not the
acceptance behaviour -- so the chunked oracle must emit exactly the one-shot tokens."""
import os

import numpy as np
import pytest

import workloads


def one_shot(oracle, b, mode=0):
    src_t = b.z_target if mode else b.p_target
    src_d = b.z_draft if mode else b.p_draft
    return oracle.spec_accept(src_t, src_d, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                              S_max=b.S_max, mode=mode)


@pytest.mark.parametrize("s_c", [1, 2, 3])
@pytest.mark.parametrize("draft_mode", ["noise", "independent", "equal"])
def test_chunked_equals_one_shot(oracle, s_c, draft_mode):
    b = workloads.make_batch(1, rep=s_c, V=300, B=12, spec_lens=[0, 1, 2, 3, 4, 5, 6, 7, 8, 2, 4, 6],
                             ctx_lens=[40, 33, 17, 64, 20, 31, 47, 16, 25, 50, 61, 19], draft_mode=draft_mode)
    ref = one_shot(oracle, b)
    ref_o, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                       H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    chunks = workloads.chunk_plan(5, b.spec_lens, s_c=s_c)
    r = oracle.verify_chunked(b, chunks)
    assert np.array_equal(r["accepted_len"], ref["accepted_len"])
    assert np.array_equal(r["n_emitted"], ref["n_emitted"])
    assert np.array_equal(r["emitted"], ref["emitted"])
    done = ~np.isnan(r["out"][:, 0, 0])
    assert np.array_equal(r["out"][done], ref_o[done])          # chunk rows == one-shot rows, bitwise
    # rows that were computed: everything up to and including the chunk holding the rejection
    any_early_reject = False
    for i in range(b.B):
        s, n = int(b.spec_lens[i]), int(ref["accepted_len"][i])
        cum = np.cumsum([c[i] for c in chunks])
        last_chunk = int(np.searchsorted(cum, min(n + 1, s), side="left")) if s else 0
        upto = int(cum[last_chunk]) if s else 0
        rows = upto + (1 if upto == s else 0)
        assert done[b.cu_q[i]: b.cu_q[i] + rows].all() and not done[b.cu_q[i] + rows: b.cu_q[i + 1]].any(), i
        any_early_reject |= rows < s + 1
    if draft_mode == "equal":
        assert r["rows_processed"] == b.N
    else:
        assert any_early_reject and r["rows_processed"] < b.N


def test_two_chunk_plan_config4_shape(oracle):
    b = workloads.make_batch(4, B=24, V=200, with_kv=False)
    chunks = workloads.chunk_plan(4, b.spec_lens)
    assert len(chunks) == 2 and np.array_equal(chunks[0] + chunks[1], b.spec_lens)
    assert np.array_equal(chunks[0], (b.spec_lens + 1) // 2)
    r = oracle.verify_chunked(b, chunks, with_attention=False)
    ref = one_shot(oracle, b)
    assert np.array_equal(r["emitted"], ref["emitted"]) and np.array_equal(r["n_emitted"], ref["n_emitted"])


def test_pipeline_overlap_figure_shape(oracle):
    """Fig. 6 shape: speculative length 4 verified as two frontiers of 2."""
    path = os.path.join(os.path.dirname(__file__), "golden", "figure_shapes.txt")
    row = [l.split("|") for l in open(path) if l.startswith("pipeline_overlap")][0]
    spec, s_c = [int(x) for x in row[1].split(",")], int(row[2])
    hits = set()
    for rep in range(12):
        b = workloads.make_batch(1, rep=rep, V=50, spec_lens=spec, ctx_lens=[30], with_kv=False)
        chunks = workloads.chunk_plan(5, b.spec_lens, s_c=s_c)
        assert [int(c[0]) for c in chunks] == [2, 2]
        r = oracle.verify_chunked(b, chunks, with_attention=False)
        ref = one_shot(oracle, b)
        assert np.array_equal(r["emitted"], ref["emitted"])
        n = int(ref["accepted_len"][0])
        assert r["rows_processed"] == (2 if n < 2 else 5)
        hits.add(n < 2)
    assert hits == {True, False}


def test_chunked_logits_mode(oracle):
    b = workloads.make_batch(1, rep=9, V=200, B=6, spec_lens=[3, 4, 0, 2, 5, 1], ctx_lens=[20] * 6, with_kv=False,
                             keep_logits=True)
    ref = one_shot(oracle, b, mode=1)
    r = oracle.verify_chunked(b, workloads.chunk_plan(5, b.spec_lens, s_c=2), with_attention=False, mode=1)
    assert np.array_equal(r["emitted"], ref["emitted"])
