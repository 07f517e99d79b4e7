"""Pins of the attention oracle (Sec. 2.1 verification pass) against things other than itself."""
import numpy as np
import pytest
from scipy.special import logsumexp

import workloads
from workloads import bf16_bits_to_f32


def _widen(b, x):
    return bf16_bits_to_f32(x).astype(np.float64) if b.dtype == "bf16" else x.astype(np.float64)


def unpage(b, i, cache):
    """Dense [ctx+q, H_kv, D] view of request i's cache, through the block table."""
    L = int(b.ctx_lens[i] + b.spec_lens[i] + 1)
    rows = []
    for t in range(L):
        pg = b.block_tables[i, t // b.P]
        rows.append(_widen(b, cache[pg, :, t % b.P, :]))
    return np.stack(rows)  # [L, H_kv, D]


def dense_attention(b):
    """Brute force: full masked score matrix per request and head, numpy softmax."""
    G = b.H_q // b.H_kv
    out = np.zeros((b.N, b.H_q, b.D))
    lse = np.zeros((b.N, b.H_q))
    for i in range(b.B):
        K, Vv = unpage(b, i, b.k_cache), unpage(b, i, b.v_cache)
        qi = _widen(b, b.q[b.cu_q[i]: b.cu_q[i + 1]])  # [q, H_q, D]
        ql, L, c = qi.shape[0], K.shape[0], int(b.ctx_lens[i])
        for h in range(b.H_q):
            S = b.scale * qi[:, h, :] @ K[:, h // G, :].T  # [q, L]
            mask = np.arange(L)[None, :] <= (c + np.arange(ql))[:, None]
            S = np.where(mask, S, -np.inf)
            W = np.exp(S - S.max(axis=1, keepdims=True))
            out[b.cu_q[i]: b.cu_q[i + 1], h] = (W / W.sum(axis=1, keepdims=True)) @ Vv[:, h // G, :]
            lse[b.cu_q[i]: b.cu_q[i + 1], h] = logsumexp(S, axis=1)
    return out, lse


def run(oracle, b, **kw):
    return oracle.verify_attention(kw.get("q", b.q), kw.get("k", b.k_cache), kw.get("v", b.v_cache),
                                   kw.get("bt", b.block_tables), kw.get("ctx", b.ctx_lens), kw.get("cu", b.cu_q),
                                   H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dense_bruteforce_config1(oracle, dtype):
    b = workloads.make_batch(1, with_probs=False, dtype=dtype)
    o, lse = run(oracle, b)
    ro, rlse = dense_attention(b)
    np.testing.assert_allclose(o, ro, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lse, rlse, rtol=1e-12, atol=1e-12)


def test_spec_len_zero_is_plain_decode(oracle):
    b = workloads.make_batch(1, with_probs=False, spec_lens=[0, 0, 0, 0])
    o, _ = run(oracle, b)
    G = b.H_q // b.H_kv
    for i in range(b.B):
        K, Vv = unpage(b, i, b.k_cache), unpage(b, i, b.v_cache)
        for h in range(b.H_q):
            s = b.scale * K[:, h // G, :] @ b.q[i, h].astype(np.float64)
            w = np.exp(s - s.max())
            np.testing.assert_allclose(o[i, h], (w / w.sum()) @ Vv[:, h // G, :], rtol=1e-11, atol=1e-13)


def test_causality_row_j_equals_decode_at_ctx_plus_j(oracle):
    b = workloads.make_batch(1, with_probs=False)
    o, lse = run(oracle, b)
    for i in range(b.B):
        for j in range(int(b.spec_lens[i]) + 1):
            r = int(b.cu_q[i]) + j
            o1, l1 = oracle.verify_attention(b.q[r: r + 1], b.k_cache, b.v_cache, b.block_tables[i: i + 1],
                                             np.array([b.ctx_lens[i] + j], np.int32), np.array([0, 1], np.int32),
                                             H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
            assert np.array_equal(o1[0], o[r]) and np.array_equal(l1[0], lse[r])


def test_page_permutation_invariance_bitwise(oracle):
    b = workloads.make_batch(1, with_probs=False)
    o, _ = run(oracle, b)
    rng = np.random.default_rng(7)
    perm = rng.permutation(b.n_pages)           # new physical location of old page p is perm[p]
    k2 = np.empty_like(b.k_cache)
    v2 = np.empty_like(b.v_cache)
    k2[perm] = b.k_cache
    v2[perm] = b.v_cache
    bt2 = np.where(b.block_tables >= 0, perm[np.maximum(b.block_tables, 0)], -1).astype(np.int32)
    o2, _ = run(oracle, b, k=k2, v=v2, bt=bt2)
    assert np.array_equal(o, o2)


def test_closed_forms(oracle):
    b = workloads.make_batch(1, with_probs=False)
    ones = np.ones_like(b.v_cache)
    o, _ = run(oracle, b, v=ones)
    np.testing.assert_allclose(o, 1.0, rtol=1e-13)
    zeros = np.zeros_like(b.k_cache)
    o, lse = run(oracle, b, k=zeros)
    G = b.H_q // b.H_kv
    for i in range(b.B):
        Vv = unpage(b, i, b.v_cache)
        for j in range(int(b.spec_lens[i]) + 1):
            L = int(b.ctx_lens[i]) + j + 1
            mean = Vv[:L].mean(axis=0)  # [H_kv, D]
            for h in range(b.H_q):
                np.testing.assert_allclose(o[b.cu_q[i] + j, h], mean[h // G], rtol=1e-10, atol=1e-13)
                np.testing.assert_allclose(lse[b.cu_q[i] + j, h], np.log(L), rtol=1e-13)


def test_gqa_group_shares_kv_head(oracle):
    b = workloads.make_batch(1, with_probs=False)
    G = b.H_q // b.H_kv
    q = b.q.copy()
    for g in range(b.H_kv):
        q[:, g * G: (g + 1) * G, :] = q[:, g * G: g * G + 1, :]
    o, _ = run(oracle, b, q=q)
    for g in range(b.H_kv):
        for k in range(1, G):
            assert np.array_equal(o[:, g * G], o[:, g * G + k])
    # and different KV heads do differ
    assert not np.array_equal(o[:, 0], o[:, G])


def test_scale_matters_and_empty_request(oracle):
    b = workloads.make_batch(1, with_probs=False)
    o1, _ = run(oracle, b)
    o2, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                    H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=2 * b.scale)
    assert np.abs(o1 - o2).max() > 1e-3
    # a request with zero rows is legal and leaves the others untouched
    cu = np.array([0, 1, 1, 4, 4 + 4], np.int32)  # request 1 has no rows; rows re-dealt: 1,0,3,4
    ctx = b.ctx_lens.copy()
    o3, _ = run(oracle, b, q=b.q[:8], cu=cu, ctx=ctx)
    o4, _ = oracle.verify_attention(b.q[1:4], b.k_cache, b.v_cache, b.block_tables[2:3], ctx[2:3],
                                    np.array([0, 3], np.int32), H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P,
                                    dtype=b.dtype, scale=b.scale)
    assert np.array_equal(o3[1:4], o4)
