"""Pins of the oracle's cache append against things other than itself: un-paging the result with
numpy fancy indexing gives [old context | new rows] per request, every other slot of the pool keeps
its bits, and attention over an appended cache equals attention over a cache that held the rows
from the start."""
import numpy as np

import workloads


def _unpage(cache, bt_row, n_tok, P):
    """Tokens 0..n_tok-1 of one request as [n_tok, H_kv, D], by numpy indexing."""
    t = np.arange(n_tok)
    return cache[bt_row[t // P], :, t % P, :]


def test_unpaged_result_is_context_then_new_rows_and_rest_untouched(oracle):
    b = workloads.make_batch(2, rep=31, with_probs=False, ctx_lens=[0, 5, 16, 31, 100], spec_lens=[3, 0, 7, 1, 4])
    rng = np.random.default_rng(1)
    k_new = rng.integers(0, 1 << 16, size=(b.N, b.H_kv, b.D)).astype(np.uint16)
    v_new = rng.integers(0, 1 << 16, size=(b.N, b.H_kv, b.D)).astype(np.uint16)
    kc, vc = oracle.kv_append(k_new, v_new, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, P=b.P)
    touched = np.zeros(b.k_cache.shape[:1] + b.k_cache.shape[2:3], bool)       # [page, slot]
    for i in range(b.B):
        c, q = int(b.ctx_lens[i]), int(b.cu_q[i + 1] - b.cu_q[i])
        for new, old, rows in ((kc, b.k_cache, k_new), (vc, b.v_cache, v_new)):
            got = _unpage(new, b.block_tables[i], c + q, b.P)
            assert np.array_equal(got[:c], _unpage(old, b.block_tables[i], c, b.P))
            assert np.array_equal(got[c:], rows[b.cu_q[i]:b.cu_q[i + 1]])
        t = np.arange(c, c + q)
        touched[b.block_tables[i][t // b.P], t % b.P] = True
    for new, old in ((kc, b.k_cache), (vc, b.v_cache)):
        same = (new == old).all(axis=(1, 3))                                   # [page, slot]
        assert same[~touched].all()
    assert touched.sum() == b.N


def test_attention_after_append_equals_attention_on_prefilled_cache(oracle):
    b = workloads.make_batch(1, rep=4, with_probs=False)
    ref, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                     H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    # pull the suffix rows out of the cache, overwrite their slots with junk, append them back
    k_new = np.zeros((b.N, b.H_kv, b.D), b.k_cache.dtype)
    v_new = np.zeros_like(k_new)
    kj, vj = b.k_cache.copy(), b.v_cache.copy()
    for i in range(b.B):
        for r in range(int(b.cu_q[i]), int(b.cu_q[i + 1])):
            t = int(b.ctx_lens[i]) + r - int(b.cu_q[i])
            pg, sl = b.block_tables[i, t // b.P], t % b.P
            k_new[r], v_new[r] = b.k_cache[pg, :, sl, :], b.v_cache[pg, :, sl, :]
            kj[pg, :, sl, :] = 77.0
            vj[pg, :, sl, :] = -55.0
    kc, vc = oracle.kv_append(k_new, v_new, kj, vj, b.block_tables, b.ctx_lens, b.cu_q, P=b.P)
    assert np.array_equal(kc, b.k_cache) and np.array_equal(vc, b.v_cache)
    out, _ = oracle.verify_attention(b.q, kc, vc, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv, D=b.D,
                                     P=b.P, dtype=b.dtype, scale=b.scale)
    assert np.array_equal(out, ref)


def test_positions_beyond_the_block_table_are_dropped(oracle):
    b = workloads.make_batch(1, rep=6, with_probs=False, ctx_lens=[10, 31], spec_lens=[2, 1])
    bt = b.block_tables[:, :2].copy()                                           # room for 32 tokens only
    k_new = np.full((b.N, b.H_kv, b.D), 3.0, np.float32)
    kc, vc = oracle.kv_append(k_new, k_new, b.k_cache, b.v_cache, bt, b.ctx_lens, b.cu_q, P=b.P)
    changed = (kc != b.k_cache).any(axis=(1, 3))
    assert changed.sum() == 3 + 1                                               # request 1: position 31 fits, 32 does not
