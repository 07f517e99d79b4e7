"""GPU parity: fsr_kv_append vs the oracle, bit-exact on the whole caches, and the append ->
attention sequence of one forward pass."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_attention, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


@pytest.mark.parametrize("cfg,kw", [(1, {}), (2, dict(ctx_lens=[0, 5, 16, 31, 100, 1000], spec_lens=[3, 0, 7, 1, 4, 8]))])
def test_append_matches_oracle_bit_for_bit(fsr, oracle, cfg, kw):
    announce(f"kv_append cfg={cfg}")
    b = workloads.make_batch(cfg, rep=41, with_probs=False, **kw)
    bf = b.dtype == "bf16"
    rng = np.random.default_rng(3)
    if bf:
        k_new = workloads.f32_to_bf16_bits(rng.standard_normal((b.N + 2, b.H_kv, b.D)).astype(np.float32))
        v_new = workloads.f32_to_bf16_bits(rng.standard_normal((b.N + 2, b.H_kv, b.D)).astype(np.float32))
    else:
        k_new = rng.standard_normal((b.N + 2, b.H_kv, b.D)).astype(np.float32)   # two slack rows
        v_new = rng.standard_normal((b.N + 2, b.H_kv, b.D)).astype(np.float32)
    d = DeviceBatch(b, probs=False)
    kc, vc = d.k_cache.clone(), d.v_cache.clone()
    fsr.kv_append(dev(k_new, bf), dev(v_new, bf), kc, vc, d.block_tables, d.ctx_lens, d.cu_q)
    torch.cuda.synchronize()
    kr, vr = oracle.kv_append(k_new[:b.N], v_new[:b.N], b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, P=b.P)
    assert np.array_equal(_bits(kc).cpu().numpy(), kr.view(np.int16 if bf else np.int32))
    assert np.array_equal(_bits(vc).cpu().numpy(), vr.view(np.int16 if bf else np.int32))
    assert not np.array_equal(kr, b.k_cache)


def test_append_then_attention_is_one_forward_pass(fsr, oracle):
    """The suffix rows' K/V are taken out of the cache (their slots filled with junk), appended by
    the library, and attention over the result matches the oracle's on the original cache."""
    announce("kv_append -> verify_attention")
    b = workloads.make_batch(2, rep=43, with_probs=False, ctx_lens=[300, 45, 513, 0, 1000], spec_lens=[8, 3, 6, 2, 5])
    k_new = np.zeros((b.N, b.H_kv, b.D), np.uint16)
    v_new = np.zeros_like(k_new)
    kj, vj = b.k_cache.copy(), b.v_cache.copy()
    for i in range(b.B):
        for r in range(int(b.cu_q[i]), int(b.cu_q[i + 1])):
            t = int(b.ctx_lens[i]) + r - int(b.cu_q[i])
            pg, sl = b.block_tables[i, t // b.P], t % b.P
            k_new[r], v_new[r] = b.k_cache[pg, :, sl, :], b.v_cache[pg, :, sl, :]
            kj[pg, :, sl, :] = 0x7F80          # +inf in bf16: attention over a slot that was not refilled blows up
            vj[pg, :, sl, :] = 0x7F80
    d = DeviceBatch(b, probs=False)
    kc, vc = dev(kj, True), dev(vj, True)
    fsr.kv_append(dev(k_new, True), dev(v_new, True), kc, vc, d.block_tables, d.ctx_lens, d.cu_q)
    out, _ = fsr.verify_attention(d.q, kc, vc, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale,
                                  out_dtype=torch.float32, max_q_len=b.S_max + 1)
    torch.cuda.synchronize()
    o_ref, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                       H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    check_attention(out, o_ref, b.dtype, b.N)


def test_positions_beyond_the_block_table_and_bad_page_ids_are_skipped(fsr, oracle):
    announce("kv_append with truncated block table and an out-of-pool page id")
    b = workloads.make_batch(1, rep=6, with_probs=False, ctx_lens=[10, 31, 3], spec_lens=[2, 1, 1])
    bt = b.block_tables[:, :2].copy()
    bt[2, 0] = b.n_pages + 5                                   # request 2 points outside the pool
    k_new = np.full((b.N, b.H_kv, b.D), 3.0, np.float32)
    d = DeviceBatch(b, probs=False)
    kc, vc = d.k_cache.clone(), d.v_cache.clone()
    fsr.kv_append(dev(k_new), dev(k_new), kc, vc, dev(bt), d.ctx_lens, d.cu_q)
    torch.cuda.synchronize()
    changed = (kc.cpu().numpy() != b.k_cache).any(axis=(1, 3))
    assert changed.sum() == 3 + 1
