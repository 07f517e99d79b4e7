"""Seeded random shapes within the documented limits, against the oracle: every combination of head grouping,
context lengths around page and tile boundaries, suffix lengths, cache layout and storage, output type, row-bound
hint and grid size that the fixed cases do not spell out."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import announce, check_accept, check_attention, dev

pytestmark = pytest.mark.gpu

HEADS = [(32, 8), (8, 8), (16, 8), (64, 8), (16, 1), (8, 2), (24, 8), (128, 8)]
EDGES = [0, 15, 16, 17, 31, 32, 33, 63, 64, 127, 128, 129, 255, 256, 511, 512, 513]


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_attention_random_cases(fsr, oracle, seed):
    rng = np.random.default_rng(seed)
    for case in range(12):
        B = int(rng.integers(1, 13))
        H_q, H_kv = HEADS[int(rng.integers(0, len(HEADS)))]
        kind = int(rng.integers(0, 4))
        ctx = (rng.integers(0, 80, size=B) if kind == 0 else rng.integers(0, 1500, size=B) if kind == 1
               else rng.choice(EDGES, size=B) if kind == 2 else rng.integers(1000, 3000, size=B))
        smax = int(rng.choice([0, 1, 3, 8, 10]))
        spec = rng.integers(0, smax + 1, size=B)
        kv8, tm = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        out_dtype = [torch.float32, torch.bfloat16][int(rng.integers(0, 2))]
        b = workloads.make_batch(2, rep=1000 * seed + case, with_probs=False, H_q=H_q, H_kv=H_kv,
                                 ctx_lens=[int(c) for c in ctx], spec_lens=[int(s) for s in spec])
        mq, nwg = int(rng.choice([0, b.S_max + 1])), int(rng.choice([0, 0, 1, 3, 17, 255]))
        announce(f"random attention seed={seed} case={case} B={B} heads={H_q}/{H_kv} ctx={[int(c) for c in ctx]} "
                 f"spec={[int(s) for s in spec]} kv8={kv8} token_major={tm} out={out_dtype} max_q_len={mq} workgroups={nwg}")
        lay = fsr.binding.KV_TOKEN_MAJOR if tm else fsr.binding.KV_HEAD_MAJOR
        to_lay = (lambda c: np.ascontiguousarray(np.swapaxes(c, 1, 2))) if tm else (lambda c: c)
        lse = torch.empty(b.N, H_q, dtype=torch.float32, device="cuda")
        if kv8:
            ks = rng.uniform(0.01, 0.05, H_kv).astype(np.float32)
            vs = rng.uniform(0.01, 0.05, H_kv).astype(np.float32)
            k8 = workloads.f32_to_e4m3_bits(workloads.bf16_bits_to_f32(b.k_cache) / ks.reshape(1, -1, 1, 1))
            v8 = workloads.f32_to_e4m3_bits(workloads.bf16_bits_to_f32(b.v_cache) / vs.reshape(1, -1, 1, 1))
            o_ref, lse_ref = oracle.verify_attention_kv8(b.q, k8, v8, ks, vs, b.block_tables, b.ctx_lens, b.cu_q, H_q=H_q,
                                                         H_kv=H_kv, D=b.D, P=b.P, scale=b.scale)
            out, _ = fsr.verify_attention_kv8(dev(b.q, True), dev(to_lay(k8)), dev(to_lay(v8)), dev(ks), dev(vs), dev(b.block_tables),
                                              dev(b.ctx_lens), dev(b.cu_q), scale=b.scale, out_dtype=out_dtype, lse=lse, max_q_len=mq,
                                              max_workgroups=nwg, kv_layout=lay)
        else:
            o_ref, lse_ref = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=H_q,
                                                     H_kv=H_kv, D=b.D, P=b.P, dtype="bf16", scale=b.scale)
            out, _ = fsr.verify_attention(dev(b.q, True), dev(to_lay(b.k_cache), True), dev(to_lay(b.v_cache), True),
                                          dev(b.block_tables), dev(b.ctx_lens), dev(b.spec_lens), dev(b.cu_q), scale=b.scale,
                                          out_dtype=out_dtype, lse=lse, max_q_len=mq, max_workgroups=nwg, kv_layout=lay)
        torch.cuda.synchronize()
        check_attention(out, o_ref, "bf16", b.N)
        np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=3e-5, atol=3e-5)


@pytest.mark.parametrize("seed", [0, 1])
def test_accept_random_cases(fsr, oracle, seed):
    rng = np.random.default_rng(100 + seed)
    for case in range(12):
        B = int(rng.integers(1, 40))
        V = int(rng.choice([17, 1000, 1001, 4096, 4097, 8191, 32000, 50257]))
        smax = int(rng.choice([1, 4, 8]))
        spec = rng.integers(0, smax + 1, size=B)
        mode = int(rng.integers(0, 3))
        bf = bool(rng.integers(0, 2)) and mode != 2
        draft_mode = ["independent", "noise", "equal"][int(rng.integers(0, 3))]
        T = float(rng.choice([1.0, 0.7, 1.3]))
        announce(f"random accept seed={seed} case={case} B={B} V={V} spec={[int(s) for s in spec]} mode={mode} bf16={bf} "
                 f"draft={draft_mode} T={T}")
        b = workloads.make_batch(2, rep=5000 + 100 * seed + case, with_kv=False, V=V, B=B, spec_lens=[int(s) for s in spec],
                                 ctx_lens=[10] * B, keep_logits=True, draft_mode=draft_mode)
        src_t, src_d = (b.p_target, b.p_draft) if mode == 0 else (b.z_target, b.z_draft)
        kw = dict(S_max=b.S_max, mode=mode, temperature=T)
        if bf:
            src_t, src_d = workloads.f32_to_bf16_bits(src_t), workloads.f32_to_bf16_bits(src_d)
            kw_ref = dict(kw, dtype="bf16")
        else:
            kw_ref = kw
        ref = oracle.spec_accept(src_t, src_d, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, **kw_ref)
        gpu = fsr.spec_accept(dev(src_t, bf), dev(src_d, bf), dev(b.draft_tokens), dev(b.u_accept), dev(b.u_sample), dev(b.cu_q),
                              dev(b.cu_d), **kw)
        torch.cuda.synchronize()
        if mode == 2:
            assert np.array_equal(gpu[0].cpu().numpy(), ref["accepted_len"])
            assert np.array_equal(gpu[1].cpu().numpy(), ref["n_emitted"])
            assert np.array_equal(gpu[2].cpu().numpy(), ref["emitted"])
        else:
            frag, mism = check_accept(gpu, ref, b.u_sample)
            assert mism == 0, (frag, mism)
