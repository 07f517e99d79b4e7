"""GPU parity on seeded random shapes: head counts, batch sizes, contexts around page and tile edges, suffixes from
none to 40 positions (one-team and two-team row groups), small grids (cut items), both cache layouts, both output types,
known and unknown row bound; the planned and the self-scheduling call must agree bit for bit and with the oracle."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_attention

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def same_bits(x, y):
    bits = torch.int16 if x.dtype == torch.bfloat16 else torch.int32
    return torch.equal(x.view(bits), y.view(bits))


@pytest.mark.parametrize("case", range(24))
def test_random_shapes(fsr, oracle, case):
    rng = np.random.default_rng(9000 + case)
    H_q, H_kv = [(32, 8), (64, 8), (16, 16), (16, 1), (48, 16), (8, 2)][rng.integers(0, 6)]
    B = int(rng.integers(1, 30))
    ctx = [int(x) for x in rng.choice([0, 1, 15, 16, 17, 31, 32, 33, 100, 500, 1000, 2500], size=B) + rng.integers(0, 40, size=B)]
    smax = int(rng.choice([0, 3, 8, 20, 40]))
    spec = [int(x) for x in rng.integers(0, smax + 1, size=B)]
    kw = {}
    mw = int(rng.choice([0, 0, 5, 64]))
    if mw:
        kw["max_workgroups"] = mw
    token_major = bool(rng.integers(0, 2))
    out_dtype = [torch.float32, torch.bfloat16][rng.integers(0, 2)]
    mq = int(rng.choice([0, max(spec) + 1]))
    announce(f"fuzz case {case}: heads {(H_q, H_kv)} B={B} spec<= {smax} max_workgroups={mw} token_major={token_major} "
             f"out={out_dtype} max_q_len={mq}")
    b = workloads.make_batch(2, rep=1000 + case, with_probs=False, H_q=H_q, H_kv=H_kv, ctx_lens=ctx, spec_lens=spec)
    d = DeviceBatch(b, probs=False)
    if token_major:
        d.k_cache = d.k_cache.transpose(1, 2).contiguous()
        d.v_cache = d.v_cache.transpose(1, 2).contiguous()
        kw["kv_layout"] = 1
    o_ref, lse_ref = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv,
                                             D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    outs = []
    for planned in (False, True):
        out = torch.full((b.N, b.H_q, b.D), float("nan"), dtype=out_dtype, device="cuda")
        lse = torch.full((b.N, b.H_q), float("nan"), dtype=torch.float32, device="cuda")
        plan = fsr.attn_plan(d.q, d.k_cache, d.block_tables, d.ctx_lens, d.cu_q, scale=b.scale, out_dtype=out_dtype, max_q_len=mq,
                             **kw) if planned else None
        fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale, out=out, lse=lse,
                             max_q_len=mq, plan=plan, **kw)
        torch.cuda.synchronize()
        outs.append((out, lse))
    assert same_bits(outs[0][0], outs[1][0]) and same_bits(outs[0][1], outs[1][1])
    check_attention(outs[1][0], o_ref, "bf16", b.N)
    np.testing.assert_allclose(outs[1][1].cpu().numpy(), lse_ref, rtol=3e-5, atol=3e-5)
