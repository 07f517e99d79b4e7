"""GPU parity: frontier (chunked) verification through the C ABI vs the chunked oracle and vs
one-shot verification (Sec. 3.3: chunking changes the schedule, not the acceptance behaviour)."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_attention, dev, fragile_draws

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


@pytest.mark.parametrize("cfg,s_c,dtype", [(5, 2, "bf16"), (5, 3, "bf16"), (4, 0, "bf16"), (5, 2, "f32")])
def test_chunked_matches_oracle_and_one_shot(fsr, oracle, cfg, s_c, dtype):
    announce(f"chunked cfg={cfg} s_c={s_c} dtype={dtype}")
    spec = [0, 1, 2, 3, 4, 5, 6, 7, 8, 2, 4, 6, 3, 8]
    ctx = [40, 33, 17, 64, 200, 31, 47, 16, 25, 50, 61, 19, 333, 90]
    kw = dict(H_q=8, H_kv=2, D=64) if dtype == "f32" else {}
    b = workloads.make_batch(cfg, rep=s_c, V=3000, spec_lens=spec, ctx_lens=ctx, dtype=dtype, **kw)
    chunks = workloads.chunk_plan(cfg, b.spec_lens, s_c=max(s_c, 1))
    ref = oracle.verify_chunked(b, chunks)
    one = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                             S_max=b.S_max)
    assert np.array_equal(ref["emitted"], one["emitted"])
    d = DeviceBatch(b)
    out = torch.full(d.q.shape, float("nan"), dtype=torch.float32, device="cuda")
    r = fsr.verify_chunked(q=d.q, k_caches=[d.k_cache], v_caches=[d.v_cache], block_tables=d.block_tables,
                           ctx_lens=d.ctx_lens, spec_lens=d.spec_lens, cu_q=d.cu_q, cu_d=d.cu_d, p_target=d.p_target,
                           p_draft=d.p_draft, draft_tokens=d.draft_tokens, u_accept=d.u_accept, u_sample=d.u_sample,
                           chunks=[dev(c) for c in chunks], scale=b.scale, S_total_max=b.S_max,
                           chunk_S_max=int(max(c.max() for c in chunks)), out=out)
    torch.cuda.synchronize()
    assert np.array_equal(r["accepted_len"].cpu().numpy(), ref["accepted_len"])
    assert np.array_equal(r["n_emitted"].cpu().numpy(), ref["n_emitted"])
    em = r["emitted"].cpu().numpy()
    frag = fragile_draws(b.u_sample, one["cdf_lo"], one["cdf_hi"])
    for i in np.where((em != ref["emitted"]).any(axis=1))[0]:
        assert frag[i], (i, em[i], ref["emitted"][i])
    o = out.cpu().numpy()
    done_ref = ~np.isnan(ref["out"][:, 0, 0])
    done_gpu = ~np.isnan(o[:, 0, 0])
    assert np.array_equal(done_ref, done_gpu)          # exactly the same rows were computed
    rows = np.where(done_ref)[0]
    check_attention(out[torch.from_numpy(rows).cuda()], ref["out"][rows], dtype, len(rows))
    assert sum(int(x.item()) for x in r["rows"]) == ref["rows_processed"]
