"""GPU parity: frontier (chunked) verification through the C ABI vs the chunked oracle and vs
one-shot verification (Sec. 3.3: chunking changes the schedule, not the acceptance behaviour)."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, chunked_case

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
    chunked_case(fsr, oracle, b, chunks, dtype)


def test_one_shot_step_with_survivor_mask_and_graph_replay(fsr, oracle):
    """attention -> accept -> survivor mask -> compaction captured in a HIP graph: every replay must
    reproduce the eager results (and those the oracle's)."""
    announce("one-shot step, eager vs graph replays")
    b = workloads.make_batch(2, rep=11, V=9000, ctx_lens=[300, 45, 513, 128, 1000, 77], spec_lens=[8, 3, 6, 0, 2, 5])
    d = DeviceBatch(b)
    i32 = dict(dtype=torch.int32, device="cuda")
    out = torch.empty_like(d.q)
    acc, nem, em = torch.empty(b.B, **i32), torch.empty(b.B, **i32), torch.empty((b.B, b.S_max + 1), **i32)
    keep = torch.empty(b.N, dtype=torch.uint8, device="cuda")
    pr = dict(new_cu_q=torch.empty(b.B + 1, **i32), new_q_lens=torch.empty(b.B, **i32), src_row=torch.empty(b.N, **i32),
              dst_row=torch.empty(b.N, **i32), n_active=torch.empty(1, **i32), active_ids=torch.empty(b.B, **i32))
    packed = torch.empty_like(out)
    ws_a = torch.empty(fsr.attn_workspace_bytes(B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P,
                                                max_pages=b.max_pages, n_pages=b.n_pages, dtype=torch.bfloat16,
                                                out_dtype=torch.bfloat16, max_q_len=b.S_max + 1), dtype=torch.uint8, device="cuda")
    ws_c = torch.empty(max(256, fsr.accept_workspace_bytes(B=b.B, V=b.V, S_max=b.S_max)), dtype=torch.uint8, device="cuda")

    def step():
        fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale,
                             out=out, workspace=ws_a, max_q_len=b.S_max + 1)
        fsr.spec_accept(d.p_target, d.p_draft, d.draft_tokens, d.u_accept, d.u_sample, d.cu_q, d.cu_d, S_max=b.S_max,
                        accepted_len=acc, n_emitted=nem, emitted=em, workspace=ws_c)
        fsr.survivor_mask(acc, d.cu_q, keep)
        fsr.prune_compact(keep, d.cu_q, payload=out, payload_out=packed, out=pr)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (out, acc, nem, em, keep, pr["new_cu_q"], pr["src_row"], pr["dst_row"], packed)]

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
        eager = snapshot()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        for rep in range(4):
            for t in (out, acc, nem, em, keep, pr["new_cu_q"], pr["src_row"], pr["dst_row"]):
                t.fill_(0) if t.dtype != torch.bfloat16 else t.zero_()  # the program's own eager work between replays
            torch.cuda.synchronize()
            g.replay()
            now = snapshot()
            n_new = int(eager[5][-1].item())
            for k, (a, e) in enumerate(zip(now, eager)):
                if k == 8:
                    a, e = a[:n_new], e[:n_new]
                assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                                   e.view(torch.int16) if e.dtype == torch.bfloat16 else e), (rep, k)
    ref = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, S_max=b.S_max)
    assert np.array_equal(eager[1].cpu().numpy(), ref["accepted_len"])
    keep_ref = np.concatenate([np.arange(s + 1) <= n for s, n in zip(b.spec_lens, ref["accepted_len"])]).astype(np.uint8)
    assert np.array_equal(eager[4].cpu().numpy(), keep_ref)
    pr_ref = oracle.prune_compact(keep_ref, b.cu_q)
    assert np.array_equal(eager[5].cpu().numpy(), pr_ref["new_cu_q"])
    assert np.array_equal(eager[6].cpu().numpy(), pr_ref["src_row"])
