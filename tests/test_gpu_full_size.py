"""GPU parity at the full sizes of workload configurations 3, 4 and 5 (the high-load batch, the
70B-shaped share with two chunks, the chunked frontier): every output of the path is compared with
the oracle on the whole batch, element by element, in the launch configuration a serving step
would use (workspaces sized by the library, bf16 caches, one call per chunk)."""
import time

import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_accept, check_attention, chunked_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def _oracle_attention(oracle, b):
    return oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                   H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)


def _one_shot(fsr, oracle, b, out_dtype):
    """attention (twice: same bits) -> accept -> survivor mask -> compaction with the attention output
    as payload, all against the oracle."""
    d = DeviceBatch(b)
    lse = torch.zeros((b.N, b.H_q), dtype=torch.float32, device="cuda")
    out, lse = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                    scale=b.scale, out_dtype=out_dtype, lse=lse, max_q_len=b.S_max + 1)
    again, _ = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                    scale=b.scale, out_dtype=out_dtype, max_q_len=b.S_max + 1)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16 if out_dtype == torch.bfloat16 else torch.int32),
                       again.view(torch.int16 if out_dtype == torch.bfloat16 else torch.int32))
    o_ref, lse_ref = _oracle_attention(oracle, b)
    err = check_attention(out, o_ref, b.dtype, b.N)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=3e-5, atol=3e-5)

    acc, nem, em = fsr.spec_accept(d.p_target, d.p_draft, d.draft_tokens, d.u_accept, d.u_sample, d.cu_q, d.cu_d,
                                   S_max=b.S_max)
    torch.cuda.synchronize()
    ref = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, S_max=b.S_max)
    n_frag, n_diff = check_accept((acc, nem, em), ref, b.u_sample)

    keep = torch.empty(b.N, dtype=torch.uint8, device="cuda")
    fsr.survivor_mask(acc, d.cu_q, keep)
    pr = fsr.prune_compact(keep, d.cu_q, suffix_close=True, payload=out)
    torch.cuda.synchronize()
    keep_ref = np.concatenate([np.arange(s + 1) <= n for s, n in zip(b.spec_lens, ref["accepted_len"])]).astype(np.uint8)
    assert np.array_equal(keep.cpu().numpy(), keep_ref)
    pr_ref = oracle.prune_compact(keep_ref, b.cu_q, suffix_close=True)
    for name in ("new_cu_q", "new_q_lens", "dst_row"):
        assert np.array_equal(pr[name].cpu().numpy(), pr_ref[name]), name
    n_new = int(pr_ref["new_cu_q"][-1])
    assert np.array_equal(pr["src_row"].cpu().numpy()[:n_new], pr_ref["src_row"][:n_new])
    packed = pr["payload"][:n_new]
    src = torch.from_numpy(pr_ref["src_row"][:n_new].astype(np.int64)).cuda()
    assert torch.equal(packed.view(torch.int16), out[src].view(torch.int16))
    return dict(err=err, fragile=n_frag, token_diffs=n_diff, accepted=int(ref["accepted_len"].sum()), kept_rows=n_new)


def test_config3_high_load_one_shot(fsr, oracle):
    announce("full size cfg3: B=128 one-shot step")
    t0 = time.time()
    b = workloads.make_batch(3)
    print(f"cfg3: N={b.N} rows, {b.kv_tokens()} cached tokens, V={b.V}; generated in {time.time() - t0:.1f} s", flush=True)
    r = _one_shot(fsr, oracle, b, torch.bfloat16)
    print(f"cfg3 one-shot: {r}", flush=True)


def test_config4_one_shot_wide_suffixes(fsr, oracle):
    """64 query heads over 8 KV heads and up to 11 rows per request: up to 88 rows share a KV head."""
    announce("full size cfg4: B=256, 64/8 heads, one-shot attention")
    t0 = time.time()
    b = workloads.make_batch(4, with_probs=False)
    print(f"cfg4: N={b.N} rows, {b.kv_tokens()} cached tokens; generated in {time.time() - t0:.1f} s", flush=True)
    d = DeviceBatch(b, probs=False)
    out, _ = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                  scale=b.scale, out_dtype=torch.float32, max_q_len=b.S_max + 1)
    torch.cuda.synchronize()
    o_ref, _ = _oracle_attention(oracle, b)
    err = check_attention(out, o_ref, b.dtype, b.N)
    print(f"cfg4 one-shot attention max rel err {err:.3e}", flush=True)


@pytest.mark.parametrize("cfg", [4, 5])
def test_chunked_configs_full_size(fsr, oracle, cfg):
    announce(f"full size cfg{cfg}: chunked verification with pruning between chunks")
    t0 = time.time()
    b = workloads.make_batch(cfg)
    chunks = workloads.chunk_plan(cfg, b.spec_lens, s_c=2)
    print(f"cfg{cfg}: B={b.B}, N={b.N} rows, {b.kv_tokens()} cached tokens, V={b.V}, {len(chunks)} chunks; "
          f"generated in {time.time() - t0:.1f} s", flush=True)
    r = chunked_case(fsr, oracle, b, chunks, b.dtype)
    print(f"cfg{cfg} chunked: {r}", flush=True)
    assert r["rows"] < r["rows_total"]  # rejections in early chunks spared the rows behind them
