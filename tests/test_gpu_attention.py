"""GPU parity: verify_attention vs the oracle, element by element.
Tolerance (the benchmark spec): 1e-5 relative for fp32 inputs, 2e-3 for bf16 inputs, relative to
max(|o_ref|, rms of the (row, head) vector)."""
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


def ref_of(oracle, b, **kw):
    return oracle.verify_attention(kw.get("q", b.q), kw.get("k", b.k_cache), kw.get("v", b.v_cache), b.block_tables,
                                   kw.get("ctx", b.ctx_lens), kw.get("cu", b.cu_q), H_q=b.H_q, H_kv=b.H_kv, D=b.D,
                                   P=b.P, dtype=b.dtype, scale=b.scale)


def run_gpu(fsr, b, d, out_dtype, max_q_len=None, want_lse=True):
    lse = torch.zeros((b.N, b.H_q), dtype=torch.float32, device="cuda") if want_lse else None
    mq = b.S_max + 1 if max_q_len is None else max_q_len
    out, lse = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                    scale=b.scale, out_dtype=out_dtype, lse=lse, max_q_len=mq)
    torch.cuda.synchronize()
    return out, lse


def test_config1_fp32(fsr, oracle):
    announce("attention config1 fp32 (generic path)")
    b = workloads.make_batch(1, with_probs=False)
    d = DeviceBatch(b, probs=False)
    o_ref, lse_ref = ref_of(oracle, b)
    out, lse = run_gpu(fsr, b, d, torch.float32)
    err = check_attention(out, o_ref, "f32", b.N)
    print(f"config1 fp32 max rel err {err:.3e}")
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("heads", [(32, 8), (8, 8), (16, 8), (64, 8), (16, 1)])
def test_bf16_fast_path_small(fsr, oracle, heads, out_dtype):
    H_q, H_kv = heads
    announce(f"attention bf16 fast small heads={heads} out={out_dtype}")
    ctx = [0, 1, 15, 16, 31, 33, 100, 257, 511, 640, 700, 1029]
    spec = [3, 0, 8, 1, 2, 7, 4, 10, 5, 6, 0, 9]
    b = workloads.make_batch(2, rep=H_q, with_probs=False, H_q=H_q, H_kv=H_kv, ctx_lens=ctx, spec_lens=spec)
    d = DeviceBatch(b, probs=False)
    o_ref, lse_ref = ref_of(oracle, b)
    out, lse = run_gpu(fsr, b, d, out_dtype)
    err = check_attention(out, o_ref, "bf16", b.N)
    print(f"heads={heads} out={out_dtype} max rel err {err:.3e}")
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=2e-5, atol=2e-5)


@pytest.mark.parametrize("max_q_len", [0, 1, 2, 5])
def test_bf16_row_bound_hint_only_changes_speed(fsr, oracle, max_q_len):
    announce(f"attention bf16 max_q_len hint={max_q_len}")
    b = workloads.make_batch(2, rep=77, with_probs=False, ctx_lens=[300, 45, 513, 128], spec_lens=[8, 3, 6, 0])
    d = DeviceBatch(b, probs=False)
    o_ref, _ = ref_of(oracle, b)
    out, _ = run_gpu(fsr, b, d, torch.float32, max_q_len=max_q_len, want_lse=False)
    check_attention(out, o_ref, "bf16", b.N)


def test_bf16_garbage_beyond_length_is_ignored(fsr, oracle):
    """Slots past a request's last token (page tails, spare pages) hold NaN: the output must not change."""
    announce("attention bf16 NaN poison beyond kv length")
    b = workloads.make_batch(2, rep=5, with_probs=False, ctx_lens=[37, 200, 16, 95], spec_lens=[2, 5, 0, 7])
    o_ref, _ = ref_of(oracle, b)
    used = np.zeros((b.n_pages, b.P), bool)
    for i in range(b.B):
        L = int(b.ctx_lens[i] + b.spec_lens[i] + 1)
        for t in range(L):
            used[b.block_tables[i, t // b.P], t % b.P] = True
    nan16 = np.uint16(0x7FC0)
    d = DeviceBatch(b, probs=False)
    kk = np.ascontiguousarray(np.moveaxis(b.k_cache, 1, 2)).copy()
    vv = np.ascontiguousarray(np.moveaxis(b.v_cache, 1, 2)).copy()
    kk[~used] = nan16
    vv[~used] = nan16
    d.k_cache = dev(np.ascontiguousarray(np.moveaxis(kk, 2, 1)), True)
    d.v_cache = dev(np.ascontiguousarray(np.moveaxis(vv, 2, 1)), True)
    out, _ = run_gpu(fsr, b, d, torch.float32, want_lse=False)
    check_attention(out, o_ref, "bf16", b.N)


def test_empty_request_and_row_capacity(fsr, oracle):
    announce("attention empty request, N_cap > N")
    b = workloads.make_batch(2, rep=6, with_probs=False, ctx_lens=[120, 64, 300], spec_lens=[2, 4, 1])
    # re-deal the rows: request 1 gets none
    cu = np.array([0, 3, 3, 5], np.int32)
    o_ref, _ = ref_of(oracle, b, q=b.q[:5], cu=cu)
    d = DeviceBatch(b, probs=False)
    out, _ = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, None, dev(cu), scale=b.scale,
                                  out_dtype=torch.float32, max_q_len=3)
    torch.cuda.synchronize()
    check_attention(out, o_ref, "bf16", 5)


def test_generic_bf16_d64(fsr, oracle):
    announce("attention bf16 D=64 (generic path)")
    b = workloads.make_batch(1, rep=2, with_probs=False, dtype="bf16")
    d = DeviceBatch(b, probs=False)
    o_ref, _ = ref_of(oracle, b)
    for od in (torch.float32, torch.bfloat16):
        out, _ = run_gpu(fsr, b, d, od, want_lse=False)
        check_attention(out, o_ref, "bf16", b.N)


def test_config2_full_size_and_determinism(fsr, oracle):
    announce("attention config2 full size")
    b = workloads.make_batch(2, with_probs=False)
    d = DeviceBatch(b, probs=False)
    o_ref, lse_ref = ref_of(oracle, b)
    out, lse = run_gpu(fsr, b, d, torch.bfloat16)
    err = check_attention(out, o_ref, "bf16", b.N)
    out32, _ = run_gpu(fsr, b, d, torch.float32, want_lse=False)
    err32 = check_attention(out32, o_ref, "bf16", b.N)
    print(f"config2: max rel err bf16-out {err:.3e}, fp32-out {err32:.3e}")
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=2e-5, atol=2e-5)
    out2, _ = run_gpu(fsr, b, d, torch.bfloat16, want_lse=False)
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))  # same bits on a re-run


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_token_major_cache_layout(fsr, oracle, out_dtype):
    """Caches laid out [n_pages, P, H_kv, D] (one block per token instead of one per head)."""
    announce(f"attention token-major KV layout out={out_dtype}")
    ctx = [0, 1, 15, 16, 31, 33, 100, 257, 511, 640, 700, 1029, 2100]
    spec = [3, 0, 8, 1, 2, 7, 4, 8, 5, 6, 0, 8, 3]
    b = workloads.make_batch(2, rep=61, with_probs=False, ctx_lens=ctx, spec_lens=spec)
    k_tm = np.ascontiguousarray(np.swapaxes(b.k_cache, 1, 2))
    v_tm = np.ascontiguousarray(np.swapaxes(b.v_cache, 1, 2))
    o_ref, lse_ref = oracle.verify_attention(b.q, k_tm, v_tm, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv,
                                             D=b.D, P=b.P, dtype=b.dtype, scale=b.scale, token_major=True)
    d = DeviceBatch(b, probs=False)
    lse = torch.zeros((b.N, b.H_q), dtype=torch.float32, device="cuda")
    out, lse = fsr.verify_attention(d.q, dev(k_tm, True), dev(v_tm, True), d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                    scale=b.scale, out_dtype=out_dtype, lse=lse, max_q_len=b.S_max + 1, kv_layout=1)
    torch.cuda.synchronize()
    check_attention(out, o_ref, "bf16", b.N)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=2e-5, atol=2e-5)


def test_token_major_generic_path_and_append(fsr, oracle):
    announce("token-major layout: fp32 generic path, and cache append")
    b = workloads.make_batch(1, rep=9, with_probs=False)
    k_tm = np.ascontiguousarray(np.swapaxes(b.k_cache, 1, 2))
    v_tm = np.ascontiguousarray(np.swapaxes(b.v_cache, 1, 2))
    o_ref, _ = oracle.verify_attention(b.q, k_tm, v_tm, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv, D=b.D,
                                       P=b.P, dtype=b.dtype, scale=b.scale, token_major=True)
    d = DeviceBatch(b, probs=False)
    out, _ = fsr.verify_attention(d.q, dev(k_tm), dev(v_tm), d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                  scale=b.scale, out_dtype=torch.float32, max_q_len=b.S_max + 1, kv_layout=1)
    torch.cuda.synchronize()
    check_attention(out, o_ref, "f32", b.N)
    rng = np.random.default_rng(2)
    k_new = rng.standard_normal((b.N, b.H_kv, b.D)).astype(np.float32)
    v_new = rng.standard_normal((b.N, b.H_kv, b.D)).astype(np.float32)
    kc, vc = dev(k_tm), dev(v_tm)
    fsr.kv_append(dev(k_new), dev(v_new), kc, vc, d.block_tables, d.ctx_lens, d.cu_q, kv_layout=1)
    torch.cuda.synchronize()
    kr, vr = oracle.kv_append(k_new, v_new, k_tm, v_tm, b.block_tables, b.ctx_lens, b.cu_q, P=b.P, token_major=True)
    assert np.array_equal(kc.cpu().numpy(), kr) and np.array_equal(vc.cpu().numpy(), vr)


def test_alternating_caches_share_one_workspace(fsr, oracle):
    """Many launches on one workspace with the cache contents swapped between two sets every time: a partial of a
    cut item left over from the launch before (same slot, same shapes, other data) must never be picked up."""
    announce("attention alternating caches on one workspace")
    b = workloads.make_batch(2, rep=41, with_probs=False, ctx_lens=[3000, 2500, 1800, 2200, 900, 1400], spec_lens=[8, 3, 5, 1, 7, 2])
    b2 = workloads.make_batch(2, rep=42, with_probs=False, ctx_lens=[3000, 2500, 1800, 2200, 900, 1400], spec_lens=[8, 3, 5, 1, 7, 2])
    assert b2.k_cache.shape == b.k_cache.shape and not np.array_equal(b.k_cache, b2.k_cache)   # b's metadata serves both
    d_bt, d_ctx, d_spec, d_cu = dev(b.block_tables), dev(b.ctx_lens), dev(b.spec_lens), dev(b.cu_q)
    sets = [(dev(x.q, True), dev(x.k_cache, True), dev(x.v_cache, True)) for x in (b, b2)]
    need = fsr.attn_workspace_bytes(B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, max_pages=b.max_pages,
                                    n_pages=b.n_pages, dtype=torch.bfloat16, out_dtype=torch.float32, max_q_len=b.S_max + 1)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    first = []
    for q, k, v in sets:
        out, _ = fsr.verify_attention(q, k, v, d_bt, d_ctx, d_spec, d_cu, scale=b.scale, out_dtype=torch.float32, workspace=ws,
                                      max_q_len=b.S_max + 1)
        first.append(out.clone())
    torch.cuda.synchronize()
    for x, o in zip((b, b2), first):
        o_ref, _ = ref_of(oracle, b, q=x.q, k=x.k_cache, v=x.v_cache)
        check_attention(o, o_ref, "bf16", b.N)
    assert not torch.equal(first[0], first[1])
    outs = [torch.empty_like(first[0]) for _ in range(2)]
    for it in range(150):
        s = it & 1
        q, k, v = sets[s]
        fsr.verify_attention(q, k, v, d_bt, d_ctx, d_spec, d_cu, scale=b.scale, out=outs[s], workspace=ws, max_q_len=b.S_max + 1)
        if it % 10 >= 8:
            torch.cuda.synchronize()
            assert torch.equal(outs[s].view(torch.int32), first[s].view(torch.int32)), f"launch {it}"
    torch.cuda.synchronize()


def test_graph_of_launches_on_one_workspace_with_two_cache_sets(fsr, oracle):
    """Eight launches captured in one HIP graph, odd and even ones over different cache contents, all on one
    workspace; replayed with eager work in between, every replay bit-identical to the eager results."""
    announce("attention graph with alternating caches")
    lens = dict(ctx_lens=[2800, 2100, 1500, 3300, 700, 1900, 2600, 1200], spec_lens=[6, 2, 8, 0, 5, 3, 7, 1])
    b = workloads.make_batch(2, rep=51, with_probs=False, **lens)
    b2 = workloads.make_batch(2, rep=52, with_probs=False, **lens)
    d_bt, d_ctx, d_spec, d_cu = dev(b.block_tables), dev(b.ctx_lens), dev(b.spec_lens), dev(b.cu_q)
    sets = [(dev(x.q, True), dev(x.k_cache, True), dev(x.v_cache, True)) for x in (b, b2)]
    need = fsr.attn_workspace_bytes(B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, max_pages=b.max_pages,
                                    n_pages=b.n_pages, dtype=torch.bfloat16, out_dtype=torch.bfloat16, max_q_len=b.S_max + 1)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    outs = [torch.empty_like(sets[0][0]) for _ in range(8)]

    def step():
        for l in range(8):
            q, k, v = sets[l & 1]
            fsr.verify_attention(q, k, v, d_bt, d_ctx, d_spec, d_cu, scale=b.scale, out=outs[l], workspace=ws, max_q_len=b.S_max + 1)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
        torch.cuda.synchronize()
        eager = [o.clone() for o in outs]
        for x, o in zip((b, b2), eager[:2]):
            o_ref, _ = ref_of(oracle, b, q=x.q, k=x.k_cache, v=x.v_cache)
            check_attention(o, o_ref, "bf16", b.N)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        for rep in range(12):
            for o in outs:
                o.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for l in range(8):
                assert torch.equal(outs[l].view(torch.int16), eager[l].view(torch.int16)), (rep, l)


def test_binding_refuses_a_workspace_in_use_on_another_stream(fsr, oracle):
    """One call in flight per workspace: the binding refuses a workspace whose last call, on another stream, may
    still be running, and takes it again once that stream has drained."""
    announce("workspace shared by two streams")
    b = workloads.make_batch(2, rep=77, with_probs=False, ctx_lens=[300, 45, 513, 700], spec_lens=[3, 0, 8, 5])
    d = DeviceBatch(b, probs=False)
    ws = torch.empty(fsr.attn_workspace_bytes(B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, max_pages=b.max_pages,
                                              n_pages=b.n_pages, dtype=torch.bfloat16, out_dtype=torch.float32, max_q_len=b.S_max + 1),
                     dtype=torch.uint8, device="cuda")
    args = (d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q)
    kw = dict(scale=b.scale, out_dtype=torch.float32, workspace=ws, max_q_len=b.S_max + 1)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s1):
        torch.cuda._sleep(200_000_000)          # keeps s1 busy for tens of milliseconds
        o1, _ = fsr.verify_attention(*args, **kw)
    with torch.cuda.stream(s2):
        with pytest.raises(fsr.FsrError):
            fsr.verify_attention(*args, **kw)
    torch.cuda.synchronize()
    with torch.cuda.stream(s2):
        o2, _ = fsr.verify_attention(*args, **kw)
    torch.cuda.synchronize()
    o_ref, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv,
                                       D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    check_attention(o1, o_ref, "bf16", b.N)
    check_attention(o2, o_ref, "bf16", b.N)
