"""GPU parity: verify_attention reading a per-step plan (fsr_attn_plan / fsr_verify_attention_planned)
against the same call building its own schedule (bit-identical) and against the oracle."""
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


def ref_of(oracle, b):
    return oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv,
                                   D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)


def both_ways(fsr, b, d, out_dtype, max_q_len, **kw):
    """(out, lse) of the self-scheduling call and of the planned call, on NaN-filled outputs."""
    res = []
    for planned in (False, True):
        out = torch.full((b.N, b.H_q, b.D), float("nan"), dtype=out_dtype, device="cuda")
        lse = torch.full((b.N, b.H_q), float("nan"), dtype=torch.float32, device="cuda")
        plan = fsr.attn_plan(d.q, d.k_cache, d.block_tables, d.ctx_lens, d.cu_q, scale=b.scale, out_dtype=out_dtype,
                             max_q_len=max_q_len, **kw) if planned else None
        fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale,
                             out=out, lse=lse, max_q_len=max_q_len, plan=plan, **kw)
        torch.cuda.synchronize()
        res.append((out, lse))
    return res


def same_bits(x, y):
    bits = torch.int16 if x.dtype == torch.bfloat16 else torch.int32
    return torch.equal(x.view(bits), y.view(bits))


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("heads", [(32, 8), (64, 8), (8, 8)])
def test_planned_equals_unplanned_small(fsr, oracle, heads, out_dtype):
    H_q, H_kv = heads
    announce(f"planned attention small heads={heads} out={out_dtype}")
    ctx = [0, 1, 15, 16, 31, 33, 100, 257, 511, 640, 700, 1029, 2000, 5, 3000]
    spec = [3, 0, 8, 1, 2, 7, 4, 10, 5, 6, 0, 9, 2, 0, 8]
    b = workloads.make_batch(2, rep=H_q + 1, with_probs=False, H_q=H_q, H_kv=H_kv, ctx_lens=ctx, spec_lens=spec)
    d = DeviceBatch(b, probs=False)
    o_ref, lse_ref = ref_of(oracle, b)
    (o0, l0), (o1, l1) = both_ways(fsr, b, d, out_dtype, b.S_max + 1)
    assert same_bits(o0, o1) and same_bits(l0, l1)
    check_attention(o1, o_ref, "bf16", b.N)
    np.testing.assert_allclose(l1.cpu().numpy(), lse_ref, rtol=2e-5, atol=2e-5)


@pytest.mark.parametrize("kw", [dict(max_workgroups=40), dict(max_workgroups=1), dict(kv_layout=1), dict()])
@pytest.mark.parametrize("max_q_len", [0, 9])
def test_planned_grid_sizes_layouts_and_unknown_row_bound(fsr, oracle, kw, max_q_len):
    announce(f"planned attention {kw} max_q_len={max_q_len}")
    b = workloads.make_batch(2, rep=31, with_probs=False, ctx_lens=[300, 45, 513, 128, 1500, 77, 0, 2047],
                             spec_lens=[8, 3, 6, 0, 2, 5, 1, 8])
    d = DeviceBatch(b, probs=False)
    if kw.get("kv_layout"):
        d.k_cache = d.k_cache.transpose(1, 2).contiguous()
        d.v_cache = d.v_cache.transpose(1, 2).contiguous()
    o_ref, _ = ref_of(oracle, b)
    (o0, l0), (o1, l1) = both_ways(fsr, b, d, torch.float32, max_q_len, **kw)
    assert same_bits(o0, o1) and same_bits(l0, l1)
    check_attention(o1, o_ref, "bf16", b.N)


def test_planned_config2_full_size_and_many_segments(fsr, oracle):
    announce("planned attention config2 full size")
    b = workloads.make_batch(2, with_probs=False)
    d = DeviceBatch(b, probs=False)
    o_ref, _ = ref_of(oracle, b)
    (o0, l0), (o1, l1) = both_ways(fsr, b, d, torch.bfloat16, b.S_max + 1)
    assert same_bits(o0, o1) and same_bits(l0, l1)
    check_attention(o1, o_ref, "bf16", b.N)
    # many short requests: a share spans tens of items, so a workgroup reads far more than its first record
    announce("planned attention B=700 short requests")
    rng = np.random.default_rng(9)
    b = workloads.make_batch(3, rep=3, with_probs=False, B=700, ctx_lens=rng.integers(0, 90, 700).tolist(),
                             spec_lens=rng.integers(0, 4, 700).tolist())
    d = DeviceBatch(b, probs=False)
    o_ref, _ = ref_of(oracle, b)
    (o0, l0), (o1, l1) = both_ways(fsr, b, d, torch.float32, b.S_max + 1)
    assert same_bits(o0, o1) and same_bits(l0, l1)
    check_attention(o1, o_ref, "bf16", b.N)


def test_plan_reused_across_layers_in_a_graph_and_refused_for_other_shapes(fsr, oracle):
    announce("planned attention: one plan, three caches, graph replays; shape mismatch refused")
    b = workloads.make_batch(2, rep=12, with_probs=False, ctx_lens=[900, 45, 513, 128, 1000, 77], spec_lens=[8, 3, 6, 0, 2, 5])
    d = DeviceBatch(b, probs=False)
    gen = torch.Generator(device="cuda"); gen.manual_seed(3)
    caches = [(d.k_cache, d.v_cache)] + [
        (torch.randn(d.k_cache.shape, generator=gen, device="cuda").to(torch.bfloat16),
         torch.randn(d.v_cache.shape, generator=gen, device="cuda").to(torch.bfloat16)) for _ in range(2)]
    mq = b.S_max + 1
    eager = []
    for k, v in caches:
        o, _ = fsr.verify_attention(d.q, k, v, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale, max_q_len=mq)
        eager.append(o)
    torch.cuda.synchronize()
    outs = [torch.empty_like(d.q) for _ in caches]
    need = fsr.attn_workspace_bytes(B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, max_pages=b.max_pages,
                                    n_pages=b.n_pages, dtype=torch.bfloat16, out_dtype=torch.bfloat16, max_q_len=mq)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    plan = fsr.attn_plan(d.q, d.k_cache, d.block_tables, d.ctx_lens, d.cu_q, scale=b.scale, max_q_len=mq)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        def step():
            fsr.attn_plan(d.q, d.k_cache, d.block_tables, d.ctx_lens, d.cu_q, scale=b.scale, max_q_len=mq, plan=plan)
            for (k, v), o in zip(caches, outs):
                fsr.verify_attention(d.q, k, v, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale, out=o,
                                     workspace=ws, max_q_len=mq, plan=plan)
        step()
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        for _ in range(3):
            for o in outs:
                o.zero_()
            plan.zero_()
            g.replay()
            stream.synchronize()
            for o, e in zip(outs, eager):
                assert same_bits(o, e)
    o_ref, _ = ref_of(oracle, b)
    check_attention(outs[0], o_ref, "bf16", b.N)
    # the same buffer with other shapes: refused on the host
    with pytest.raises(fsr.FsrError) as ei:
        fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale,
                             max_q_len=3, plan=plan)
    assert ei.value.code == -2
    with pytest.raises(fsr.FsrError):
        fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale,
                             max_q_len=mq, plan=torch.zeros(1 << 20, dtype=torch.uint8, device="cuda"))
    # a plan buffer whose contents were lost (zeroed) while the host still knows it: the kernel leaves `out` alone
    plan.zero_()
    out = torch.full_like(d.q, 7.0)
    fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q, scale=b.scale, out=out,
                         max_q_len=mq, plan=plan)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


@pytest.mark.parametrize("kw", [dict(), dict(max_workgroups=3), dict(max_workgroups=37), dict(kv_layout=1)])
@pytest.mark.parametrize("heads", [(32, 8), (64, 8), (48, 16), (16, 1)])
def test_wide_row_groups_take_two_teams_of_waves(fsr, oracle, heads, kw):
    """Suffixes whose G * q_len rows exceed four query tiles: row groups of two teams (some with a short or
    empty second team, some requests with several groups), cut by share boundaries at small grids; the planned and
    the self-scheduling kernel agree bit for bit and with the oracle."""
    H_q, H_kv = heads
    announce(f"wide row groups heads={heads} {kw}")
    ctx = [700, 0, 1, 31, 33, 257, 1500, 2047, 90, 3100, 16, 640]
    spec = [32, 24, 12, 13, 6, 25, 11, 30, 0, 23, 17, 5]
    b = workloads.make_batch(2, rep=90 + H_q, with_probs=False, H_q=H_q, H_kv=H_kv, ctx_lens=ctx, spec_lens=spec)
    d = DeviceBatch(b, probs=False)
    if kw.get("kv_layout"):
        d.k_cache = d.k_cache.transpose(1, 2).contiguous()
        d.v_cache = d.v_cache.transpose(1, 2).contiguous()
    o_ref, lse_ref = ref_of(oracle, b)
    (o0, l0), (o1, l1) = both_ways(fsr, b, d, torch.float32, b.S_max + 1, **kw)
    assert same_bits(o0, o1) and same_bits(l0, l1)
    check_attention(o1, o_ref, "bf16", b.N)
    np.testing.assert_allclose(l1.cpu().numpy(), lse_ref, rtol=2e-5, atol=2e-5)
