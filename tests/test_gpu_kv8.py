"""GPU parity: verification attention over 8-bit (E4M3) KV caches vs the oracle reading the same bytes.
The bytes widen exactly, so the bound is the bf16-cache kernel's: 2e-3 relative on the fp32 output (measured
~1e-5), a bf16 output within its rounding on top."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import announce, check_attention, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def quantise(b, seed, poison=False):
    """The batch's bf16 caches re-stored as E4M3 bytes with per-head scales; unused slots optionally NaN codes."""
    rng = np.random.default_rng(seed)
    k_scale = rng.uniform(0.01, 0.05, b.H_kv).astype(np.float32)
    v_scale = rng.uniform(0.01, 0.05, b.H_kv).astype(np.float32)
    kf, vf = workloads.bf16_bits_to_f32(b.k_cache), workloads.bf16_bits_to_f32(b.v_cache)
    k8 = workloads.f32_to_e4m3_bits(kf / k_scale.reshape(1, -1, 1, 1))
    v8 = workloads.f32_to_e4m3_bits(vf / v_scale.reshape(1, -1, 1, 1))
    if poison:
        used = np.zeros((b.n_pages, b.P), bool)
        for i in range(b.B):
            for t in range(int(b.ctx_lens[i] + b.spec_lens[i] + 1)):
                used[b.block_tables[i, t // b.P], t % b.P] = True
        for c in (k8, v8):
            m = np.moveaxis(c, 1, 2)      # view [page, slot, head, d]
            m[~used] = 0x7F               # NaN code
    return k8, v8, k_scale, v_scale


def run_pair(fsr, oracle, b, k8, v8, k_scale, v_scale, out_dtype, token_major=False, max_q_len=None):
    o_ref, lse_ref = oracle.verify_attention_kv8(b.q, k8, v8, k_scale, v_scale, b.block_tables, b.ctx_lens, b.cu_q,
                                                 H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, scale=b.scale)
    kd, vd = (np.ascontiguousarray(np.swapaxes(c, 1, 2)) if token_major else c for c in (k8, v8))
    lse = torch.empty(b.N, b.H_q, dtype=torch.float32, device="cuda")
    args = (dev(b.q, True), dev(kd), dev(vd), dev(k_scale), dev(v_scale), dev(b.block_tables), dev(b.ctx_lens), dev(b.cu_q))
    kw = dict(scale=b.scale, out_dtype=out_dtype, max_q_len=b.S_max + 1 if max_q_len is None else max_q_len,
              kv_layout=fsr.binding.KV_TOKEN_MAJOR if token_major else fsr.binding.KV_HEAD_MAJOR)
    out, _ = fsr.verify_attention_kv8(*args, lse=lse, **kw)
    # the same call reading a per-step plan (one plan serves bf16 and 8-bit caches): bit-identical
    plan = fsr.attn_plan(args[0], args[1], args[5], args[6], args[7], **kw)
    lse_p = torch.full_like(lse, float("nan"))
    out_p, _ = fsr.verify_attention_kv8(*args, lse=lse_p, plan=plan, **kw)
    torch.cuda.synchronize()
    bits = torch.int16 if out.dtype == torch.bfloat16 else torch.int32
    assert torch.equal(out.view(bits), out_p.view(bits)) and torch.equal(lse.view(torch.int32), lse_p.view(torch.int32))
    err = check_attention(out, o_ref, "bf16", b.N)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=2e-5, atol=2e-5)
    return err


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("heads", [(32, 8), (8, 8), (64, 8), (16, 1)])
def test_kv8_small(fsr, oracle, heads, out_dtype):
    H_q, H_kv = heads
    announce(f"attention kv8 small heads={heads} out={out_dtype}")
    ctx = [0, 1, 15, 16, 31, 33, 100, 257, 511, 640, 700, 1029]
    spec = [3, 0, 8, 1, 2, 7, 4, 10, 5, 6, 0, 9]
    b = workloads.make_batch(2, rep=H_q + 1, with_probs=False, H_q=H_q, H_kv=H_kv, ctx_lens=ctx, spec_lens=spec)
    err = run_pair(fsr, oracle, b, *quantise(b, H_q), out_dtype)
    print(f"kv8 heads={heads} out={out_dtype} max rel err {err:.3e}")


def test_kv8_token_major_and_nan_codes_beyond_length(fsr, oracle):
    announce("attention kv8 token-major + NaN codes beyond length")
    b = workloads.make_batch(2, rep=9, with_probs=False, ctx_lens=[37, 200, 16, 95, 1500], spec_lens=[2, 5, 0, 7, 8])
    q = quantise(b, 1, poison=True)
    run_pair(fsr, oracle, b, *q, torch.float32, token_major=False)
    run_pair(fsr, oracle, b, *q, torch.float32, token_major=True)


def test_kv8_every_code_decodes_as_the_format_says(fsr, oracle):
    """A one-row request whose single key is constant and whose value row runs through every byte code: the
    output is the decoded values themselves (softmax over one key), so each finite code is checked on its own."""
    announce("attention kv8 all codes")
    b = workloads.make_batch(2, rep=11, with_probs=False, H_q=8, H_kv=8, ctx_lens=[0, 0], spec_lens=[0, 0])
    k8 = np.full(b.k_cache.shape, 0x38, np.uint8)   # 1.0
    v8 = np.zeros(b.v_cache.shape, np.uint8)
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], np.uint8)   # 254 finite codes
    for i in range(2):
        page = b.block_tables[i, 0]
        for h in range(8):
            v8[page, h, 0, :] = codes[(np.arange(128) + 128 * i + 17 * h) % len(codes)]
    ones = np.ones(8, np.float32)
    o_ref, _ = oracle.verify_attention_kv8(b.q, k8, v8, ones, ones, b.block_tables, b.ctx_lens, b.cu_q,
                                           H_q=8, H_kv=8, D=b.D, P=b.P, scale=b.scale)
    out, _ = fsr.verify_attention_kv8(dev(b.q, True), dev(k8), dev(v8), dev(ones), dev(ones), dev(b.block_tables),
                                      dev(b.ctx_lens), dev(b.cu_q), scale=b.scale, out_dtype=torch.float32, max_q_len=1)
    torch.cuda.synchronize()
    # (the row's own probability is exp2 of a rounding residue, not exactly 1: a few ulp, far below the 6 % between codes)
    np.testing.assert_allclose(out.cpu().numpy().astype(np.float64), o_ref, rtol=1e-6, atol=0)


def test_kv8_config2_sampled_rows(fsr, oracle):
    """Workload 2's shape with 8-bit caches, in the launch configuration of the bench; checked on 3 requests."""
    announce("attention kv8 config2")
    b = workloads.make_batch(2, with_probs=False)
    k8, v8, ks, vs = quantise(b, 2)
    out, _ = fsr.verify_attention_kv8(dev(b.q, True), dev(k8), dev(v8), dev(ks), dev(vs), dev(b.block_tables), dev(b.ctx_lens),
                                      dev(b.cu_q), scale=b.scale, out_dtype=torch.float32, max_q_len=b.S_max + 1)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    for i in (0, 7, 15):
        r0, r1 = int(b.cu_q[i]), int(b.cu_q[i + 1])
        o_ref, _ = oracle.verify_attention_kv8(b.q[r0:r1], k8, v8, ks, vs, b.block_tables[i:i + 1], b.ctx_lens[i:i + 1],
                                               np.array([0, r1 - r0], np.int32), H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, scale=b.scale)
        check_attention(torch.from_numpy(out[r0:r1]), o_ref, "bf16", r1 - r0)


def test_kv8_unsupported_shapes_are_refused(fsr):
    announce("attention kv8 refusals")
    q = torch.zeros(4, 8, 64, dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros(2, 8, 16, 64, dtype=torch.uint8, device="cuda")
    sc = torch.ones(8, device="cuda")
    bt = torch.zeros(1, 2, dtype=torch.int32, device="cuda")
    with pytest.raises(fsr.FsrError) as e:
        fsr.verify_attention_kv8(q, kc, kc, sc, sc, bt, torch.zeros(1, dtype=torch.int32, device="cuda"),
                                 torch.tensor([0, 4], dtype=torch.int32, device="cuda"), scale=1.0)
    assert e.value.code == -3


@pytest.mark.parametrize("token_major", [False, True])
def test_kv8_append_bytes_match_oracle_then_attention(fsr, oracle, token_major):
    """Quantising append: every stored byte equals the oracle's (fp32 division, nearest-even E4M3, saturation,
    NaN), over magnitudes from the subnormal range to beyond 448; then attention over the appended caches."""
    announce(f"kv8 append token_major={token_major}")
    b = workloads.make_batch(2, rep=21, with_probs=False, ctx_lens=[0, 5, 16, 47, 300], spec_lens=[3, 0, 8, 2, 6])
    rng = np.random.default_rng(7)
    k8, v8, ks, vs = quantise(b, 3)
    mag = 10.0 ** rng.uniform(-4, 1.5, size=(b.N, b.H_kv, b.D))             # x / scale spans 2^-12 .. ~3000
    k_new = (rng.standard_normal((b.N, b.H_kv, b.D)) * mag).astype(np.float32)
    v_new = rng.standard_normal((b.N, b.H_kv, b.D)).astype(np.float32) * 0.05
    k_new[0, 0, :4] = [np.nan, 1e30, -1e30, 0.0]
    k_bits, v_bits = workloads.f32_to_bf16_bits(k_new), workloads.f32_to_bf16_bits(v_new)
    lay = fsr.binding.KV_TOKEN_MAJOR if token_major else fsr.binding.KV_HEAD_MAJOR
    to_lay = (lambda c: np.ascontiguousarray(np.swapaxes(c, 1, 2))) if token_major else (lambda c: c)
    kc_ref, vc_ref = oracle.kv_append_kv8(k_bits, v_bits, to_lay(k8), to_lay(v8), ks, vs, b.block_tables, b.ctx_lens, b.cu_q,
                                          P=b.P, token_major=token_major)
    kc, vc = dev(to_lay(k8)), dev(to_lay(v8))
    fsr.kv_append_kv8(dev(k_bits, True), dev(v_bits, True), kc, vc, dev(ks), dev(vs), dev(b.block_tables), dev(b.ctx_lens),
                      dev(b.cu_q), kv_layout=lay)
    torch.cuda.synchronize()
    assert np.array_equal(kc.cpu().numpy(), kc_ref) and np.array_equal(vc.cpu().numpy(), vc_ref)
    assert (kc_ref != to_lay(k8)).any()
    # attention over what was appended (the NaN element sits in request 0's own rows: give that row a finite value first)
    if not token_major:
        k_bits2 = k_bits.copy(); k_bits2[0, 0, :4] = 0
        kc2_ref, vc2_ref = oracle.kv_append_kv8(k_bits2, v_bits, k8, v8, ks, vs, b.block_tables, b.ctx_lens, b.cu_q, P=b.P)
        kc2, vc2 = dev(k8), dev(v8)
        fsr.kv_append_kv8(dev(k_bits2, True), dev(v_bits, True), kc2, vc2, dev(ks), dev(vs), dev(b.block_tables), dev(b.ctx_lens), dev(b.cu_q))
        o_ref, _ = oracle.verify_attention_kv8(b.q, kc2_ref, vc2_ref, ks, vs, b.block_tables, b.ctx_lens, b.cu_q,
                                               H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, scale=b.scale)
        out, _ = fsr.verify_attention_kv8(dev(b.q, True), kc2, vc2, dev(ks), dev(vs), dev(b.block_tables), dev(b.ctx_lens),
                                          dev(b.cu_q), scale=b.scale, out_dtype=torch.float32, max_q_len=b.S_max + 1)
        torch.cuda.synchronize()
        check_attention(out, o_ref, "bf16", b.N)


def test_kv8_empty_requests_small_grid_and_append_without_a_page(fsr, oracle):
    """Requests without rows cost nothing; a persistent grid cut down to a few workgroups gives the same result; an
    append whose position has no page (beyond max_pages * P) or whose page id is outside the pool is skipped."""
    announce("kv8 edge cases")
    b = workloads.make_batch(2, rep=31, with_probs=False, ctx_lens=[40, 7, 300, 0, 64], spec_lens=[2, 0, 5, 1, 3])
    k8, v8, ks, vs = quantise(b, 5)
    # requests 1 and 3 get no rows in this call
    q_lens = np.array([3, 0, 6, 0, 4], np.int32)
    cu = workloads.exclusive_offsets(q_lens)
    rows = np.concatenate([np.arange(b.cu_q[i], b.cu_q[i] + q_lens[i]) for i in range(b.B)])
    q = np.ascontiguousarray(b.q[rows])
    o_ref, _ = oracle.verify_attention_kv8(q, k8, v8, ks, vs, b.block_tables, b.ctx_lens, cu, H_q=b.H_q, H_kv=b.H_kv, D=b.D,
                                           P=b.P, scale=b.scale)
    for n_wg in (0, 3):
        out, _ = fsr.verify_attention_kv8(dev(q, True), dev(k8), dev(v8), dev(ks), dev(vs), dev(b.block_tables), dev(b.ctx_lens),
                                          dev(cu), scale=b.scale, out_dtype=torch.float32, max_q_len=6, max_workgroups=n_wg)
        torch.cuda.synchronize()
        check_attention(out, o_ref, "bf16", len(rows))
    # append: request 0's rows land past its last page when the table is cut to 2 pages (32 tokens, ctx = 40);
    # request 2 points at a page outside the pool
    bt = b.block_tables[:, :2].copy()
    ctx = np.array([40, 7, 10, 0, 12], np.int32)
    bt[2, 0] = b.n_pages + 5
    rng = np.random.default_rng(9)
    k_new = workloads.f32_to_bf16_bits(rng.standard_normal((len(rows), b.H_kv, b.D)).astype(np.float32))
    v_new = workloads.f32_to_bf16_bits(rng.standard_normal((len(rows), b.H_kv, b.D)).astype(np.float32))
    kc, vc = dev(k8), dev(v8)
    fsr.kv_append_kv8(dev(k_new, True), dev(v_new, True), kc, vc, dev(ks), dev(vs), dev(bt), dev(ctx), dev(cu))
    torch.cuda.synchronize()
    bt_ref = bt.copy(); bt_ref[2, 0] = 0   # the oracle has no notion of a bad page id: drop request 2's rows instead
    cu_ref_lens = q_lens.copy(); cu_ref_lens[2] = 0
    keep = np.concatenate([np.arange(cu[i], cu[i] + cu_ref_lens[i]) for i in range(b.B)]).astype(int)
    kc_ref, vc_ref = oracle.kv_append_kv8(k_new[keep], v_new[keep], k8, v8, ks, vs, bt_ref, ctx,
                                          workloads.exclusive_offsets(cu_ref_lens), P=b.P)
    assert np.array_equal(kc.cpu().numpy(), kc_ref) and np.array_equal(vc.cpu().numpy(), vc_ref)
    assert (kc_ref != k8).any()     # request 4's rows did land
