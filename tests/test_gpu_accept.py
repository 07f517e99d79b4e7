"""GPU parity: spec_accept vs the oracle.  accepted_len / n_emitted bit-exact; emitted tokens
bit-exact except draws whose uniform lies within 1e-6 of a CDF boundary (counted)."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_accept, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def run_pair(fsr, oracle, b, mode=0, temperature=1.0):
    d = DeviceBatch(b, kv=False, logits=bool(mode))
    if mode:
        ref = oracle.spec_accept(b.z_target, b.z_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                                 S_max=b.S_max, mode=1, temperature=temperature)
        gpu = fsr.spec_accept(d.z_target, d.z_draft, d.draft_tokens, d.u_accept, d.u_sample, d.cu_q, d.cu_d,
                              S_max=b.S_max, mode=1, temperature=temperature)
    else:
        ref = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                                 S_max=b.S_max)
        gpu = fsr.spec_accept(d.p_target, d.p_draft, d.draft_tokens, d.u_accept, d.u_sample, d.cu_q, d.cu_d,
                              S_max=b.S_max)
    torch.cuda.synchronize()
    return check_accept(gpu, ref, b.u_sample), ref


@pytest.mark.parametrize("draft_mode", ["independent", "noise", "equal"])
@pytest.mark.parametrize("rep", [0, 1])
def test_config1_tiny(fsr, oracle, draft_mode, rep):
    announce(f"accept config1 {draft_mode} rep={rep}")
    b = workloads.make_batch(1, rep=rep, with_kv=False, draft_mode=draft_mode)
    (frag, mism), ref = run_pair(fsr, oracle, b)
    assert mism == 0
    if draft_mode == "equal":
        assert np.array_equal(ref["accepted_len"], b.spec_lens)


@pytest.mark.parametrize("V", [1000, 1001, 4096, 4097, 9999, 128256])
def test_vocab_sizes_and_ragged_tail(fsr, oracle, V):
    announce(f"accept V={V}")
    b = workloads.make_batch(2, rep=V % 7, with_kv=False, V=V, B=24,
                             spec_lens=[0, 1, 2, 3, 4, 5, 6, 7, 8, 1, 2, 3] * 2, ctx_lens=[10] * 24)
    (frag, mism), ref = run_pair(fsr, oracle, b)
    print(f"V={V}: fragile={frag} mismatches={mism}")
    assert mism == 0
    assert 0 < (ref["accepted_len"] < b.spec_lens).sum() < b.B


def test_config2_full_vocab(fsr, oracle):
    announce("accept config2")
    b = workloads.make_batch(2, with_kv=False)
    (frag, mism), ref = run_pair(fsr, oracle, b)
    print(f"config2: fragile={frag} mismatches={mism} accepted={ref['accepted_len'].sum()}/{b.spec_lens.sum()}")
    assert mism == 0


def test_no_bonus_rows_and_row_maps(fsr, oracle):
    announce("accept row maps / no bonus")
    b = workloads.make_batch(1, rep=3, with_kv=False, V=5000, B=10, spec_lens=[3, 0, 4, 2, 5, 1, 6, 2, 3, 4],
                             ctx_lens=[8] * 10, draft_mode="noise")
    rng = np.random.default_rng(0)
    # storage rows shuffled; call rows reach them through the maps; odd requests lose their bonus row
    perm_t, perm_d = rng.permutation(b.N), rng.permutation(b.N_d)
    p_t = np.empty_like(b.p_target); p_t[perm_t] = b.p_target
    p_d = np.empty_like(b.p_draft); p_d[perm_d] = b.p_draft
    toks = np.empty_like(b.draft_tokens); toks[perm_d] = b.draft_tokens
    u_a = np.empty_like(b.u_accept); u_a[perm_d] = b.u_accept
    t_lens = b.spec_lens + 1 - (np.arange(b.B) % 2)
    t_lens[b.spec_lens == 0] = 1
    cu_t = workloads.exclusive_offsets(t_lens)
    t_rows = np.concatenate([perm_t[b.cu_q[i]: b.cu_q[i] + t_lens[i]] for i in range(b.B)]).astype(np.int32)
    d_rows = perm_d.astype(np.int32)
    ref = oracle.spec_accept(p_t, p_d, toks, u_a, b.u_sample, cu_t, b.cu_d, S_max=b.S_max, t_rows=t_rows, d_rows=d_rows)
    gpu = fsr.spec_accept(dev(p_t), dev(p_d), dev(toks), dev(u_a), dev(b.u_sample), dev(cu_t), dev(b.cu_d),
                          S_max=b.S_max, t_rows=dev(t_rows), d_rows=dev(d_rows))
    torch.cuda.synchronize()
    frag, mism = check_accept(gpu, ref, b.u_sample)
    assert mism == 0
    full = ref["accepted_len"] == b.spec_lens
    assert (ref["n_emitted"][full & (t_lens == b.spec_lens)] == b.spec_lens[full & (t_lens == b.spec_lens)]).all()


def test_degenerate_rows(fsr, oracle):
    """Zero residual (p == q on the rejected row cannot happen, but p <= q everywhere can't either);
    exercise: one-hot target, one-hot draft with p(x)=0, zero-probability tails, u = 0."""
    announce("accept degenerate")
    V, B = 4500, 6
    rng = np.random.default_rng(4)
    spec = np.ones(B, np.int32)
    cu_d = workloads.exclusive_offsets(spec)
    cu_t = workloads.exclusive_offsets(spec + 1)
    p = workloads.softmax_rows_f32(rng.standard_normal((2 * B, V)).astype(np.float32) * 2)
    q = workloads.softmax_rows_f32(rng.standard_normal((B, V)).astype(np.float32) * 2)
    toks = rng.integers(0, V, size=B).astype(np.int32)
    p[0] = 0; p[0, 4321] = 1.0                      # one-hot target
    q[1] = 0; q[1, toks[1]] = 1.0; p[2, toks[1]] = 0  # one-hot draft; request 1 target row is row 2
    p[4, 3000:] = 0                                 # request 2: mass only in the first chunk
    p[6, :4096] = 0                                 # request 3: mass only in the last chunk
    q[3, :4096] = 0
    u_a = np.array([0.5, 0.0, 0.999, 0.5, 0.0, 0.25], np.float32)
    u_s = np.array([0.0, 0.999999, 0.5, 0.75, 0.0, 0.33], np.float32)
    ref = oracle.spec_accept(p, q, toks, u_a, u_s, cu_t, cu_d, S_max=1)
    gpu = fsr.spec_accept(dev(p), dev(q), dev(toks), dev(u_a), dev(u_s), dev(cu_t), dev(cu_d), S_max=1)
    torch.cuda.synchronize()
    frag, mism = check_accept(gpu, ref, u_s)
    assert mism == 0


@pytest.mark.parametrize("T", [1.0, 0.7])
def test_logits_mode(fsr, oracle, T):
    announce(f"accept LOGITS T={T}")
    b = workloads.make_batch(2, rep=5, with_kv=False, V=20011, B=12, spec_lens=[0, 1, 2, 3, 4, 5, 6, 7, 8, 2, 4, 1],
                             ctx_lens=[10] * 12, keep_logits=True)
    (frag, mism), ref = run_pair(fsr, oracle, b, mode=1, temperature=T)
    print(f"LOGITS T={T}: fragile={frag} mismatches={mism}")
    assert mism == 0


@pytest.mark.parametrize("draft_mode", ["independent", "noise", "equal"])
@pytest.mark.parametrize("T", [1.0, 0.8])
def test_logits_mode_with_enough_rows_for_two_passes(fsr, oracle, draft_mode, T):
    """A call with room for several thousand rows: the library normalises the rows of the first two drafts, tests them, and
    reads the later rows only of the requests still undecided.  Requests rejected at draft 0, 1, 2 and later, requests
    accepted whole, with 0, 1, 2 and 3 drafts, with and without a bonus row, and rows reached through maps."""
    announce(f"accept LOGITS two passes {draft_mode} T={T}")
    B = 189
    spec = np.array(([0, 1, 2, 3, 4, 5, 6, 7, 8] * 21), np.int32)
    b = workloads.make_batch(2, rep=11, with_kv=False, V=33001, B=B, spec_lens=spec.tolist(), ctx_lens=[10] * B,
                             keep_logits=True, draft_mode=draft_mode)
    (frag, mism), ref = run_pair(fsr, oracle, b, mode=1, temperature=T)
    assert mism == 0
    n = ref["accepted_len"]
    if draft_mode == "equal":
        assert np.array_equal(n, spec)
    else:
        assert {0, 1, 2} <= set(n[spec >= 4].tolist()) or draft_mode == "noise"
        assert (n[spec >= 4] >= 3).any() or draft_mode == "independent"
    # odd requests lose their bonus row; rows shuffled in storage
    rng = np.random.default_rng(1)
    perm_t, perm_d = rng.permutation(b.N), rng.permutation(b.N_d)
    z_t = np.empty_like(b.z_target); z_t[perm_t] = b.z_target
    z_d = np.empty_like(b.z_draft); z_d[perm_d] = b.z_draft
    toks = np.empty_like(b.draft_tokens); toks[perm_d] = b.draft_tokens
    u_a = np.empty_like(b.u_accept); u_a[perm_d] = b.u_accept
    t_lens = spec + 1 - (np.arange(B) % 2)
    t_lens[spec == 0] = 1
    cu_t = workloads.exclusive_offsets(t_lens)
    t_rows = np.concatenate([perm_t[b.cu_q[i]: b.cu_q[i] + t_lens[i]] for i in range(B)]).astype(np.int32)
    kw = dict(S_max=b.S_max, mode=1, temperature=T)
    ref = oracle.spec_accept(z_t, z_d, toks, u_a, b.u_sample, cu_t, b.cu_d, t_rows=t_rows, d_rows=perm_d.astype(np.int32), **kw)
    gpu = fsr.spec_accept(dev(z_t), dev(z_d), dev(toks), dev(u_a), dev(b.u_sample), dev(cu_t), dev(b.cu_d),
                          t_rows=dev(t_rows), d_rows=dev(perm_d.astype(np.int32)), **kw)
    torch.cuda.synchronize()
    frag, mism = check_accept(gpu, ref, b.u_sample)
    assert mism == 0


@pytest.mark.parametrize("B", [12, 189])
@pytest.mark.parametrize("T", [1.0, 0.05])
def test_logits_mode_masked_vocabulary_and_sharp_temperature(fsr, oracle, B, T):
    """Logits with half the vocabulary masked to -inf (the target's mask differs from the draft's, so some drafted
    tokens have target probability exactly 0 and must be rejected, and the residual is 0 wherever both are masked), at
    T = 1 and at a temperature that puts exp's argument hundreds below zero; one pass (B = 12) and two (B = 189)."""
    announce(f"accept LOGITS masked B={B} T={T}")
    spec = np.array(([0, 1, 2, 3, 4, 5, 6, 7, 8] * 21)[:B], np.int32)
    V = 20011
    b = workloads.make_batch(2, rep=13, with_kv=False, V=V, B=B, spec_lens=spec.tolist(), ctx_lens=[10] * B,
                             keep_logits=True, draft_mode="noise")
    rng = np.random.default_rng(5)
    z_t, z_d = b.z_target.copy(), b.z_draft.copy()
    mask_d = rng.random((b.N_d, V)) < 0.5
    mask_d[np.arange(b.N_d), b.draft_tokens] = False          # a drafted token has positive draft probability
    z_d[mask_d] = -np.inf
    mask_t = rng.random((b.N, V)) < 0.5
    mask_t[np.arange(b.N), rng.integers(0, V, b.N)] = False    # no target row is masked entirely
    z_t[mask_t] = -np.inf
    kw = dict(S_max=b.S_max, mode=1, temperature=T)
    ref = oracle.spec_accept(z_t, z_d, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, **kw)
    gpu = fsr.spec_accept(dev(z_t), dev(z_d), dev(b.draft_tokens), dev(b.u_accept), dev(b.u_sample), dev(b.cu_q),
                          dev(b.cu_d), **kw)
    torch.cuda.synchronize()
    frag, mism = check_accept(gpu, ref, b.u_sample)
    print(f"masked LOGITS B={B} T={T}: fragile={frag} mismatches={mism} accepted={ref['accepted_len'].sum()}/{b.N_d}")
    assert mism == 0
    # no emitted token is one the target masks at its position
    em, n = ref["emitted"], ref["accepted_len"]
    for i in range(B):
        for k in range(ref["n_emitted"][i]):
            assert not mask_t[b.cu_q[i] + k, em[i, k]]
    assert 0 < n.sum() < b.N_d


@pytest.mark.parametrize("mode", [0, 1])
def test_invalid_request_is_flagged_not_faulted(fsr, oracle, mode):
    announce(f"accept invalid request mode={mode}")
    b = workloads.make_batch(1, with_kv=False, keep_logits=bool(mode))
    d = DeviceBatch(b, kv=False, logits=bool(mode))
    rows_t, rows_d = (d.z_target, d.z_draft) if mode else (d.p_target, d.p_draft)
    acc, nem, em = fsr.spec_accept(rows_t, rows_d, d.draft_tokens, d.u_accept, d.u_sample, d.cu_q, d.cu_d,
                                   S_max=2, mode=mode)  # requests with 3 and 4 drafts exceed S_max
    torch.cuda.synchronize()
    acc = acc.cpu().numpy()
    assert (acc[b.spec_lens > 2] == -1).all() and (acc[b.spec_lens <= 2] >= 0).all()


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("V", [1000, 20011])
def test_bf16_rows(fsr, oracle, mode, V):
    """Probabilities / logits stored as bf16: same decisions as the oracle reading the same bits."""
    announce(f"accept bf16 rows mode={mode} V={V}")
    b = workloads.make_batch(2, rep=7, with_kv=False, V=V, B=12, spec_lens=[0, 1, 2, 3, 4, 5, 6, 7, 8, 2, 4, 1],
                             ctx_lens=[10] * 12, keep_logits=True)
    src_t, src_d = (b.z_target, b.z_draft) if mode else (b.p_target, b.p_draft)
    bits_t, bits_d = workloads.f32_to_bf16_bits(src_t), workloads.f32_to_bf16_bits(src_d)
    kw = dict(S_max=b.S_max, mode=mode, temperature=0.9)
    ref = oracle.spec_accept(bits_t, bits_d, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, dtype="bf16", **kw)
    gpu = fsr.spec_accept(dev(bits_t, True), dev(bits_d, True), dev(b.draft_tokens), dev(b.u_accept), dev(b.u_sample),
                          dev(b.cu_q), dev(b.cu_d), **kw)
    torch.cuda.synchronize()
    frag, mism = check_accept(gpu, ref, b.u_sample)
    print(f"bf16 rows mode={mode} V={V}: fragile={frag} mismatches={mism}")
    assert mism == 0
    assert 0 < ref["accepted_len"].sum() < b.N_d
