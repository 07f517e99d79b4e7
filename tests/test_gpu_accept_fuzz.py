"""GPU parity: spec_accept in LOGITS mode on seeded random cases -- batch sizes on both sides of the two-pass limit,
suffix bounds 1..12, vocabularies with and without a ragged end and spanning one or several statistic groups, four
temperatures, three kinds of drafts, fp32 and bf16 rows, -inf masks, requests without their bonus row, and rows
reached through shuffled maps -- against the oracle, to the same bar as the other accept tests."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import announce, check_accept, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


@pytest.mark.parametrize("case", range(20))
def test_logits_mode_random_case(fsr, oracle, case):
    rng = np.random.default_rng(7000 + case)
    S_max = int(rng.integers(1, 13))
    big = case % 2 == 0
    lim = 3072 // (2 * S_max + 1)
    B = int(rng.integers(lim + 1, lim + 150)) if big else int(rng.integers(1, 40))
    V = int(rng.choice([257, 1000, 4096, 4097, 9001] if big else [257, 4097, 9001, 33001, 70001]))
    T = float(rng.choice([1.0, 0.7, 0.2, 1.8]))
    mode = str(rng.choice(["noise", "independent", "equal"]))
    bf16 = bool(rng.random() < 0.3)
    masked = bool(rng.random() < 0.4)
    announce(f"accept LOGITS random case {case}: B={B} S_max={S_max} V={V} T={T} {mode} bf16={bf16} masked={masked}")
    spec = rng.integers(0, S_max + 1, B).astype(np.int32)
    spec[rng.integers(0, B)] = S_max
    b = workloads.make_batch(2, rep=1000 + case, with_kv=False, V=V, B=B, spec_lens=spec.tolist(), ctx_lens=[10] * B,
                             keep_logits=True, draft_mode=mode)
    z_t, z_d = b.z_target, b.z_draft
    if masked:
        m = rng.random(z_t.shape) < 0.3
        m[np.arange(b.N), rng.integers(0, V, b.N)] = False       # no row is masked entirely
        z_t = z_t.copy(); z_t[m] = -np.inf
        m = rng.random(z_d.shape) < 0.3
        m[np.arange(b.N_d), b.draft_tokens] = False               # a drafted token has positive draft probability
        z_d = z_d.copy(); z_d[m] = -np.inf
    t_lens = (spec + 1 - (rng.random(B) < 0.3)).astype(np.int32)  # some requests come without their bonus row
    t_lens[spec == 0] = 1
    perm_t, perm_d = rng.permutation(b.N), rng.permutation(b.N_d)
    zt = np.empty_like(z_t); zt[perm_t] = z_t
    zd = np.empty_like(z_d); zd[perm_d] = z_d
    toks = np.empty_like(b.draft_tokens); toks[perm_d] = b.draft_tokens
    ua = np.empty_like(b.u_accept); ua[perm_d] = b.u_accept
    cu_t = workloads.exclusive_offsets(t_lens)
    t_rows = np.concatenate([perm_t[b.cu_q[i]: b.cu_q[i] + t_lens[i]] for i in range(B)]).astype(np.int32)
    d_rows = perm_d.astype(np.int32)
    kw = dict(S_max=S_max, mode=1, temperature=T)
    if bf16:
        zt, zd = workloads.f32_to_bf16_bits(zt), workloads.f32_to_bf16_bits(zd)
    ref = oracle.spec_accept(zt, zd, toks, ua, b.u_sample, cu_t, b.cu_d, t_rows=t_rows, d_rows=d_rows,
                             dtype="bf16" if bf16 else "f32", **kw)
    gpu = fsr.spec_accept(dev(zt, bf16), dev(zd, bf16), dev(toks), dev(ua), dev(b.u_sample), dev(cu_t), dev(b.cu_d),
                          t_rows=dev(t_rows), d_rows=dev(d_rows), **kw)
    torch.cuda.synchronize()
    frag, mism = check_accept(gpu, ref, b.u_sample)
    assert mism == 0
