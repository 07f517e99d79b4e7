"""GPU parity: the greedy (temperature 0) mode of fsr_spec_accept vs the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import announce, chunked_case, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def _plant_runs(b, z):
    """Make leading runs of drafts equal to the target's arg-max so that accepted lengths vary."""
    for i in range(b.B):
        for j in range(max(int(b.spec_lens[i]) - (i % 4), 0)):
            b.draft_tokens[b.cu_d[i] + j] = int(np.argmax(z[b.cu_q[i] + j]))


def _compare(fsr, oracle, z, toks, cu_t, cu_d, S_max, **maps):
    B = len(cu_t) - 1
    kw = {k: dev(v) for k, v in maps.items()}
    acc, nem, em = fsr.spec_accept(dev(z), None, dev(toks), None, None, dev(cu_t), dev(cu_d), S_max=S_max,
                                   mode=2, **kw)
    torch.cuda.synchronize()
    ref = oracle.greedy_accept(z, toks, cu_t, cu_d, S_max=S_max, **maps)
    assert np.array_equal(acc.cpu().numpy(), ref["accepted_len"])
    assert np.array_equal(nem.cpu().numpy(), ref["n_emitted"])
    assert np.array_equal(em.cpu().numpy(), ref["emitted"])
    return ref


@pytest.mark.parametrize("V", [1, 5, 1000, 4095, 4097, 20001])
def test_vocab_sizes_ties_and_misaligned_rows(fsr, oracle, V):
    announce(f"greedy accept V={V}")
    rng = np.random.default_rng(V)
    spec = np.array([0, 1, 4, 8, 3, 6, 2], np.int32)
    cu_t, cu_d = workloads.exclusive_offsets(spec + 1), workloads.exclusive_offsets(spec)
    z = (rng.integers(-6, 7, size=(int(cu_t[-1]), V)) * 0.25).astype(np.float32)   # coarse: many tied maxima
    z[1] = -0.0
    z[1, V // 2] = 0.0                                                              # -0 and +0 are equal
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    for i, s in enumerate(spec):
        for j in range(max(int(s) - (i % 3), 0)):
            toks[cu_d[i] + j] = int(np.argmax(z[cu_t[i] + j]))
    ref = _compare(fsr, oracle, z, toks, cu_t, cu_d, 8)
    if V > 1:
        assert (ref["accepted_len"] < spec).any()


def test_nan_scores_count_as_minus_infinity(fsr, oracle):
    """NaN scores never win the arg-max (they count as -inf; ties to the lowest id), on rows long enough to span
    several workgroups with the NaNs in different chunks."""
    announce("greedy accept with NaN scores")
    rng = np.random.default_rng(77)
    V = 9001
    spec = np.array([3, 0, 2, 5, 1], np.int32)
    cu_t, cu_d = workloads.exclusive_offsets(spec + 1), workloads.exclusive_offsets(spec)
    z = rng.standard_normal((int(cu_t[-1]), V)).astype(np.float32)
    z[rng.random(z.shape) < 0.05] = np.nan
    z[0, 0] = np.nan                      # a NaN in front of the row
    z[1] = np.nan                         # a row of NaN alone -> token 0
    z[2] = -np.inf
    z[2, ::3] = np.nan                    # NaN and -inf tie -> lowest id
    z[3, :4500] = np.nan                  # whole first chunk NaN
    z[4, 5000] = np.inf
    z[4, 7000] = np.nan
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    clean = np.where(np.isnan(z), -np.inf, z)
    for i, s in enumerate(spec):
        for j in range(max(int(s) - (i % 2), 0)):
            toks[cu_d[i] + j] = int(np.argmax(clean[cu_t[i] + j]))
    ref = _compare(fsr, oracle, z, toks, cu_t, cu_d, 5)
    # request 1 has no drafts: its only row is row 4, whose maximum is the +inf at 5000 (the NaN at 7000 loses)
    assert ref["emitted"][1, 0] == 5000 and ref["accepted_len"].sum() > 0


def test_config2_full_vocab_and_row_maps(fsr, oracle):
    announce("greedy accept config2 full vocabulary, with row maps")
    b = workloads.make_batch(2, rep=2, with_kv=False, keep_logits=True)
    _plant_runs(b, b.z_target)
    ref = _compare(fsr, oracle, b.z_target, b.draft_tokens, b.cu_q, b.cu_d, b.S_max)
    print(f"greedy cfg2: accepted {int(ref['accepted_len'].sum())} of {b.N_d}")
    perm = np.random.default_rng(1).permutation(b.N).astype(np.int32)
    inv = np.argsort(perm).astype(np.int32)
    dperm = np.random.default_rng(2).permutation(b.N_d).astype(np.int32)
    dinv = np.argsort(dperm).astype(np.int32)
    _compare(fsr, oracle, b.z_target[perm], b.draft_tokens[dperm], b.cu_q, b.cu_d, b.S_max, t_rows=inv, d_rows=dinv)


def test_no_bonus_rows_and_invalid_request(fsr, oracle):
    announce("greedy accept without bonus rows; an inconsistent request is flagged")
    rng = np.random.default_rng(4)
    V = 300
    spec = np.array([2, 3, 0, 4], np.int32)
    cu_d = workloads.exclusive_offsets(spec)
    cu_t = cu_d.copy()                                  # no bonus rows at all
    z = rng.standard_normal((max(int(cu_t[-1]), 1), V)).astype(np.float32)
    toks = np.array([int(np.argmax(z[r])) for r in range(int(cu_d[-1]))], np.int32)
    toks[cu_d[1] + 1] = (toks[cu_d[1] + 1] + 1) % V
    ref = _compare(fsr, oracle, z, toks, cu_t, cu_d, 4)
    assert list(ref["n_emitted"]) == [2, 2, 0, 4]
    bad_cu_t = cu_t.copy()
    bad_cu_t[2:] += 3                                   # request 1 now has 3 more target rows than drafts
    zz = rng.standard_normal((int(bad_cu_t[-1]), V)).astype(np.float32)
    acc, nem, em = fsr.spec_accept(dev(zz), None, dev(toks), None, None, dev(bad_cu_t), dev(cu_d), S_max=4,
                                   mode=2)
    torch.cuda.synchronize()
    assert acc.cpu().numpy()[1] == -1 and nem.cpu().numpy()[1] == -1 and (em.cpu().numpy()[1] == -1).all()


def test_chunked_greedy_matches_oracle_and_one_shot(fsr, oracle):
    announce("chunked verification in greedy mode")
    spec = [0, 1, 2, 3, 4, 5, 6, 7, 8, 2, 4, 6, 3, 8]
    ctx = [40, 33, 17, 64, 200, 31, 47, 16, 25, 50, 61, 19, 333, 90]
    b = workloads.make_batch(5, rep=6, V=3000, spec_lens=spec, ctx_lens=ctx, keep_logits=True)
    _plant_runs(b, b.z_target)
    b.p_target = b.z_target
    chunks = workloads.chunk_plan(5, b.spec_lens, s_c=2)
    chunked_case(fsr, oracle, b, chunks, b.dtype, mode="greedy")
