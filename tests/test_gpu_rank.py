"""GPU parity: the early-exit rank check (Sec. 3.2 / Sec. 4) through the C ABI vs the oracle,
bit-exact (integer work), and its composition with compaction, attention on the surviving rows
and the restore to the original layout."""
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


def _compare(fsr, oracle, z_host, toks, cu_q, cu_d, K, dtype):
    z_dev = dev(z_host, bf16=(dtype == "bf16"))
    rank, keep = fsr.topk_rank_check(z_dev, dev(toks), dev(cu_q), dev(cu_d), K=K)
    torch.cuda.synchronize()
    ref = oracle.topk_rank_check(z_host, toks, cu_q, cu_d, K=K, dtype=dtype)
    n_d, n = int(cu_d[-1]), int(cu_q[-1])
    assert np.array_equal(rank.cpu().numpy()[:n_d], ref["rank"])
    assert np.array_equal(keep.cpu().numpy()[:n], ref["keep"])
    return ref


@pytest.mark.parametrize("K", [0, 1, 10])
def test_config1_tiny(fsr, oracle, K):
    announce(f"rank check config1 K={K}")
    b = workloads.make_batch(1, rep=5, keep_logits=True)
    _compare(fsr, oracle, b.z_target, b.draft_tokens, b.cu_q, b.cu_d, K, "f32")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1, 7, 1000, 8191, 8193, 20001])
def test_ragged_vocab_misaligned_rows_and_ties(fsr, oracle, V, dtype):
    """Row starts that are not 16-byte aligned (odd V), chunk tails, and coarse scores with many ties."""
    announce(f"rank check V={V} dtype={dtype}")
    rng = np.random.default_rng(V)
    spec = np.array([3, 0, 5, 1, 8], np.int32)
    cu_q, cu_d = workloads.exclusive_offsets(spec + 1), workloads.exclusive_offsets(spec)
    N = int(cu_q[-1])
    z = (rng.integers(-40, 41, size=(N, V)) * 0.125).astype(np.float32)
    toks = rng.integers(0, V, size=int(cu_d[-1])).astype(np.int32)
    zh = z if dtype == "f32" else workloads.f32_to_bf16_bits(z)
    for K in (1, 10):
        _compare(fsr, oracle, zh, toks, cu_q, cu_d, K, dtype)


def test_compacted_layout_capacity_slack_and_invalid_tokens(fsr, oracle):
    announce("rank check on a compacted layout with slack rows and out-of-range ids")
    rng = np.random.default_rng(9)
    V = 3001
    spec = np.array([4, 3, 0, 2, 6], np.int32)
    q_lens = np.array([2, 4, 1, 0, 7], np.int32)
    cu_q, cu_d = workloads.exclusive_offsets(q_lens), workloads.exclusive_offsets(spec)
    N, N_d = int(cu_q[-1]), int(cu_d[-1])
    z = rng.standard_normal((N + 3, V)).astype(np.float32)          # 3 slack rows
    toks = np.concatenate([rng.integers(0, V, size=N_d), [5, 5]]).astype(np.int32)  # 2 slack drafts
    toks[cu_d[1] + 1] = V + 3
    toks[cu_d[4]] = -2
    rank, keep = fsr.topk_rank_check(dev(z), dev(toks), dev(cu_q), dev(cu_d), K=10,
                                     rank=torch.full((N_d + 2,), 77, dtype=torch.int32, device="cuda"),
                                     keep_mask=torch.full((N + 3,), 9, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    ref = oracle.topk_rank_check(z[:N], toks[:N_d], cu_q, cu_d, K=10)
    assert np.array_equal(rank.cpu().numpy()[:N_d], ref["rank"]) and (rank.cpu().numpy()[N_d:] == 77).all()
    assert np.array_equal(keep.cpu().numpy()[:N], ref["keep"]) and (keep.cpu().numpy()[N:] == 9).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_config2_full_vocab(fsr, oracle, dtype):
    announce(f"rank check config2 full vocabulary dtype={dtype}")
    b = workloads.make_batch(2, rep=1, with_kv=False, keep_logits=True)
    z = b.z_target if dtype == "f32" else workloads.f32_to_bf16_bits(b.z_target)
    ref = _compare(fsr, oracle, z, b.draft_tokens, b.cu_q, b.cu_d, 10, dtype)
    print(f"config2 {dtype}: {int((ref['rank'] < 10).sum())} of {len(ref['rank'])} drafts inside the top 10")


def test_check_compact_attend_restore(fsr, oracle):
    """The early-exit flow of Sec. 3.2: rank check on intermediate scores -> compaction of the query
    rows -> attention on the surviving rows only -> restore to the original layout.  Surviving rows
    carry the values full attention gives them; pruned rows carry none."""
    announce("rank check -> compact -> attention -> restore")
    ctx = [300, 45, 513, 128, 1000, 77, 2048]
    spec = [8, 3, 6, 0, 2, 5, 7]
    b = workloads.make_batch(2, rep=13, V=5000, ctx_lens=ctx, spec_lens=spec, keep_logits=True)
    d = DeviceBatch(b)
    K = 3
    rank, keep = fsr.topk_rank_check(dev(b.z_target), d.draft_tokens, d.cu_q, d.cu_d, K=K)
    pr = fsr.prune_compact(keep, d.cu_q, suffix_close=True, payload=d.q)
    out_c, _ = fsr.verify_attention(pr["payload"], d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens,
                                    pr["new_cu_q"], scale=b.scale, out_dtype=torch.float32, max_q_len=b.S_max + 1)
    restored, has = fsr.prune_restore(out_c, pr["dst_row"])
    torch.cuda.synchronize()
    ref = oracle.topk_rank_check(b.z_target, b.draft_tokens, b.cu_q, b.cu_d, K=K)
    pc = oracle.prune_compact(ref["keep"], b.cu_q, suffix_close=True)
    has_ref = (pc["dst_row"] >= 0).astype(np.uint8)
    assert np.array_equal(has.cpu().numpy(), has_ref)
    assert 0 < has_ref.sum() < b.N
    o_ref, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                       H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    rows = np.where(has_ref == 1)[0]
    check_attention(restored[torch.from_numpy(rows).cuda()], o_ref[rows], b.dtype, len(rows))
    assert not restored[torch.from_numpy(np.where(has_ref == 0)[0]).cuda()].any()
