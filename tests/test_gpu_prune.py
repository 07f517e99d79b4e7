"""GPU parity: prune_compact / prune_restore / prune_scatter vs the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import announce, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def _compare(fsr, oracle, keep, cu, suffix_close, pay, N_cap):
    ref = oracle.prune_compact(keep[: int(cu[-1])], cu, suffix_close=suffix_close, payload=pay[: int(cu[-1])])
    keep_d = dev(keep)
    r = fsr.prune_compact(keep_d, dev(cu), suffix_close=suffix_close, payload=dev(pay))
    torch.cuda.synchronize()
    N = int(cu[-1])
    n_new = int(ref["new_cu_q"][-1])
    assert np.array_equal(r["new_cu_q"].cpu().numpy(), ref["new_cu_q"])
    assert np.array_equal(r["new_q_lens"].cpu().numpy(), ref["new_q_lens"])
    src = r["src_row"].cpu().numpy()
    dst = r["dst_row"].cpu().numpy()
    assert np.array_equal(src[:N], ref["src_row"]) and (src[N:] == -1).all()
    assert np.array_equal(dst[:N], ref["dst_row"]) and (dst[N:] == -1).all()
    assert int(r["n_active"].item()) == ref["n_active"]
    assert np.array_equal(r["active_ids"].cpu().numpy(), ref["active_ids"])
    assert np.array_equal(r["payload"].cpu().numpy()[:n_new], ref["payload"])
    # restore and scatter
    back_ref, has_ref = oracle.prune_restore(ref["payload"], ref["dst_row"], pad_byte=0xAB)
    back, has = fsr.prune_restore(r["payload"], r["dst_row"], pad_word=0xABABABAB)
    torch.cuda.synchronize()
    assert np.array_equal(has.cpu().numpy()[:N], has_ref)
    assert np.array_equal(back.cpu().numpy()[:N], back_ref)
    base = torch.full_like(r["payload"], -7)
    fsr.prune_scatter(r["payload"], r["src_row"], r["new_cu_q"][len(cu) - 1:], base)
    torch.cuda.synchronize()
    exp = np.full_like(pay, -7)
    exp[ref["src_row"][:n_new]] = ref["payload"]
    assert np.array_equal(base.cpu().numpy(), exp)


@pytest.mark.parametrize("suffix_close", [True, False])
@pytest.mark.parametrize("seed,B,maxlen,width", [(0, 1, 5, 4), (1, 37, 9, 6), (2, 512, 11, 64), (3, 2500, 4, 3), (4, 300, 0, 4)])
def test_prune_random(fsr, oracle, suffix_close, seed, B, maxlen, width):
    announce(f"prune_random seed={seed} B={B} suffix_close={suffix_close}")
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, maxlen + 1, size=B)
    cu = workloads.exclusive_offsets(lens)
    N = int(cu[-1])
    N_cap = N + 5
    keep = ((rng.random(N_cap) < 0.75) * rng.integers(1, 255, size=N_cap)).astype(np.uint8)
    pay = rng.integers(-1000, 1000, size=(N_cap, width)).astype(np.int32)
    _compare(fsr, oracle, keep, cu, suffix_close, pay, N_cap)


def test_prune_all_keep_all_drop_and_figure_shape(fsr, oracle):
    announce("prune identities")
    cu = workloads.exclusive_offsets(np.array([4, 4, 4]))
    pay = np.arange(12 * 8, dtype=np.int32).reshape(12, 8)
    for keep in (np.ones(12, np.uint8), np.zeros(12, np.uint8),
                 np.array([1, 1, 0, 0, 1, 1, 1, 1, 1, 0, 0, 0], np.uint8)):
        _compare(fsr, oracle, keep, cu, True, pay, 12)


def test_prune_wide_rows_16B_path(fsr, oracle):
    announce("prune wide bf16-like rows")
    rng = np.random.default_rng(9)
    lens = rng.integers(1, 10, size=64)
    cu = workloads.exclusive_offsets(lens)
    N = int(cu[-1])
    keep = (rng.random(N) < 0.6).astype(np.uint8)
    pay = rng.integers(-2**31, 2**31 - 1, size=(N, 2048), dtype=np.int64).astype(np.int32)  # 8 KB rows
    _compare(fsr, oracle, keep, cu, True, pay, N)


@pytest.mark.parametrize("seed,B,maxlen", [(0, 1, 5), (1, 37, 9), (2, 700, 11), (3, 2500, 4)])
def test_survivor_compact_equals_mask_then_compact(fsr, oracle, seed, B, maxlen):
    """The one-call form (accepted lengths in, re-packed batch out) against the oracle's mask + compaction and
    against the two separate calls, bit for bit; invalid requests (accepted_len = -1) keep nothing."""
    announce(f"survivor_compact seed={seed} B={B}")
    rng = np.random.default_rng(100 + seed)
    lens = rng.integers(0, maxlen + 1, size=B)
    cu = workloads.exclusive_offsets(lens)
    N = int(cu[-1])
    N_cap = N + 3
    acc = rng.integers(-1, maxlen + 2, size=B).astype(np.int32)      # some beyond the request's rows, some -1
    pay = rng.integers(-1000, 1000, size=(N_cap, 8)).astype(np.int32)
    keep_ref = np.concatenate([np.arange(l) <= a for l, a in zip(lens, acc)] + [np.zeros(0, bool)]).astype(np.uint8)
    ref = oracle.prune_compact(keep_ref, cu, suffix_close=True, payload=pay[:N])
    keep_d = torch.full((N_cap,), 9, dtype=torch.uint8, device="cuda")
    r = fsr.survivor_compact(dev(acc), dev(cu), N_cap, keep_mask=keep_d, payload=dev(pay))
    keep2 = torch.full((N_cap,), 9, dtype=torch.uint8, device="cuda")
    fsr.survivor_mask(dev(acc), dev(cu), keep2)
    r2 = fsr.prune_compact(keep2, dev(cu), suffix_close=True, payload=dev(pay))
    torch.cuda.synchronize()
    n_new = int(ref["new_cu_q"][-1])
    assert np.array_equal(keep_d.cpu().numpy()[:N], keep_ref) and (keep_d.cpu().numpy()[N:] == 9).all()
    assert torch.equal(keep_d, keep2)
    for name in ("new_cu_q", "new_q_lens", "src_row", "dst_row", "n_active", "active_ids"):
        assert torch.equal(r[name], r2[name]), name
    assert np.array_equal(r["new_cu_q"].cpu().numpy(), ref["new_cu_q"])
    assert np.array_equal(r["src_row"].cpu().numpy()[:N], ref["src_row"])
    assert np.array_equal(r["dst_row"].cpu().numpy()[:N], ref["dst_row"])
    assert np.array_equal(r["payload"].cpu().numpy()[:n_new], ref["payload"])
    # without the optional mask output
    r3 = fsr.survivor_compact(dev(acc), dev(cu), N_cap)
    torch.cuda.synchronize()
    assert torch.equal(r3["src_row"], r["src_row"])
