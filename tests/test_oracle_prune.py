"""Pins of the compaction oracle (Sec. 3.2 pruning, Sec. 3.3 discard beyond the rejection point)."""
import numpy as np
import pytest

import workloads


def py_reference(keep, cu, suffix_close):
    B = len(cu) - 1
    new_len, src = [], []
    for i in range(B):
        seg = [int(k != 0) for k in keep[cu[i]: cu[i + 1]]]
        if suffix_close:
            n = 0
            while n < len(seg) and seg[n]:
                n += 1
            rows = list(range(cu[i], cu[i] + n))
        else:
            rows = [cu[i] + j for j, k in enumerate(seg) if k]
        new_len.append(len(rows))
        src += rows
    return new_len, src


@pytest.mark.parametrize("suffix_close", [True, False])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_python_loops(oracle, suffix_close, seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 40))
    lens = rng.integers(0, 9, size=B)
    cu = workloads.exclusive_offsets(lens)
    N = int(cu[-1])
    keep = (rng.random(N) < 0.7).astype(np.uint8) * rng.integers(1, 255, size=N).astype(np.uint8)
    pay = rng.integers(0, 1 << 30, size=(N, 5)).astype(np.int32)
    r = oracle.prune_compact(keep, cu, suffix_close=suffix_close, payload=pay)
    new_len, src = py_reference(keep, cu, suffix_close)
    assert list(r["new_q_lens"]) == new_len
    assert list(r["new_cu_q"]) == [0] + list(np.cumsum(new_len))
    n_new = len(src)
    assert list(r["src_row"][:n_new]) == src and (r["src_row"][n_new:] == -1).all()
    dst = np.full(N, -1)
    dst[src] = np.arange(n_new)
    assert np.array_equal(r["dst_row"], dst)
    act = [i for i in range(B) if new_len[i] > 0]
    assert r["n_active"] == len(act) and list(r["active_ids"][: len(act)]) == act
    assert (r["active_ids"][len(act):] == -1).all()
    assert np.array_equal(r["payload"], pay[src])
    # restore(compact(x)) = x on kept rows, pad elsewhere
    back, has = oracle.prune_restore(r["payload"], r["dst_row"], pad_byte=0xFF)
    assert np.array_equal(has.astype(bool), dst >= 0)
    assert np.array_equal(back[dst >= 0], pay[dst >= 0])
    assert (back[dst < 0] == -1).all()


def test_identities(oracle):
    lens = np.array([3, 0, 4, 1, 2])
    cu = workloads.exclusive_offsets(lens)
    N = int(cu[-1])
    r = oracle.prune_compact(np.ones(N, np.uint8), cu)
    assert np.array_equal(r["new_cu_q"], cu) and np.array_equal(r["src_row"], np.arange(N))
    assert np.array_equal(r["dst_row"], np.arange(N)) and r["n_active"] == 4
    assert list(r["active_ids"]) == [0, 2, 3, 4, -1]
    r = oracle.prune_compact(np.zeros(N, np.uint8), cu)
    assert (r["new_cu_q"] == 0).all() and r["n_active"] == 0 and (r["dst_row"] == -1).all()
    # suffix closure: 1,0,1 keeps one row; without closure two
    r = oracle.prune_compact(np.array([1, 0, 1], np.uint8), np.array([0, 3], np.int32))
    assert r["new_q_lens"][0] == 1 and list(r["dst_row"]) == [0, -1, -1]
    r = oracle.prune_compact(np.array([1, 0, 1], np.uint8), np.array([0, 3], np.int32), suffix_close=False)
    assert r["new_q_lens"][0] == 2 and list(r["dst_row"]) == [0, -1, 1]
    # empty batch
    r = oracle.prune_compact(np.zeros(0, np.uint8), np.array([0], np.int32))
    assert list(r["new_cu_q"]) == [0] and r["n_active"] == 0


def test_figure_shapes_fixture(oracle):
    """Fig. 5 shape: 3 requests x 3 drafts; prune the rejected suffix of two of them."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "figure_shapes.txt")
    rows = [l.split("|") for l in open(path) if l.strip() and not l.startswith("#")]
    shapes = {r[0].strip(): [int(x) for x in r[1].split(",")] for r in rows}
    spec = np.array(shapes["early_exit_workflow"])
    cu = workloads.exclusive_offsets(spec + 1)          # 4 rows per request
    keep = np.ones(int(cu[-1]), np.uint8)
    keep[cu[0] + 2:cu[1]] = 0                           # request 0: suffix from row 2 pruned
    keep[cu[2] + 1:cu[3]] = 0                           # request 2: suffix from row 1 pruned
    r = oracle.prune_compact(keep, cu)
    assert list(r["new_q_lens"]) == [2, 4, 1] and int(r["new_cu_q"][-1]) == 7
    x = np.arange(12, dtype=np.float32)[:, None] * np.ones((1, 3), np.float32)
    back, has = oracle.prune_restore(x[r["src_row"][:7]], r["dst_row"])
    assert list(has) == [1, 1, 0, 0, 1, 1, 1, 1, 1, 0, 0, 0]
