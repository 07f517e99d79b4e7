"""CPU oracle of the verification hot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It shares no code with the HIP library and never imports it.

The arithmetic lives in ``faser_oracle.c`` (plain C, fp64, one loop per sum); this module
compiles it with gcc, marshals numpy arrays, and spells out the chunked (frontier)
verification schedule of Sec. 3.3 of the paper in python loops on top of the C steps.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "faser_oracle.c")
_LIB = os.path.join(_HERE, "libfaser_oracle.so")
_lib = None

F32, BF16, F64 = 0, 1, 2
PROBS, LOGITS, GREEDY = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent outputs only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def n_threads() -> int:
    """Host threads the oracle's OpenMP loops use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return int(env.split(",")[0])
        except ValueError:
            pass
    return os.cpu_count() or 1


def verify_attention(q, k_cache, v_cache, block_tables, ctx_lens, cu_q, *, H_q, H_kv, D, P, dtype, scale,
                     token_major=False):
    """Sec. 2.1 verification attention over the paged cache; returns (out[N,H_q,D], lse[N,H_q]) in fp64.
    Caches are [n_pages, H_kv, P, D]; with token_major they are [n_pages, P, H_kv, D], which is the same
    cache with two axes swapped and is handled as exactly that."""
    lib = _load()
    if token_major:
        k_cache, v_cache = np.swapaxes(k_cache, 1, 2), np.swapaxes(v_cache, 1, 2)
    code = BF16 if dtype == "bf16" else F32
    st = np.uint16 if code == BF16 else np.float32
    q, k_cache, v_cache = _c(q, st), _c(k_cache, st), _c(v_cache, st)
    bt, ctx, cu = _c(block_tables, np.int32), _c(ctx_lens, np.int32), _c(cu_q, np.int32)
    B = len(ctx)
    N = int(cu[-1])
    out = np.zeros((N, H_q, D), dtype=np.float64)
    lse = np.zeros((N, H_q), dtype=np.float64)
    rc = lib.fo_verify_attention(_p(q), _p(k_cache), _p(v_cache), _p(bt), _p(ctx), _p(cu), _p(out), _p(lse),
                                 ctypes.c_int(B), ctypes.c_int(H_q), ctypes.c_int(H_kv), ctypes.c_int(D),
                                 ctypes.c_int(P), ctypes.c_int(bt.shape[1]), ctypes.c_int(code),
                                 ctypes.c_double(scale))
    if rc != 0:
        raise ValueError(f"fo_verify_attention: {rc}")
    return out, lse


def decode_e4m3(codes):
    """Values of OCP E4M3 bytes as fp64 (NaN for the two NaN codes)."""
    lib = _load()
    codes = _c(codes, np.uint8)
    out = np.empty(codes.shape, dtype=np.float64)
    lib.fo_decode_e4m3(_p(codes), _p(out), ctypes.c_int64(codes.size))
    return out


def encode_e4m3(x):
    """E4M3 bytes of fp32 values: nearest, ties to the even code, saturating at 448."""
    lib = _load()
    x = _c(x, np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    lib.fo_encode_e4m3(_p(x), _p(out), ctypes.c_int64(x.size))
    return out


def kv_append_kv8(k_new_bits, v_new_bits, k_cache8, v_cache8, k_scale, v_scale, block_tables, ctx_lens, cu_q, *, P,
                  token_major=False):
    """Cache append into 8-bit caches: a bf16 key element x of KV head g is stored as the E4M3 byte of
    fl32(x / k_scale[g]) (one fp32 division, then one rounding to 8 bits), values likewise; then the bytes go
    where fo_kv_append puts them.  Returns the updated (k_cache8, v_cache8)."""
    def quantise(bits, scale):
        x = (_c(bits, np.uint16).astype(np.uint32) << 16).view(np.float32)
        y = (x / np.asarray(scale, dtype=np.float32).reshape(1, -1, 1)).astype(np.float32)
        return encode_e4m3(y)
    return kv_append(quantise(k_new_bits, k_scale), quantise(v_new_bits, v_scale), k_cache8, v_cache8, block_tables,
                     ctx_lens, cu_q, P=P, token_major=token_major)


def verify_attention_kv8(q_bits, k_cache8, v_cache8, k_scale, v_scale, block_tables, ctx_lens, cu_q, *, H_q, H_kv, D, P,
                         scale, token_major=False):
    """The same attention with the caches stored as E4M3 bytes: cached key = decode(byte) * k_scale[kv head],
    cached value = decode(byte) * v_scale[kv head]; queries are bf16 bit patterns.  Everything is widened to
    fp64 first (exactly), then the plain definition runs."""
    lib = _load()
    if token_major:
        k_cache8, v_cache8 = np.swapaxes(k_cache8, 1, 2), np.swapaxes(v_cache8, 1, 2)
    ks = np.asarray(k_scale, dtype=np.float32).astype(np.float64).reshape(1, H_kv, 1, 1)
    vs = np.asarray(v_scale, dtype=np.float32).astype(np.float64).reshape(1, H_kv, 1, 1)
    k = _c(decode_e4m3(k_cache8) * ks, np.float64)
    v = _c(decode_e4m3(v_cache8) * vs, np.float64)
    qb = _c(q_bits, np.uint16)
    q = _c((qb.astype(np.uint32) << 16).view(np.float32).astype(np.float64), np.float64)
    bt, ctx, cu = _c(block_tables, np.int32), _c(ctx_lens, np.int32), _c(cu_q, np.int32)
    N = int(cu[-1])
    out = np.zeros((N, H_q, D), dtype=np.float64)
    lse = np.zeros((N, H_q), dtype=np.float64)
    rc = lib.fo_verify_attention(_p(q), _p(k), _p(v), _p(bt), _p(ctx), _p(cu), _p(out), _p(lse),
                                 ctypes.c_int(len(ctx)), ctypes.c_int(H_q), ctypes.c_int(H_kv), ctypes.c_int(D),
                                 ctypes.c_int(P), ctypes.c_int(bt.shape[1]), ctypes.c_int(F64), ctypes.c_double(scale))
    if rc != 0:
        raise ValueError(f"fo_verify_attention: {rc}")
    return out, lse


def spec_accept(p_target, p_draft, draft_tokens, u_accept, u_sample, cu_t, cu_d, *, S_max,
                t_rows=None, d_rows=None, mode=PROBS, temperature=1.0, dtype="f32"):
    """Sec. 2.1 accept-until-first-mismatch with recovery/bonus token.

    Returns dict(accepted_len[B], n_emitted[B], emitted[B,S_max+1], cdf_lo[B], cdf_hi[B], tok_below[B],
    tok_above[B]): the last four describe the drawn token's place in the row it was drawn from (its CDF
    interval, and the nearest positive-mass token ids on either side, -1 if none).
    """
    if mode == GREEDY:
        return greedy_accept(p_target, draft_tokens, cu_t, cu_d, S_max=S_max, t_rows=t_rows, d_rows=d_rows)
    lib = _load()
    row_t = np.float32 if dtype == "f32" else np.uint16  # bf16 rows come as bit patterns
    p_target, p_draft = _c(p_target, row_t), _c(p_draft, row_t)
    V = p_target.shape[1]
    toks, ua, us = _c(draft_tokens, np.int32), _c(u_accept, np.float32), _c(u_sample, np.float32)
    cu_t, cu_d = _c(cu_t, np.int32), _c(cu_d, np.int32)
    tr = None if t_rows is None else _c(t_rows, np.int32)
    dr = None if d_rows is None else _c(d_rows, np.int32)
    B = len(cu_t) - 1
    acc = np.zeros(B, np.int32)
    nem = np.zeros(B, np.int32)
    em = np.full((B, S_max + 1), -1, np.int32)
    lo = np.full(B, np.nan)
    hi = np.full(B, np.nan)
    below = np.full(B, -1, np.int32)
    above = np.full(B, -1, np.int32)
    rc = lib.fo_spec_accept(_p(p_target), _p(p_draft), _p(toks), _p(ua), _p(us), _p(cu_t), _p(cu_d), _p(tr), _p(dr),
                            _p(acc), _p(nem), _p(em), _p(lo), _p(hi), _p(below), _p(above), ctypes.c_int(B), ctypes.c_int(V),
                            ctypes.c_int(S_max), ctypes.c_int(mode), ctypes.c_double(temperature),
                            ctypes.c_int(F32 if dtype == "f32" else BF16))
    if rc != 0:
        raise ValueError(f"fo_spec_accept: {rc}")
    return dict(accepted_len=acc, n_emitted=nem, emitted=em, cdf_lo=lo, cdf_hi=hi, tok_below=below, tok_above=above)


def greedy_accept(target, draft_tokens, cu_t, cu_d, *, S_max, t_rows=None, d_rows=None):
    """Sec. 2.1 at temperature 0: drafts are accepted while they equal the target row's arg-max (lowest id
    among equal maxima); the next row's arg-max is the token after the accepted run.

    Returns dict(accepted_len[B], n_emitted[B], emitted[B,S_max+1], cdf_lo, cdf_hi) (the last two all NaN:
    nothing is drawn)."""
    lib = _load()
    z = _c(target, np.float32)
    V = z.shape[1]
    toks = _c(draft_tokens, np.int32)
    cu_t, cu_d = _c(cu_t, np.int32), _c(cu_d, np.int32)
    tr = None if t_rows is None else _c(t_rows, np.int32)
    dr = None if d_rows is None else _c(d_rows, np.int32)
    B = len(cu_t) - 1
    acc = np.zeros(B, np.int32)
    nem = np.zeros(B, np.int32)
    em = np.full((B, S_max + 1), -1, np.int32)
    rc = lib.fo_greedy_accept(_p(z), _p(toks), _p(cu_t), _p(cu_d), _p(tr), _p(dr), _p(acc), _p(nem), _p(em),
                              ctypes.c_int(B), ctypes.c_int(V), ctypes.c_int(S_max))
    if rc != 0:
        raise ValueError(f"fo_greedy_accept: {rc}")
    return dict(accepted_len=acc, n_emitted=nem, emitted=em, cdf_lo=np.full(B, np.nan), cdf_hi=np.full(B, np.nan),
                tok_below=np.full(B, -1, np.int32), tok_above=np.full(B, -1, np.int32))


def prune_compact(keep_mask, cu_q, *, suffix_close=True, payload=None):
    """Sec. 3.2 / 3.3 row pruning; returns dict of the new ragged layout and row maps."""
    lib = _load()
    keep, cu = _c(keep_mask, np.uint8), _c(cu_q, np.int32)
    B = len(cu) - 1
    N = int(cu[-1])
    assert len(keep) == N
    new_cu = np.zeros(B + 1, np.int32)
    new_len = np.zeros(B, np.int32)
    src = np.full(N, -1, np.int32)
    dst = np.full(N, -1, np.int32)
    n_act = np.zeros(1, np.int32)
    act = np.full(B, -1, np.int32)
    pin = pout = None
    row_bytes = 0
    if payload is not None:
        pay = np.ascontiguousarray(payload)
        assert pay.shape[0] == N
        row_bytes = pay.nbytes // max(N, 1) if N else 0
        pin = pay.view(np.uint8).reshape(N, row_bytes) if N else np.zeros((0, 0), np.uint8)
        pout = np.zeros_like(pin)
    lib.fo_prune_compact(_p(keep), _p(cu), _p(new_cu), _p(new_len), _p(src), _p(dst), _p(n_act), _p(act),
                         _p(pin), _p(pout), ctypes.c_int64(row_bytes), ctypes.c_int(B),
                         ctypes.c_int(1 if suffix_close else 0))
    res = dict(new_cu_q=new_cu, new_q_lens=new_len, src_row=src, dst_row=dst, n_active=int(n_act[0]),
               active_ids=act)
    if payload is not None:
        n_new = int(new_cu[-1])
        res["payload"] = pout.view(pay.dtype).reshape((N,) + pay.shape[1:])[:n_new]
    return res


def prune_restore(compact, dst_row, *, pad_byte=0):
    """Sec. 3.2 / Sec. 4: scatter compacted rows back to the original layout."""
    lib = _load()
    dst = _c(dst_row, np.int32)
    N = len(dst)
    comp = np.ascontiguousarray(compact)
    row_shape = comp.shape[1:]
    row_bytes = int(np.prod(row_shape)) * comp.dtype.itemsize
    cin = comp.view(np.uint8).reshape(comp.shape[0], row_bytes)
    out = np.zeros((N, row_bytes), np.uint8)
    has = np.zeros(N, np.uint8)
    lib.fo_prune_restore(_p(cin), _p(dst), _p(out), _p(has), ctypes.c_int64(row_bytes), ctypes.c_int(N),
                         ctypes.c_int(pad_byte))
    return out.view(comp.dtype).reshape((N,) + row_shape), has


def kv_append(k_new, v_new, k_cache, v_cache, block_tables, ctx_lens, cu_q, *, P, token_major=False):
    """Store this call's key / value rows ([N, H_kv, D]) into copies of the paged caches
    ([n_pages, H_kv, P, D]; [n_pages, P, H_kv, D] with token_major) at positions ctx_lens[i] + j; returns
    the two new caches in the layout they came in."""
    if token_major:
        kc, vc = kv_append(k_new, v_new, np.swapaxes(k_cache, 1, 2), np.swapaxes(v_cache, 1, 2), block_tables, ctx_lens,
                           cu_q, P=P)
        return np.ascontiguousarray(np.swapaxes(kc, 1, 2)), np.ascontiguousarray(np.swapaxes(vc, 1, 2))
    lib = _load()
    kc, vc = np.array(k_cache, copy=True, order="C"), np.array(v_cache, copy=True, order="C")
    kn, vn = np.ascontiguousarray(k_new), np.ascontiguousarray(v_new)
    assert kn.dtype == kc.dtype and vn.dtype == vc.dtype and kn.shape == vn.shape
    bt, ctx, cu = _c(block_tables, np.int32), _c(ctx_lens, np.int32), _c(cu_q, np.int32)
    B = len(ctx)
    H_kv, D = kc.shape[1], kc.shape[3]
    assert kc.shape[2] == P and kn.shape[1:] == (H_kv, D)
    lib.fo_kv_append(_p(kn), _p(vn), _p(kc), _p(vc), _p(bt), _p(ctx), _p(cu), ctypes.c_int(B), ctypes.c_int(H_kv),
                     ctypes.c_int(D), ctypes.c_int(P), ctypes.c_int(bt.shape[1]), ctypes.c_int(kc.dtype.itemsize))
    return kc, vc


def topk_rank_check(logits, draft_tokens, cu_q, cu_d, *, K, dtype="f32"):
    """Sec. 3.2 / Sec. 4 early-exit check: rank of every draft among its row's scores and the
    (not yet suffix-closed) keep mask over the active rows.  ``logits`` [N, V] is fp32, or bf16 bit
    patterns (uint16) with dtype="bf16"."""
    lib = _load()
    z = _c(logits, np.float32 if dtype == "f32" else np.uint16)
    toks, cq, cd = _c(draft_tokens, np.int32), _c(cu_q, np.int32), _c(cu_d, np.int32)
    B = len(cq) - 1
    N, N_d = int(cq[-1]), int(cd[-1])
    V = z.shape[1]
    assert z.shape[0] >= N and len(toks) >= N_d
    rank = np.full(N_d, -1, np.int32)
    keep = np.zeros(N, np.uint8)
    rc = lib.fo_topk_rank_check(_p(z), _p(toks), _p(cq), _p(cd), _p(rank), _p(keep), ctypes.c_int(B), ctypes.c_int(V),
                                ctypes.c_int(int(K)), ctypes.c_int(F32 if dtype == "f32" else BF16))
    if rc != 0:
        raise ValueError(f"fo_topk_rank_check: {rc}")
    return dict(rank=rank, keep=keep)


def verify_chunked(batch, chunks: List[np.ndarray], *, with_attention=True, mode=PROBS, temperature=1.0):
    """Frontier (chunked) verification of one step, Sec. 3.3.

    ``chunks[k][i]`` is the number of drafts of request i verified in chunk k.  A request's
    bonus row rides with the chunk that verifies its last draft (or with chunk 0 when it
    has no drafts).  After every chunk the accept step runs on that chunk's rows; a request
    with a rejection commits its accepted prefix and recovery token and every later row of
    it is discarded, so later chunks hold no row of it.

    Returns dict(accepted_len, n_emitted, emitted [B,S_max+1], rows_processed, and, with
    attention, out [N,H_q,D] with NaN on rows that were never computed).
    """
    B, S_max = batch.B, batch.S_max
    cu_q, cu_d = batch.cu_q, batch.cu_d
    N = batch.N
    pos = np.zeros(B, np.int64)
    active = np.ones(B, bool)
    acc_total = np.zeros(B, np.int32)
    n_em = np.zeros(B, np.int32)
    emitted = np.full((B, S_max + 1), -1, np.int32)
    out = np.full((N, batch.H_q, batch.D), np.nan) if with_attention else None
    rows_processed = 0
    p_src = batch.z_target if mode == LOGITS else batch.p_target
    q_src = batch.z_draft if mode == LOGITS else batch.p_draft
    for k, nk in enumerate(chunks):
        nk = np.asarray(nk, np.int64)
        t_mask = np.zeros(N, np.uint8)
        d_mask = np.zeros(batch.N_d, np.uint8)
        ctx_k = batch.ctx_lens.copy()
        for i in range(B):
            if not active[i]:
                continue
            last = pos[i] + nk[i] == batch.spec_lens[i]
            first_and_empty = batch.spec_lens[i] == 0 and k == 0
            t_i = int(nk[i]) + (1 if (last and (nk[i] > 0 or first_and_empty)) else 0)
            t_mask[cu_q[i] + pos[i]: cu_q[i] + pos[i] + t_i] = 1
            d_mask[cu_d[i] + pos[i]: cu_d[i] + pos[i] + nk[i]] = 1
            ctx_k[i] = batch.ctx_lens[i] + pos[i]
        tsel = prune_compact(t_mask, cu_q, suffix_close=False, payload=batch.q if with_attention else None)
        dsel = prune_compact(d_mask, cu_d, suffix_close=False)
        n_rows = int(tsel["new_cu_q"][-1])
        rows_processed += n_rows
        if n_rows == 0:
            continue
        if with_attention:
            o_k, _ = verify_attention(tsel["payload"], batch.k_cache, batch.v_cache, batch.block_tables, ctx_k,
                                      tsel["new_cu_q"], H_q=batch.H_q, H_kv=batch.H_kv, D=batch.D, P=batch.P,
                                      dtype=batch.dtype, scale=batch.scale)
            out[tsel["src_row"][:n_rows]] = o_k
        S_k = int(nk.max()) if len(nk) else 0
        r = spec_accept(p_src, q_src, batch.draft_tokens, batch.u_accept, batch.u_sample, tsel["new_cu_q"],
                        dsel["new_cu_q"], S_max=S_k, t_rows=tsel["src_row"][:n_rows],
                        d_rows=dsel["src_row"][: int(dsel["new_cu_q"][-1])], mode=mode, temperature=temperature)
        for i in range(B):
            if not active[i]:
                continue
            ne = int(r["n_emitted"][i])
            emitted[i, n_em[i]: n_em[i] + ne] = r["emitted"][i, :ne]
            n_em[i] += ne
            acc_total[i] += r["accepted_len"][i]
            if r["accepted_len"][i] < nk[i]:
                active[i] = False
            pos[i] += nk[i]
            if pos[i] >= batch.spec_lens[i]:
                active[i] = False
    return dict(accepted_len=acc_total, n_emitted=n_em, emitted=emitted, rows_processed=rows_processed, out=out)
