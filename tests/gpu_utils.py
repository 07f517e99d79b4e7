"""Helpers shared by the GPU parity tests: host batch -> device tensors, error metrics."""
import sys

import numpy as np
import torch


def announce(msg):
    """Name the case before a GPU step so a fault can be traced to it."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def dev(x, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x if not bf16 else x.view(np.int16)))
    t = t.cuda()
    return t.view(torch.bfloat16) if bf16 else t


class DeviceBatch:
    def __init__(self, b, probs=True, kv=True, logits=False):
        bf = b.dtype == "bf16"
        self.b = b
        self.ctx_lens, self.spec_lens = dev(b.ctx_lens), dev(b.spec_lens)
        self.cu_q, self.cu_d = dev(b.cu_q), dev(b.cu_d)
        self.block_tables = dev(b.block_tables)
        if kv:
            self.q, self.k_cache, self.v_cache = dev(b.q, bf), dev(b.k_cache, bf), dev(b.v_cache, bf)
        if probs:
            self.p_target, self.p_draft = dev(b.p_target), dev(b.p_draft)
            self.draft_tokens, self.u_accept, self.u_sample = dev(b.draft_tokens), dev(b.u_accept), dev(b.u_sample)
        if logits:
            self.z_target, self.z_draft = dev(b.z_target), dev(b.z_draft)


def attn_rel_err(o_gpu: np.ndarray, o_ref: np.ndarray):
    """|o_gpu - o_ref| / max(|o_ref|, rms of the (row, head) vector), elementwise."""
    rms = np.sqrt((o_ref ** 2).mean(axis=-1, keepdims=True))
    return np.abs(o_gpu - o_ref) / np.maximum(np.abs(o_ref), rms)


def check_attention(o_gpu_t: torch.Tensor, o_ref: np.ndarray, in_dtype: str, n_rows: int):
    """Tolerance of the benchmark spec: 1e-5 relative for fp32 inputs, 2e-3 for bf16 inputs, measured
    on the value before the output cast; a bf16 output adds its own rounding, at most half an ulp
    (2^-8 relative)."""
    o = o_gpu_t[:n_rows].float().cpu().numpy().astype(np.float64)
    ref = o_ref[:n_rows]
    assert np.isfinite(o).all()
    tol = 1e-5 if in_dtype == "f32" else 2e-3
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), rms)
    bound = tol * den
    if o_gpu_t.dtype == torch.bfloat16:
        bound = bound + 2.0 ** -8 * np.abs(ref)
    bad = np.abs(o - ref) > bound
    err = (np.abs(o - ref) / den).max() if o.size else 0.0
    assert not bad.any(), f"{bad.sum()} of {bad.size} elements out of tolerance; max rel err {err:.3e}"
    return err


def fragile_draws(u_sample, cdf_lo, cdf_hi, band=1e-6):
    """Requests whose uniform lies within `band` of an edge of the oracle token's CDF interval."""
    u = u_sample.astype(np.float64)
    with np.errstate(invalid="ignore"):
        return (np.abs(u - cdf_lo) < band) | (np.abs(u - cdf_hi) < band)


def check_tokens(em, ref, u_sample, band=1e-6):
    """Emitted tokens against the oracle's: bit-exact, except that a request whose uniform lies within
    `band` of an edge of the drawn token's CDF interval may carry, at the drawn position only, the
    nearest positive-mass token on the side of that edge.  Returns (fragile requests, requests that
    differ); any other difference fails."""
    frag = fragile_draws(u_sample, ref["cdf_lo"], ref["cdf_hi"], band)
    u = u_sample.astype(np.float64)
    diff_rows = np.where((em != ref["emitted"]).any(axis=1))[0]
    for i in diff_rows:
        n = int(ref["accepted_len"][i])
        cols = np.where(em[i] != ref["emitted"][i])[0]
        assert cols.tolist() == [n], f"request {i}: emitted {em[i]} vs oracle {ref['emitted'][i]} differ outside the drawn position {n}"
        allowed = set()
        if abs(u[i] - ref["cdf_lo"][i]) < band and ref["tok_below"][i] >= 0:
            allowed.add(int(ref["tok_below"][i]))
        if abs(u[i] - ref["cdf_hi"][i]) < band and ref["tok_above"][i] >= 0:
            allowed.add(int(ref["tok_above"][i]))
        assert int(em[i, n]) in allowed, (
            f"request {i}: token {em[i, n]} vs oracle {ref['emitted'][i, n]}; u={u[i]!r}, interval "
            f"[{ref['cdf_lo'][i]!r}, {ref['cdf_hi'][i]!r}), neighbours {ref['tok_below'][i]}/{ref['tok_above'][i]}")
    return int(frag.sum()), len(diff_rows)


def check_accept(gpu, ref, u_sample):
    """accepted_len / n_emitted bit-exact; emitted by check_tokens.  Returns (fragile, differing)."""
    acc, nem, em = (t.cpu().numpy() for t in gpu)
    assert np.array_equal(acc, ref["accepted_len"])
    assert np.array_equal(nem, ref["n_emitted"])
    return check_tokens(em, ref, u_sample)


def chunked_case(fsr, oracle, b, chunks, dtype, mode="probs"):
    """Frontier verification of batch ``b`` through the C ABI against the chunked oracle and the
    one-shot accept: lengths bit-exact, tokens bit-exact except fragile draws, exactly the same rows
    computed, attention rows within tolerance, same number of rows processed."""
    o_mode, g_mode = (oracle.GREEDY, 2) if mode == "greedy" else (oracle.PROBS, 0)
    ref = oracle.verify_chunked(b, chunks, mode=o_mode)
    one = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d,
                             S_max=b.S_max, mode=o_mode)
    assert np.array_equal(ref["emitted"], one["emitted"])
    d = DeviceBatch(b)
    out = torch.full(d.q.shape, float("nan"), dtype=torch.float32, device="cuda")
    r = fsr.verify_chunked(q=d.q, k_caches=[d.k_cache], v_caches=[d.v_cache], block_tables=d.block_tables,
                           ctx_lens=d.ctx_lens, spec_lens=d.spec_lens, cu_q=d.cu_q, cu_d=d.cu_d, p_target=d.p_target,
                           p_draft=d.p_draft, draft_tokens=d.draft_tokens, u_accept=d.u_accept, u_sample=d.u_sample,
                           chunks=[dev(c) for c in chunks], scale=b.scale, S_total_max=b.S_max,
                           chunk_S_max=int(max(c.max() for c in chunks)), out=out, mode=g_mode)
    torch.cuda.synchronize()
    assert np.array_equal(r["accepted_len"].cpu().numpy(), ref["accepted_len"])
    assert np.array_equal(r["n_emitted"].cpu().numpy(), ref["n_emitted"])
    em = r["emitted"].cpu().numpy()
    n_frag, n_diff = check_tokens(em, one, b.u_sample)
    o = out.cpu().numpy()
    done_ref = ~np.isnan(ref["out"][:, 0, 0])
    done_gpu = ~np.isnan(o[:, 0, 0])
    assert np.array_equal(done_ref, done_gpu)          # exactly the same rows were computed
    rows = np.where(done_ref)[0]
    err = check_attention(out[torch.from_numpy(rows).cuda()], ref["out"][rows], dtype, len(rows))
    assert sum(int(x.item()) for x in r["rows"]) == ref["rows_processed"]
    return dict(err=err, rows=len(rows), rows_total=b.N, fragile=n_frag, token_diffs=n_diff, accepted=int(ref["accepted_len"].sum()))
