"""Seeded synthetic verification batches (inputs only).

This module serves both the CPU oracle and the HIP path and therefore holds none of
the verification method's arithmetic: it draws shapes, lengths, page tables, Q/K/V
values, logits/probabilities, draft tokens and uniforms.  Everything is generated on
the host with ``numpy.random.Generator(PCG64(seed))``.

The batches stand in for the paper's serving workloads (Sec. 6.1: ShareGPT, LongBench,
HumanEval prompts under an Azure-trace arrival process; Sec. 6.2.4: run-time batch sizes
and chosen speculative lengths), none of which are reproduced here: only their shapes
(ragged per-request speculative length inside one continuous batch, Sec. 3.1; paged KV
cache of a continuous-batching engine, Sec. 2.1) are mirrored.
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
import math
import os
from typing import Optional

import numpy as np

PAGE = 16


# --------------------------------------------------------------------------------------
# bf16 helpers (storage format conversion only)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the 8-bit OCP E4M3 format (nearest, ties to the even code; magnitudes above 448, the largest
    finite value, saturate to it) and return the byte patterns.  Storage format conversion only."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.arange(127)
    e, m = codes >> 3, codes & 7
    values = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1 + m / 8.0) * 2.0 ** (e - 7.0))  # codes 0x00 .. 0x7e, increasing
    mid = (values[:-1] + values[1:]) / 2
    mag = np.minimum(np.abs(x).astype(np.float64), values[-1])
    lo = np.searchsorted(mid, mag, side="left")           # mid[lo-1] < mag <= mid[lo]
    tie = (lo < len(mid)) & (mag == mid[np.minimum(lo, len(mid) - 1)])
    code = np.where(tie & (lo % 2 == 1), lo + 1, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | np.uint8(0x80), code).astype(np.uint8)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _parallel_chunks(rng: np.random.Generator, n: int, chunk: int, fill) -> None:
    """Call fill(child_rng, a, b) for the chunks [a, b) of range(n), each chunk with its own child
    generator spawned from ``rng`` (so the result does not depend on the number of threads)."""
    starts = list(range(0, n, chunk))
    kids = rng.spawn(len(starts))
    with concurrent.futures.ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(lambda t: fill(t[0], t[1], min(n, t[1] + chunk)), zip(kids, starts)))


def _normal_store(rng: np.random.Generator, shape, dtype: str, chunk: int = 1 << 22) -> np.ndarray:
    """N(0,1) values in the storage format: fp32, or bf16 bit patterns (uint16).  Arrays larger than
    one chunk are filled chunk by chunk from child generators, several chunks at a time."""
    n = int(np.prod(shape))
    if n <= chunk:
        x = rng.standard_normal(n, dtype=np.float32)
        return (x if dtype == "f32" else f32_to_bf16_bits(x)).reshape(shape)
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)

    def fill(child, a, b):
        x = child.standard_normal(b - a, dtype=np.float32)
        out[a:b] = x if dtype == "f32" else f32_to_bf16_bits(x)

    _parallel_chunks(rng, n, chunk, fill)
    return out.reshape(shape)


# --------------------------------------------------------------------------------------
# batch container
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class VerifyBatch:
    """One verification step over a continuous batch.

    Request i has committed context ``ctx_lens[i]`` and speculative length
    ``spec_lens[i]``; it contributes ``spec_lens[i] + 1`` query rows (the last committed
    token followed by its drafts), concatenated over requests with offsets ``cu_q``.
    The K/V of those rows are already in the cache at logical positions
    ``ctx_lens[i] .. ctx_lens[i] + spec_lens[i]``.
    """

    name: str
    seed: int
    dtype: str                 # "f32" or "bf16" (Q/K/V storage; bf16 held as uint16 bits)
    B: int
    H_q: int
    H_kv: int
    D: int
    P: int
    V: int
    ctx_lens: np.ndarray       # [B] i32
    spec_lens: np.ndarray      # [B] i32
    cu_q: np.ndarray           # [B+1] i32 query/target row offsets
    cu_d: np.ndarray           # [B+1] i32 draft row offsets
    block_tables: np.ndarray   # [B, max_pages] i32, -1 where unused
    n_pages: int
    q: Optional[np.ndarray] = None          # [N, H_q, D]
    k_cache: Optional[np.ndarray] = None    # [n_pages, H_kv, P, D]
    v_cache: Optional[np.ndarray] = None
    z_target: Optional[np.ndarray] = None   # [N, V] f32 logits
    z_draft: Optional[np.ndarray] = None    # [N_d, V] f32 logits
    p_target: Optional[np.ndarray] = None   # [N, V] f32 probabilities
    p_draft: Optional[np.ndarray] = None    # [N_d, V] f32
    draft_tokens: Optional[np.ndarray] = None  # [N_d] i32
    u_accept: Optional[np.ndarray] = None   # [N_d] f32 in [0,1)
    u_sample: Optional[np.ndarray] = None   # [B] f32 in [0,1)
    extra: dict = dataclasses.field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(self.cu_q[-1])

    @property
    def N_d(self) -> int:
        return int(self.cu_d[-1])

    @property
    def max_pages(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def S_max(self) -> int:
        return int(self.spec_lens.max()) if self.B else 0

    def kv_tokens(self) -> int:
        return int((self.ctx_lens.astype(np.int64) + self.spec_lens + 1).sum())

    def attention_bytes(self) -> int:
        """Algorithmic bytes of one attention call: K and V once, q in, o out, block table."""
        e = 4 if self.dtype == "f32" else 2
        t = self.ctx_lens.astype(np.int64) + self.spec_lens + 1
        kv = 2 * int(t.sum()) * self.H_kv * self.D * e
        qo = 2 * self.N * self.H_q * self.D * e
        bt = 4 * int(((t + self.P - 1) // self.P).sum())
        return kv + qo + bt


def exclusive_offsets(lens: np.ndarray) -> np.ndarray:
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    np.cumsum(lens, out=cu[1:])
    return cu


# --------------------------------------------------------------------------------------
# pieces
# --------------------------------------------------------------------------------------
def build_paged_kv(rng, ctx_lens, q_lens, H_kv, D, P, dtype, spare_pages=3, permute=True):
    """Allocate pages for ctx+q tokens per request out of a randomly permuted pool.

    Every slot of the pool (tails of last pages and spare pages included) holds N(0,1)
    values, so a kernel that reads past a request's length produces a visible error.
    """
    tok = ctx_lens.astype(np.int64) + q_lens
    npg = (tok + P - 1) // P
    total = int(npg.sum()) + spare_pages
    max_pages = int(npg.max()) if len(npg) else 1
    max_pages = max(max_pages, 1)
    perm = rng.permutation(total).astype(np.int32) if permute else np.arange(total, dtype=np.int32)
    bt = np.full((len(tok), max_pages), -1, dtype=np.int32)
    a = 0
    for i, n in enumerate(npg):
        bt[i, : int(n)] = perm[a : a + int(n)]
        a += int(n)
    k = _normal_store(rng, (total, H_kv, P, D), dtype)
    v = _normal_store(rng, (total, H_kv, P, D), dtype)
    return bt, total, k, v


def softmax_rows_f32(z: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    """fp64 softmax of logits, rounded to fp32: how the synthetic probability inputs are made."""
    out = np.empty(z.shape, dtype=np.float32)
    step = max(1, (1 << 21) // max(1, z.shape[1]))

    def block(a):
        x = z[a : a + step].astype(np.float64) / temperature
        x -= x.max(axis=1, keepdims=True)
        np.exp(x, out=x)
        x /= x.sum(axis=1, keepdims=True)
        out[a : a + step] = x

    with concurrent.futures.ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(block, range(0, z.shape[0], step)))
    return out


def sample_rows(rng, p: np.ndarray) -> np.ndarray:
    """One token per row, drawn from the row's distribution (the draft model's own sampling)."""
    tok = np.empty(p.shape[0], dtype=np.int32)
    u = rng.random(p.shape[0])

    def one(r):
        c = np.cumsum(p[r].astype(np.float64))
        tok[r] = min(int(np.searchsorted(c, u[r] * c[-1], side="right")), p.shape[1] - 1)

    with concurrent.futures.ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(one, range(p.shape[0])))
    return tok


def build_probs(rng, cu_q, cu_d, V, sigma_t=2.0, draft_mode="noise", sigma_noise=0.5, keep_logits=True):
    """Target logits ~ N(0, sigma_t^2) per target row; draft logits per draft row.

    draft_mode: "noise" = target logits of the same position + N(0, sigma_noise^2);
                "independent" = fresh N(0, sigma_t^2); "equal" = target logits.
    Draft row n of request i pairs with target row n of request i.
    """
    N, N_d, B = int(cu_q[-1]), int(cu_d[-1]), len(cu_q) - 1
    z_t = (rng.standard_normal((N, V), dtype=np.float32) * np.float32(sigma_t)) if N else np.zeros((0, V), np.float32)
    z_d = np.empty((N_d, V), dtype=np.float32)
    for i in range(B):
        d = int(cu_d[i + 1] - cu_d[i])
        if d == 0:
            continue
        src = z_t[cu_q[i] : cu_q[i] + d]
        dst = slice(int(cu_d[i]), int(cu_d[i]) + d)
        if draft_mode == "equal":
            z_d[dst] = src
        elif draft_mode == "independent":
            z_d[dst] = rng.standard_normal((d, V), dtype=np.float32) * np.float32(sigma_t)
        else:
            z_d[dst] = src + rng.standard_normal((d, V), dtype=np.float32) * np.float32(sigma_noise)
    p_t = softmax_rows_f32(z_t)
    p_d = softmax_rows_f32(z_d) if draft_mode != "equal" else None
    if draft_mode == "equal":
        p_d = np.empty((N_d, V), dtype=np.float32)
        for i in range(B):
            d = int(cu_d[i + 1] - cu_d[i])
            p_d[int(cu_d[i]) : int(cu_d[i]) + d] = p_t[cu_q[i] : cu_q[i] + d]
    toks = sample_rows(rng, p_d)
    if not keep_logits:
        z_t = z_d = None
    return z_t, z_d, p_t, p_d, toks


# --------------------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------------------
CONFIGS = {
    1: dict(name="tiny", B=4, H_q=8, H_kv=2, D=64, dtype="f32", V=1000),
    2: dict(name="llama3_8b_layer", B=16, H_q=32, H_kv=8, D=128, dtype="bf16", V=128256),
    3: dict(name="high_load", B=128, H_q=32, H_kv=8, D=128, dtype="bf16", V=128256),
    4: dict(name="70b_share", B=256, H_q=64, H_kv=8, D=128, dtype="bf16", V=128256),
    5: dict(name="chunked_frontier", B=512, H_q=32, H_kv=8, D=128, dtype="bf16", V=152064),
}


def draw_lengths(cfg: int, rng, B: int):
    """Context and speculative lengths of configuration ``cfg`` for B requests."""
    if cfg == 1:
        ctx = rng.integers(64, 257, size=B)
        base = np.array([0, 2, 3, 4])
        spec = base[np.arange(B) % 4]
    elif cfg == 2:
        ctx = rng.integers(1024, 4097, size=B)
        spec = rng.integers(1, 9, size=B)
    elif cfg == 3:
        ctx = np.minimum(np.floor(rng.lognormal(math.log(2048), 0.8, size=B)), 8192).astype(np.int64)
        ctx = np.maximum(ctx, 1)
        w = 0.7 ** np.arange(8)
        spec = rng.choice(8, size=B, p=w / w.sum())
    elif cfg == 4:
        ctx = np.clip(np.floor(rng.lognormal(math.log(2048), 1.0, size=B)), 16, 16384).astype(np.int64)
        spec = rng.integers(1, 11, size=B)
    elif cfg == 5:
        ctx = rng.integers(512, 8193, size=B)
        spec = rng.integers(2, 9, size=B)
    else:
        raise ValueError(f"unknown config {cfg}")
    return ctx.astype(np.int32), spec.astype(np.int32)


def make_batch(cfg: int, rep: int = 0, *, B: Optional[int] = None, V: Optional[int] = None,
               with_kv: bool = True, with_probs: bool = True, draft_mode: Optional[str] = None,
               dtype: Optional[str] = None, keep_logits: bool = False,
               ctx_lens=None, spec_lens=None, H_q=None, H_kv=None, D=None) -> VerifyBatch:
    """Build configuration ``cfg`` (1..5) with seed 1000*cfg + rep.

    ``B``/``V``/``dtype``/head-shape overrides give reduced or varied versions of the same
    recipe for tests; explicit ``ctx_lens``/``spec_lens`` replace the drawn lengths.
    """
    c = dict(CONFIGS[cfg])
    if B is not None:
        c["B"] = B
    if V is not None:
        c["V"] = V
    if dtype is not None:
        c["dtype"] = dtype
    for k_, v_ in (("H_q", H_q), ("H_kv", H_kv), ("D", D)):
        if v_ is not None:
            c[k_] = v_
    seed = 1000 * cfg + rep
    rng = np.random.Generator(np.random.PCG64(seed))
    ctx, spec = draw_lengths(cfg, rng, c["B"])
    if ctx_lens is not None:
        ctx = np.asarray(ctx_lens, dtype=np.int32)
        c["B"] = len(ctx)
    if spec_lens is not None:
        spec = np.asarray(spec_lens, dtype=np.int32)
    assert len(ctx) == len(spec) == c["B"]
    q_lens = spec + 1
    cu_q = exclusive_offsets(q_lens)
    cu_d = exclusive_offsets(spec)
    N = int(cu_q[-1])
    vb = VerifyBatch(name=c["name"], seed=seed, dtype=c["dtype"], B=c["B"], H_q=c["H_q"], H_kv=c["H_kv"],
                     D=c["D"], P=PAGE, V=c["V"], ctx_lens=ctx, spec_lens=spec, cu_q=cu_q, cu_d=cu_d,
                     block_tables=np.full((c["B"], 1), -1, np.int32), n_pages=0)
    if with_kv:
        bt, n_pages, k, v = build_paged_kv(rng, ctx, q_lens, c["H_kv"], c["D"], PAGE, c["dtype"])
        vb.block_tables, vb.n_pages, vb.k_cache, vb.v_cache = bt, n_pages, k, v
        vb.q = _normal_store(rng, (N, c["H_q"], c["D"]), c["dtype"])
    if with_probs:
        prng = np.random.Generator(np.random.PCG64(seed + 500))
        mode = draft_mode or ("independent" if cfg == 1 else "noise")
        z_t, z_d, p_t, p_d, toks = build_probs(prng, cu_q, cu_d, c["V"], draft_mode=mode, keep_logits=keep_logits)
        vb.z_target, vb.z_draft, vb.p_target, vb.p_draft, vb.draft_tokens = z_t, z_d, p_t, p_d, toks
        vb.u_accept = prng.random(int(cu_d[-1]), dtype=np.float32)
        vb.u_sample = prng.random(c["B"], dtype=np.float32)
    return vb


def chunk_plan(cfg: int, spec_lens: np.ndarray, s_c: int = 2):
    """Per-request chunk boundaries over draft positions.

    cfg 4: two chunks, the first holding ceil(s/2) drafts; otherwise frontiers of ``s_c``
    drafts.  Returns a list of [B] arrays (number of drafts of each request in chunk k);
    the bonus row rides with the request's last non-empty chunk.
    """
    spec = spec_lens.astype(np.int64)
    if cfg == 4:
        a = (spec + 1) // 2
        return [a.astype(np.int32), (spec - a).astype(np.int32)]
    n_chunks = int(max(1, math.ceil(spec.max() / s_c))) if len(spec) else 1
    out = []
    for k in range(n_chunks):
        out.append(np.clip(spec - k * s_c, 0, s_c).astype(np.int32))
    return out
