"""Frontier (chunked) verification driver: sequences the C-ABI calls of one step (Sec. 3.3).

Pure call sequencing: every mask, offset, gather, attention, accept decision and state
update is produced by the library's kernels on the device; nothing is read back to the
host between chunks.  ``ChunkedVerifier`` allocates every buffer once, so that ``run()`` is
launches only and can be captured into a HIP graph; ``verify_chunked`` is the one-shot form.
"""
from __future__ import annotations

from typing import Callable, List, Optional

import torch

from . import binding as B_


class ChunkedVerifier:
    """One verification step in chunks over fixed inputs.

    ``k_caches`` / ``v_caches`` are lists with one cache per transformer layer (attention runs
    once per layer on each chunk's rows).  ``chunks[k]`` is a device int32 [B] tensor with the
    number of drafts of each request in chunk k.  ``use_plan``: build the attention schedule
    once per chunk (``fsr_attn_plan``) instead of once per layer launch.
    """

    def __init__(self, *, q, k_caches, v_caches, block_tables, ctx_lens, spec_lens, cu_q, cu_d, p_target, p_draft,
                 draft_tokens, u_accept, u_sample, chunks: List[torch.Tensor], scale, mode=B_.PROBS, temperature=1.0,
                 out: Optional[torch.Tensor] = None, S_total_max: int, chunk_S_max: int, use_plan: bool = True):
        self.a = dict(q=q, k_caches=k_caches, v_caches=v_caches, block_tables=block_tables, ctx_lens=ctx_lens,
                      spec_lens=spec_lens, cu_q=cu_q, cu_d=cu_d, p_target=p_target, p_draft=p_draft,
                      draft_tokens=draft_tokens, u_accept=u_accept, u_sample=u_sample, chunks=chunks, scale=scale,
                      mode=mode, temperature=temperature)
        dev = q.device
        Bn = ctx_lens.shape[0]
        N, N_d = q.shape[0], draft_tokens.shape[0]
        self.Bn, self.N, self.N_d, self.chunk_S_max = Bn, N, N_d, chunk_S_max
        i32 = dict(dtype=torch.int32, device=dev)
        u8 = dict(dtype=torch.uint8, device=dev)
        self.pos, self.active, self.n_out, self.acc_total = (torch.empty(Bn, **i32) for _ in range(4))
        self.out_tokens = torch.empty((Bn, S_total_max + 1), **i32)
        self.t_mask = torch.empty(N, **u8)
        self.d_mask = torch.empty(max(N_d, 1), **u8)[:N_d]
        self.chunk_ctx = torch.empty(Bn, **i32)
        self.q_chunk = torch.empty_like(q)
        self.out = torch.zeros_like(q) if out is None else out
        self.o_chunk = torch.empty_like(self.out)

        def maps(n):
            return dict(new_cu_q=torch.empty(Bn + 1, **i32), new_q_lens=torch.empty(Bn, **i32), src_row=torch.empty(n, **i32),
                        dst_row=torch.empty(n, **i32), n_active=torch.empty(1, **i32), active_ids=torch.empty(Bn, **i32))

        self.tsel, self.dsel = maps(N), (maps(N_d) if N_d else None)
        self.zero_cu = torch.zeros(Bn + 1, **i32)
        self.acc, self.nem = torch.empty(Bn, **i32), torch.empty(Bn, **i32)
        self.em = torch.empty((Bn, chunk_S_max + 1), **i32)
        k0 = k_caches[0]
        n_pages, H_kv, P, D = k0.shape
        shape = dict(B=Bn, N_cap=N, H_q=q.shape[1], H_kv=H_kv, D=D, P=P, max_pages=block_tables.shape[1], n_pages=n_pages,
                     dtype=q.dtype, out_dtype=self.out.dtype, max_q_len=chunk_S_max + 1)
        self.ws_attn = torch.empty(max(256, B_.attn_workspace_bytes(**shape)), **u8)
        V = p_target.shape[1]
        self.ws_acc = torch.empty(max(256, B_.accept_workspace_bytes(B=Bn, V=V, S_max=chunk_S_max, mode=mode,
                                                                     temperature=temperature)), **u8)
        self.plan = None
        if use_plan and B_.attn_path(**shape) == B_.PATH_STREAM:
            self.plan = B_.attn_plan(self.q_chunk, k0, block_tables, ctx_lens, cu_q, scale=scale, out_dtype=self.out.dtype,
                                     max_q_len=chunk_S_max + 1)

    def run(self, mark: Optional[Callable[[str, int, "ChunkedVerifier"], None]] = None):
        """Enqueue the whole step on the current stream.  ``mark(stage, k, self)`` (eager runs only) is called
        at "attn_begin" / "attn_end" (around chunk k's attention launches) and "chunk_end", e.g. to record events
        or to look at the chunk's row selection."""
        a = self.a
        Bn = self.Bn
        B_.frontier_init(a["spec_lens"], self.pos, self.active, self.n_out, self.acc_total, self.out_tokens)
        for k, chunk_len in enumerate(a["chunks"]):
            B_.frontier_plan(a["ctx_lens"], a["spec_lens"], a["cu_q"], a["cu_d"], self.pos, self.active, chunk_len, self.t_mask,
                             self.d_mask, self.chunk_ctx)
            tsel = B_.prune_compact(self.t_mask, a["cu_q"], suffix_close=False, payload=a["q"], payload_out=self.q_chunk,
                                    out=self.tsel)
            dsel = B_.prune_compact(self.d_mask, a["cu_d"], suffix_close=False, out=self.dsel) if self.N_d else None
            if self.plan is not None:
                B_.attn_plan(self.q_chunk, a["k_caches"][0], a["block_tables"], self.chunk_ctx, tsel["new_cu_q"],
                             scale=a["scale"], out_dtype=self.out.dtype, max_q_len=self.chunk_S_max + 1, plan=self.plan)
            if mark is not None:
                mark("attn_begin", k, self)
            for k_cache, v_cache in zip(a["k_caches"], a["v_caches"]):
                B_.verify_attention(self.q_chunk, k_cache, v_cache, a["block_tables"], self.chunk_ctx, None, tsel["new_cu_q"],
                                    scale=a["scale"], out=self.o_chunk, workspace=self.ws_attn,
                                    max_q_len=self.chunk_S_max + 1, plan=self.plan)
            if mark is not None:
                mark("attn_end", k, self)
            # the chunk's rows go back to their original positions; rows of other chunks keep their values
            B_.prune_scatter(self.o_chunk, tsel["src_row"], tsel["new_cu_q"][Bn:], self.out)
            B_.spec_accept(a["p_target"], a["p_draft"], a["draft_tokens"], a["u_accept"], a["u_sample"], tsel["new_cu_q"],
                           dsel["new_cu_q"] if dsel else self.zero_cu, S_max=self.chunk_S_max, t_rows=tsel["src_row"],
                           d_rows=dsel["src_row"] if dsel else None, mode=a["mode"], temperature=a["temperature"],
                           accepted_len=self.acc, n_emitted=self.nem, emitted=self.em, workspace=self.ws_acc)
            B_.frontier_commit(a["spec_lens"], chunk_len, self.acc, self.nem, self.em, self.pos, self.active, self.n_out,
                               self.acc_total, self.out_tokens)
            if mark is not None:
                mark("chunk_end", k, self)
        return dict(accepted_len=self.acc_total, n_emitted=self.n_out, emitted=self.out_tokens, out=self.out)


def verify_chunked(*, q, k_caches, v_caches, block_tables, ctx_lens, spec_lens, cu_q, cu_d, p_target, p_draft,
                   draft_tokens, u_accept, u_sample, chunks: List[torch.Tensor], scale, mode=B_.PROBS,
                   temperature=1.0, out: Optional[torch.Tensor] = None, S_total_max: int, chunk_S_max: int,
                   use_plan: bool = True):
    """Verify every request's suffix chunk by chunk (one eager pass).  Returns dict(accepted_len, n_emitted,
    emitted [B, S_total_max+1], out (attention output of the last layer scattered to the original row layout,
    untouched on rows never computed), rows (per-chunk row counts, device tensors))."""
    v = ChunkedVerifier(q=q, k_caches=k_caches, v_caches=v_caches, block_tables=block_tables, ctx_lens=ctx_lens,
                        spec_lens=spec_lens, cu_q=cu_q, cu_d=cu_d, p_target=p_target, p_draft=p_draft,
                        draft_tokens=draft_tokens, u_accept=u_accept, u_sample=u_sample, chunks=chunks, scale=scale,
                        mode=mode, temperature=temperature, out=out, S_total_max=S_total_max, chunk_S_max=chunk_S_max,
                        use_plan=use_plan)
    rows = []
    res = v.run(mark=lambda stage, k, s: rows.append(s.tsel["new_cu_q"][-1:].clone()) if stage == "chunk_end" else None)
    res["rows"] = rows
    return res
