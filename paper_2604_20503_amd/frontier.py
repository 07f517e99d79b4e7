"""Frontier (chunked) verification driver: sequences the C-ABI calls of one step (Sec. 3.3).

Pure call sequencing: every mask, offset, gather, attention, accept decision and state
update is produced by the library's kernels on the device; nothing is read back to the
host between chunks.
"""
from __future__ import annotations

from typing import List, Optional

import torch

from . import binding as B_


def verify_chunked(*, q, k_caches, v_caches, block_tables, ctx_lens, spec_lens, cu_q, cu_d, p_target, p_draft,
                   draft_tokens, u_accept, u_sample, chunks: List[torch.Tensor], scale, mode=B_.PROBS,
                   temperature=1.0, out: Optional[torch.Tensor] = None, S_total_max: int, chunk_S_max: int):
    """Verify every request's suffix chunk by chunk.

    ``k_caches`` / ``v_caches`` are lists with one cache per transformer layer (attention runs
    once per layer on each chunk's rows).  ``chunks[k]`` is a device int32 [B] tensor with the
    number of drafts of each request in chunk k.  Returns dict(accepted_len, n_emitted,
    emitted [B, S_total_max+1], out (attention output of the last layer scattered to the
    original row layout, untouched on rows never computed), rows (per-chunk row counts,
    device tensors)).
    """
    dev = q.device
    Bn = ctx_lens.shape[0]
    N, N_d = q.shape[0], draft_tokens.shape[0]
    i32 = dict(dtype=torch.int32, device=dev)
    pos, active, n_out, acc_total = (torch.empty(Bn, **i32) for _ in range(4))
    out_tokens = torch.empty((Bn, S_total_max + 1), **i32)
    B_.frontier_init(spec_lens, pos, active, n_out, acc_total, out_tokens)
    t_mask = torch.empty(N, dtype=torch.uint8, device=dev)
    d_mask = torch.empty(max(N_d, 1), dtype=torch.uint8, device=dev)[:N_d]
    chunk_ctx = torch.empty(Bn, **i32)
    q_chunk = torch.empty_like(q)
    if out is None:
        out = torch.zeros_like(q)
    o_chunk = torch.empty_like(out)
    rows = []
    for chunk_len in chunks:
        B_.frontier_plan(ctx_lens, spec_lens, cu_q, cu_d, pos, active, chunk_len, t_mask, d_mask, chunk_ctx)
        tsel = B_.prune_compact(t_mask, cu_q, suffix_close=False, payload=q, payload_out=q_chunk)
        dsel = B_.prune_compact(d_mask, cu_d, suffix_close=False) if N_d else None
        for k_cache, v_cache in zip(k_caches, v_caches):
            B_.verify_attention(q_chunk, k_cache, v_cache, block_tables, chunk_ctx, None, tsel["new_cu_q"], scale=scale,
                                out=o_chunk, max_q_len=chunk_S_max + 1)
        # the chunk's rows go back to their original positions; rows of other chunks keep their values
        B_.prune_scatter(o_chunk, tsel["src_row"], tsel["new_cu_q"][Bn:], out)
        acc, nem, em = B_.spec_accept(p_target, p_draft, draft_tokens, u_accept, u_sample, tsel["new_cu_q"],
                                      dsel["new_cu_q"] if dsel else torch.zeros(Bn + 1, **i32), S_max=chunk_S_max,
                                      t_rows=tsel["src_row"], d_rows=dsel["src_row"] if dsel else None, mode=mode,
                                      temperature=temperature)
        B_.frontier_commit(spec_lens, chunk_len, acc, nem, em, pos, active, n_out, acc_total, out_tokens)
        rows.append(tsel["new_cu_q"][-1:])
    return dict(accepted_len=acc_total, n_emitted=n_out, emitted=out_tokens, out=out, rows=rows)
