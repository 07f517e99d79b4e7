#!/usr/bin/env python3
"""Benchmark of the verification hot path on one MI355X.

A "step" is one target-side verification step over the Llama-3-8B-shaped ragged batch
(configuration 2 of the workload table): for each of the model's 32 layers one
``verify_attention`` call on that layer's own paged KV cache, then ``spec_accept`` on the
step's target/draft distributions (vocabulary 128256), then ``survivor_mask`` +
``prune_compact`` re-packing the surviving rows.  All inputs are resident in HBM before the
timed region; the 32 layers use 32 distinct caches (5 GB) so the reads come from HBM and not
from the last-level cache.  The step is captured once into a HIP graph and replayed.

``--workload 3|4|5`` runs the same one-shot step at the batch shapes of the other configurations
(their layers cycle through as many distinct caches as fit 16 GB); the metric is quoted on the default.
``--workload 4|5 --chunked`` runs those configurations' own schedules instead: two chunks (workload 4)
or frontiers of two drafts (workload 5), each chunk = row selection, attention over every layer on the
chunk's rows only, accept, commit; K/V of a request are read again by every chunk it takes part in.

Prints ONE JSON line: verified draft tokens/s (sum of the speculative lengths submitted per
step / step time), the HBM roofline of the dominant kernel (attention), per-kernel figures for the
other calls of the step ("kernels"), and the CPU oracle timed beside it on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

N_LAYERS = 32           # Llama-3-8B depth: attention calls per verification step
WORKLOADS = {
    2: "cfg2 llama3_8b_layer: B=16, 32 q / 8 kv heads, D=128, bf16 paged KV (page 16, permuted), "
       "ctx U[1024,4096], spec U[1,8], vocab 128256",
    3: "cfg3 high_load: B=128, 32 q / 8 kv heads, D=128, bf16 paged KV, ctx lognormal(median 2048) <= 8192, "
       "spec geometric 0..7, vocab 128256",
    4: "cfg4 70b_share, one-shot: B=256, 64 q / 8 kv heads, D=128, bf16 paged KV, ctx lognormal(median 2048) in "
       "[16,16384], spec U[1,10], vocab 128256",
    5: "cfg5 chunked_frontier shapes, one-shot: B=512, 32 q / 8 kv heads, D=128, bf16 paged KV, ctx U[512,8192], "
       "spec U[2,8], vocab 152064",
}
HBM_PEAK_GBS = 8000.0   # MI355X HBM3E peak


def build_step(fsr, torch, b, n_layers, seed, cache_budget_bytes=16e9, use_plan=True, variants=False):
    """Device buffers and a closure running one full step without allocating.  The layers cycle
    through as many distinct KV caches as fit the budget (all 32 at workload 2)."""
    def dev(x, bf16=False):
        t = torch.from_numpy(np.ascontiguousarray(x.view(np.int16) if bf16 else x)).cuda()
        return t.view(torch.bfloat16) if bf16 else t

    q = dev(b.q, True)
    k0, v0 = dev(b.k_cache, True), dev(b.v_cache, True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    k_caches, v_caches = [k0], [v0]
    kv_bytes = 2 * k0.numel() * k0.element_size()
    n_caches = int(max(1, min(n_layers, cache_budget_bytes // kv_bytes)))

    def draw_like(t):  # other layers: same shape and distribution, drawn on the device in slabs
        o = torch.empty_like(t)
        flat = o.view(-1)
        for a in range(0, flat.numel(), 1 << 28):
            n = min(1 << 28, flat.numel() - a)
            flat[a:a + n] = torch.randn(n, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        return o

    for _ in range(1, n_caches):
        k_caches.append(draw_like(k0))
        v_caches.append(draw_like(v0))
    bt, ctx, spec, cu_q, cu_d = dev(b.block_tables), dev(b.ctx_lens), dev(b.spec_lens), dev(b.cu_q), dev(b.cu_d)
    p_t, p_d = dev(b.p_target), dev(b.p_draft)
    toks, u_a, u_s = dev(b.draft_tokens), dev(b.u_accept), dev(b.u_sample)
    S_max = b.S_max
    out = torch.empty_like(q)
    ws_attn = torch.empty(max(256, fsr.attn_workspace_bytes(
        B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, max_pages=b.max_pages, n_pages=b.n_pages,
        dtype=torch.bfloat16, out_dtype=torch.bfloat16, max_q_len=S_max + 1)), dtype=torch.uint8, device="cuda")
    ws_acc = torch.empty(max(256, fsr.accept_workspace_bytes(B=b.B, V=b.V, S_max=S_max)), dtype=torch.uint8,
                         device="cuda")
    i32 = dict(dtype=torch.int32, device="cuda")
    acc, nem = torch.empty(b.B, **i32), torch.empty(b.B, **i32)
    em = torch.empty((b.B, S_max + 1), **i32)
    keep = torch.empty(b.N, dtype=torch.uint8, device="cuda")
    prune_out = dict(new_cu_q=torch.empty(b.B + 1, **i32), new_q_lens=torch.empty(b.B, **i32),
                     src_row=torch.empty(b.N, **i32), dst_row=torch.empty(b.N, **i32), n_active=torch.empty(1, **i32),
                     active_ids=torch.empty(b.B, **i32))
    packed = torch.empty_like(out)

    plan = fsr.attn_plan(q, k0, bt, ctx, cu_q, scale=b.scale, max_q_len=S_max + 1) if use_plan else None

    def attention_all_layers():
        # the step's schedule once (lengths and block tables are the same for every layer), then the layers
        if use_plan:
            fsr.attn_plan(q, k0, bt, ctx, cu_q, scale=b.scale, max_q_len=S_max + 1, plan=plan)
        for l in range(n_layers):
            fsr.verify_attention(q, k_caches[l % n_caches], v_caches[l % n_caches], bt, ctx, spec, cu_q, scale=b.scale,
                                 out=out, workspace=ws_attn, max_q_len=S_max + 1, plan=plan)

    def tail():
        fsr.spec_accept(p_t, p_d, toks, u_a, u_s, cu_q, cu_d, S_max=S_max, accepted_len=acc, n_emitted=nem, emitted=em,
                        workspace=ws_acc)
        fsr.survivor_compact(acc, cu_q, b.N, keep_mask=keep, payload=out, payload_out=packed, out=prune_out)

    def step():
        attention_all_layers()
        tail()

    def accept_only():
        fsr.spec_accept(p_t, p_d, toks, u_a, u_s, cu_q, cu_d, S_max=S_max, accepted_len=acc, n_emitted=nem, emitted=em,
                        workspace=ws_acc)

    def compact_only():
        fsr.survivor_compact(acc, cu_q, b.N, keep_mask=keep, payload=out, payload_out=packed, out=prune_out)

    rank = torch.empty(max(int(b.cu_d[-1]), 1), **i32)

    def rank_only():  # early-exit check on the step's target rows (stand-ins for intermediate scores); not part of the step
        fsr.topk_rank_check(p_t, toks, cu_q, cu_d, K=10, rank=rank[:int(b.cu_d[-1])], keep_mask=keep)

    calls = dict(accept=accept_only, compact=compact_only, rank=rank_only)
    if getattr(b, "z_target", None) is not None:  # --logits: the same acceptance from logits (softmax inside the call)
        z_t, z_d = dev(b.z_target), dev(b.z_draft)
        ws_lg = torch.empty(max(256, fsr.accept_workspace_bytes(B=b.B, V=b.V, S_max=S_max, mode=1)), dtype=torch.uint8,
                            device="cuda")
        acc_l, nem_l, em_l = torch.empty_like(acc), torch.empty_like(nem), torch.empty_like(em)

        def accept_logits_only():  # not part of the step
            fsr.spec_accept(z_t, z_d, toks, u_a, u_s, cu_q, cu_d, S_max=S_max, mode=1, temperature=1.0, accepted_len=acc_l,
                            n_emitted=nem_l, emitted=em_l, workspace=ws_lg)

        calls["accept_logits"] = accept_logits_only

    extra_layers = 0
    if variants:  # --variants: the other forms of the same kernels, each timed on its own (not part of the step)
        # attention over 8-bit caches (E4M3 bytes, one scale per KV head): as many distinct caches as the bf16 ones
        n8 = int(max(1, min(n_layers, n_caches)))
        k8 = [torch.randint(0, 120, k0.shape, dtype=torch.uint8, device="cuda", generator=gen) for _ in range(n8)]
        v8 = [torch.randint(0, 120, k0.shape, dtype=torch.uint8, device="cuda", generator=gen) for _ in range(n8)]
        sc8 = torch.full((b.H_kv,), 0.02, dtype=torch.float32, device="cuda")
        out8 = torch.empty_like(q)
        extra_layers = n_layers

        def attention_kv8_all_layers():
            if use_plan:
                fsr.attn_plan(q, k0, bt, ctx, cu_q, scale=b.scale, max_q_len=S_max + 1, plan=plan)
            for l in range(n_layers):
                fsr.verify_attention_kv8(q, k8[l % n8], v8[l % n8], sc8, sc8, bt, ctx, cu_q, scale=b.scale, out=out8,
                                         workspace=ws_attn, max_q_len=S_max + 1, plan=plan)

        # append of the call's own K/V rows (bf16 and quantising), into caches of their own
        k_new = torch.randn((b.N, b.H_kv, b.D), device="cuda", generator=gen).to(torch.bfloat16)
        v_new = torch.randn((b.N, b.H_kv, b.D), device="cuda", generator=gen).to(torch.bfloat16)
        k_app, v_app = k0.clone(), v0.clone()

        def append_only():
            fsr.kv_append(k_new, v_new, k_app, v_app, bt, ctx, cu_q)

        def append_kv8_only():
            fsr.kv_append_kv8(k_new, v_new, k8[0], v8[0], sc8, sc8, bt, ctx, cu_q)

        # greedy acceptance (arg-max of every target row) and the restore of the compacted rows to their old places
        ws_gr = torch.empty(max(256, fsr.accept_workspace_bytes(B=b.B, V=b.V, S_max=S_max, mode=2)), dtype=torch.uint8,
                            device="cuda")
        acc_g, nem_g, em_g = torch.empty_like(acc), torch.empty_like(nem), torch.empty_like(em)

        def greedy_only():
            fsr.spec_accept(p_t, None, toks, None, None, cu_q, cu_d, S_max=S_max, mode=2, accepted_len=acc_g, n_emitted=nem_g,
                            emitted=em_g, workspace=ws_gr)

        restored = torch.empty_like(out)
        has_value = torch.empty(b.N, dtype=torch.uint8, device="cuda")

        def restore_only():
            fsr.prune_restore(packed, prune_out["dst_row"], restored=restored, has_value=has_value)

        calls.update(attention_kv8=attention_kv8_all_layers, kv_append=append_only, kv_append_kv8=append_kv8_only,
                     greedy_accept=greedy_only, prune_restore=restore_only)

    state = dict(q=q, k0=k0, v0=v0, out=out, acc=acc, nem=nem, em=em, prune=prune_out, packed=packed, variant_layers=extra_layers,
                 n_caches=n_caches, kv_bytes=kv_bytes, k_caches=k_caches, v_caches=v_caches,
                 dev=dict(bt=bt, ctx=ctx, spec=spec, cu_q=cu_q, cu_d=cu_d, p_t=p_t, p_d=p_d, toks=toks, u_a=u_a, u_s=u_s),
                 calls=calls)
    return step, attention_all_layers, tail, state


def kernel_figures(b, st, times_us):
    """Algorithmic bytes of the step's other calls (what the method must move, from this batch's own outcome) next
    to their measured durations.  accept (PROBS): 8 bytes of gathers per draft + one target row (bonus) or one
    target and one draft row (rejection) per request; compaction: mask + offsets in, maps out, the surviving
    payload rows in and out; rank check: one score row per draft."""
    acc = st["acc"].cpu().numpy()
    d = b.spec_lens.astype(np.int64)
    rows = np.where(acc < d, 2, 1)                 # every request here has its bonus row
    accept_bytes = int((rows * 4 * b.V + 8 * d).sum())
    n_new = int(st["prune"]["new_cu_q"][-1].item())
    row_bytes = b.H_q * b.D * 2
    compact_bytes = b.N + 4 * (b.B + 1) + 4 * (2 * b.N + 3 * b.B) + b.N + 2 * n_new * row_bytes
    rank_bytes = int(d.sum()) * 4 * b.V

    def fig(us, nbytes, launches, note):
        gbs = nbytes / us / 1e3
        return dict(us=us, launches=launches, algorithmic_bytes=nbytes, achieved_GBs=gbs, frac_of_hbm_peak=gbs / HBM_PEAK_GBS,
                    note=note)

    extra = {}
    if "accept_logits" in times_us:
        # LOGITS mode: the rows that have to be normalised are those of the drafts tested (one target and one draft row
        # each, up to and including the first rejection) and the bonus row; the row(s) sampled from are read once more
        tested = np.minimum(acc + 1, d)
        norm_rows = 2 * tested + (acc == d)
        logits_bytes = int(((norm_rows + rows) * 4 * b.V + 8 * d).sum())
        all_rows_bytes = int((2 * d + 1).sum()) * 4 * b.V
        if b.B * (2 * b.S_max + 1) >= 3072 and b.S_max > 3:  # two passes: rows of the first two drafts, then the rest of the undecided
            pend = (np.minimum(acc, 2) == np.minimum(d, 2)) & (d > 2)
            read_rows = np.minimum(d + 1, 3) + np.minimum(d, 2) + pend * ((d + 1 - 3) + (d - 2))
        else:
            read_rows = 2 * d + 1
        read_bytes = int(((read_rows + rows) * 4 * b.V).sum())
        extra["spec_accept_logits"] = fig(
            times_us["accept_logits"], logits_bytes, 3,
            "accept_stats_kernel (twice, with a first accept_decide_kernel in between, when the call holds 3072 rows or more) + accept_decide_kernel + "
            f"accept_sample_kernel, T = 1; normalising every row of the call would read {all_rows_bytes} bytes; "
            f"this call reads {read_bytes} bytes; "
            f"not part of the timed step")
    if "attention_kv8" in times_us:
        L = st["variant_layers"]
        kv8_bytes = b.attention_bytes() - b.kv_tokens() * b.H_kv * b.D * 2   # K and V at one byte per element
        extra["verify_attention_kv8"] = fig(times_us["attention_kv8"] / L, kv8_bytes, 1,
                                            "verify_attention over E4M3 caches, per layer call (planned like the bf16 call unless --no-plan); not part of the timed step")
        rows_bytes = 2 * b.N * b.H_kv * b.D * 2
        extra["kv_append"] = fig(times_us["kv_append"], 2 * rows_bytes, 1, "kv_append_kernel: the call's bf16 K and V rows in, the same bytes into the pages")
        extra["kv_append_kv8"] = fig(times_us["kv_append_kv8"], rows_bytes + rows_bytes // 2, 1,
                                     "kv_append8_kernel: bf16 rows in, E4M3 bytes into the pages")
        extra["greedy_accept"] = fig(times_us["greedy_accept"], b.N * 4 * b.V + 4 * int(d.sum()), 3,
                                     "greedy_init_kernel + greedy_argmax_kernel + greedy_decide_kernel: every target row of the call once")
        extra["prune_restore"] = fig(times_us["prune_restore"], (n_new + b.N) * row_bytes + 5 * b.N, 1,
                                     "restore_rows_kernel: surviving rows back to their old places, filler elsewhere")
    return {
        **extra,
        "spec_accept": fig(times_us["accept"], accept_bytes, 2, "accept_decide_kernel + accept_sample_kernel"),
        "survivor_compact": fig(times_us["compact"], compact_bytes, 2,
                                f"prune_scan_kernel + gather_rows_kernel; {n_new} of {b.N} rows of {row_bytes} bytes survive"),
        "topk_rank_check": fig(times_us["rank"], rank_bytes, 3,
                               "rank_init + rank_count + rank_mask over the target rows, K = 10; not part of the timed step"),
    }


def chunked_run(args, fsr, torch, workloads, b):
    """The configuration's own chunked schedule (Sec. 3.3), every buffer preallocated, whole step in one HIP graph.
    Returns (ms per step, per-chunk table, attention totals)."""
    from paper_2604_20503_amd.frontier import ChunkedVerifier

    step, _, _, st = build_step(fsr, torch, b, args.layers, seed=2002, use_plan=False)
    del step
    d = st["dev"]
    chunks = workloads.chunk_plan(args.workload, b.spec_lens)
    dev_chunks = [torch.from_numpy(c).cuda() for c in chunks]
    layers = [(st["k_caches"][l % st["n_caches"]], st["v_caches"][l % st["n_caches"]]) for l in range(args.layers)]
    v = ChunkedVerifier(q=st["q"], k_caches=[k for k, _ in layers], v_caches=[x for _, x in layers], block_tables=d["bt"],
                        ctx_lens=d["ctx"], spec_lens=d["spec"], cu_q=d["cu_q"], cu_d=d["cu_d"], p_target=d["p_t"],
                        p_draft=d["p_d"], draft_tokens=d["toks"], u_accept=d["u_a"], u_sample=d["u_s"], chunks=dev_chunks,
                        scale=b.scale, out=st["out"], S_total_max=b.S_max, chunk_S_max=int(max(c.max() for c in chunks)),
                        use_plan=not args.no_plan)
    stream = torch.cuda.Stream()
    table = [dict() for _ in chunks]
    ev = {}
    with torch.cuda.stream(stream):
        # eager pass 1: what every chunk works on (read back between chunks; never part of a timed run)
        def look(stage, k, s):
            if stage != "attn_end":
                return
            stream.synchronize()
            ql = s.tsel["new_q_lens"].cpu().numpy().astype(np.int64)
            cc = s.chunk_ctx.cpu().numpy().astype(np.int64)
            act = ql > 0
            tok = (cc + ql)[act]
            table[k].update(rows=int(ql.sum()), requests=int(act.sum()), kv_tokens=int(tok.sum()),
                            attention_bytes_per_layer=int(2 * tok.sum() * b.H_kv * b.D * 2 + 2 * ql.sum() * b.H_q * b.D * 2 +
                                                          4 * ((tok + b.P - 1) // b.P).sum()))
        res = v.run(mark=look)
        stream.synchronize()
        # eager pass 2: HIP events around every chunk's attention layers
        for _ in range(2):
            def stamp(stage, k, s):
                if stage in ("attn_begin", "attn_end"):
                    e = torch.cuda.Event(enable_timing=True)
                    e.record(stream)
                    ev[(stage, k)] = e
            v.run(mark=stamp)
            stream.synchronize()
        for k in range(len(chunks)):
            us = ev[("attn_begin", k)].elapsed_time(ev[("attn_end", k)]) * 1e3 / args.layers
            table[k]["attention_us_per_layer"] = us
            table[k]["achieved_GBs"] = table[k]["attention_bytes_per_layer"] / us / 1e3 if us > 0 else 0.0
        # the timed region: the whole step as one graph
        run = v.run
        if not args.no_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                v.run()
            run = g.replay
        for _ in range(max(1, args.warmup)):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / args.steps, table, res, st, chunks


def cpu_baseline(b, n_layers):
    """The oracle as it stands, timed on this host: one layer of attention on the full batch
    (median of 3, scaled by the layer count) plus the accept and compaction steps at full size."""
    import oracle
    oracle.build()
    t_attn = []
    for _ in range(3):
        t0 = time.perf_counter()
        oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv,
                                D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
        t_attn.append(time.perf_counter() - t0)
    t0 = time.perf_counter()
    r = oracle.spec_accept(b.p_target, b.p_draft, b.draft_tokens, b.u_accept, b.u_sample, b.cu_q, b.cu_d, S_max=b.S_max)
    t_acc = time.perf_counter() - t0
    keep = (np.arange(b.N) - np.repeat(b.cu_q[:-1], b.spec_lens + 1) <= np.repeat(r["accepted_len"], b.spec_lens + 1))
    t0 = time.perf_counter()
    oracle.prune_compact(keep.astype(np.uint8), b.cu_q, suffix_close=True)
    t_pr = time.perf_counter() - t0
    t_step = n_layers * statistics.median(t_attn) + t_acc + t_pr
    return dict(value=float(b.spec_lens.sum()) / t_step, unit="tokens/s", cores=oracle.n_threads(), kind="oracle",
                sample=f"full batch; 1 of {n_layers} attention layers timed (median of 3 = "
                       f"{statistics.median(t_attn):.3f} s) and scaled by {n_layers}; accept ({t_acc * 1e3:.1f} ms) and "
                       f"compaction ({t_pr * 1e3:.2f} ms) at full size"), r


def overlap_measure(fsr, torch, workloads, b, n_layers, n_draft_cus, reps=5):
    """Sec. 3.3's spatial sharing on MI355X: the step's attention layers on a stream that owns all but
    ``n_draft_cus`` compute units, a stand-in drafter on a stream that owns the rest, each timed alone
    and both at once (eager launches, HIP events on each stream).  The stand-in drafter is the decode
    attention of a draft-model-shaped batch (8 query / 2 KV heads, D = 128, one row per request, the
    same context lengths, 8 layers with their own caches, 4 autoregressive steps): HBM-bound like the
    real one, without its GEMMs."""
    from paper_2604_20503_amd.streams import split_device

    def dev(x, bf16=False):
        t = torch.from_numpy(np.ascontiguousarray(x.view(np.int16) if bf16 else x)).cuda()
        return t.view(torch.bfloat16) if bf16 else t

    draft_s, verify_s = split_device(n_draft_cus)
    # verification side: the workload's own tensors, 8 distinct caches are enough to stay out of the last-level cache
    q, bt, ctx, spec, cu_q = dev(b.q, True), dev(b.block_tables), dev(b.ctx_lens), dev(b.spec_lens), dev(b.cu_q)
    k0, v0 = dev(b.k_cache, True), dev(b.v_cache, True)
    kv = [(k0, v0)] + [(torch.randn_like(k0, dtype=torch.float32).to(torch.bfloat16),
                        torch.randn_like(v0, dtype=torch.float32).to(torch.bfloat16)) for _ in range(7)]
    out = torch.empty_like(q)
    S = b.S_max + 1

    def ws_for(batch, mq):
        return torch.empty(max(256, fsr.attn_workspace_bytes(
            B=batch.B, N_cap=batch.N, H_q=batch.H_q, H_kv=batch.H_kv, D=batch.D, P=batch.P, max_pages=batch.max_pages,
            n_pages=batch.n_pages, dtype=torch.bfloat16, out_dtype=torch.bfloat16, max_q_len=mq)), dtype=torch.uint8, device="cuda")

    ws_v = ws_for(b, S)

    def verify(n_wg):
        for l in range(n_layers):
            k, v = kv[l % len(kv)]
            fsr.verify_attention(q, k, v, bt, ctx, spec, cu_q, scale=b.scale, out=out, workspace=ws_v, max_q_len=S,
                                 max_workgroups=n_wg)

    # drafter stand-in
    db = workloads.make_batch(2, rep=1, with_probs=False, H_q=8, H_kv=2, ctx_lens=b.ctx_lens, spec_lens=[0] * b.B)
    dq, dbt, dctx, dcu = dev(db.q, True), dev(db.block_tables), dev(db.ctx_lens), dev(db.cu_q)
    dk0, dv0 = dev(db.k_cache, True), dev(db.v_cache, True)
    dkv = [(dk0, dv0)] + [(torch.randn_like(dk0, dtype=torch.float32).to(torch.bfloat16),
                           torch.randn_like(dv0, dtype=torch.float32).to(torch.bfloat16)) for _ in range(7)]
    dout = torch.empty_like(dq)
    ws_d = ws_for(db, 1)

    def draft(n_wg):
        for _ in range(4):
            for k, v in dkv:
                fsr.verify_attention(dq, k, v, dbt, dctx, None, dcu, scale=db.scale, out=dout, workspace=ws_d, max_q_len=1,
                                     max_workgroups=n_wg)

    def timed(jobs):
        """jobs: list of (stream, fn).  Returns per-job mean ms with all jobs running at once."""
        for st, fn in jobs:  # warm-up
            with torch.cuda.stream(st):
                fn()
        torch.cuda.synchronize()
        acc = [0.0] * len(jobs)
        for _ in range(reps):
            ev = []
            for st, fn in jobs:
                a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                with torch.cuda.stream(st):
                    a.record(st)
                    fn()
                    e.record(st)
                ev.append((a, e))
            torch.cuda.synchronize()
            for i, (a, e) in enumerate(ev):
                acc[i] += a.elapsed_time(e) / reps
        return acc

    cur = torch.cuda.current_stream()
    n_all = draft_s.n_cus + verify_s.n_cus
    res = {"draft_cus": draft_s.n_cus, "verify_cus": verify_s.n_cus,
           "verify_ms_whole_device": timed([(cur, lambda: verify(0))])[0],
           "verify_ms_share_alone": timed([(verify_s.stream, lambda: verify(verify_s.n_cus))])[0],
           "draft_ms_whole_device": timed([(cur, lambda: draft(0))])[0],
           "draft_ms_share_alone": timed([(draft_s.stream, lambda: draft(draft_s.n_cus))])[0]}
    both = timed([(verify_s.stream, lambda: verify(verify_s.n_cus)), (draft_s.stream, lambda: draft(draft_s.n_cus))])
    res["verify_ms_share_concurrent"], res["draft_ms_share_concurrent"] = both
    res["serial_ms_whole_device"] = res["verify_ms_whole_device"] + res["draft_ms_whole_device"]
    res["concurrent_ms"] = max(both)
    res["note"] = (f"{n_all} compute units split by stream CU masks; stand-in drafter = decode attention of a "
                   "draft-shaped batch (8 q / 2 kv heads, 8 layers x 4 steps); eager launches")
    return res


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the committed counter summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
    scaled by a plain copy of known size) and the file it came from, or (None, None) if there is no summary for
    this kernel and workload.  A figure measured on an earlier build of the kernel is still that build's: the
    summary names the commit."""
    rel = os.path.join("profiles", f"{kernel}_cfg{workload}_hbm_traffic.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1]), rel
    except OSError:
        pass
    return None, None



def probe_table(fsr, torch, gib=2, reps=5):
    """--probe: GB/s of the plain-read probe in its three access patterns against the workgroup count (256
    workgroups = one per compute unit, 8 MB in flight; the attention kernel keeps up to 33 MB in flight)."""
    src = torch.zeros(gib << 30, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    table = {}
    with torch.cuda.stream(stream):
        for name, mode in (("front_to_back", 0), ("scattered_4k_blocks", 1), ("scattered_4k_blocks_as_64_byte_row_segments", 2)):
            for wg in (128, 256, 1024, 4096):
                sink = torch.empty(wg, dtype=torch.int64, device="cuda")
                fsr.hbm_read_probe(src, sink, wg, mode)
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
                for a, e in ev:
                    a.record(stream)
                    fsr.hbm_read_probe(src, sink, wg, mode)
                    e.record(stream)
                torch.cuda.synchronize()
                table.setdefault(name, {})[str(wg)] = round((gib << 30) / (statistics.mean(a.elapsed_time(e) for a, e in ev) * 1e-3) / 1e9, 1)
    return {"probe": "fsr_hbm_read_probe", "bytes": gib << 30, "unit": "GB/s", "by_workgroups": table}


def plain_read_rates(fsr, torch, gib=2, reps=5):
    """GB/s of fsr_hbm_read_probe (plain streaming loads over a buffer larger than the on-die caches), front
    to back and in scattered 4 KB blocks (how a paged cache with 16-token pages lays out one head's K or V),
    timed with HIP events on the launch stream: the practical ceilings next to which `achieved` is read."""
    src = torch.zeros(gib << 30, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    out = {}
    with torch.cuda.stream(stream):
        sink = fsr.hbm_read_probe(src)
        for name, scatter in (("plain_read_GBs", False), ("scattered_4k_read_GBs", True)):
            fsr.hbm_read_probe(src, sink, scatter_4k=scatter)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, e in ev:
                a.record(stream)
                fsr.hbm_read_probe(src, sink, scatter_4k=scatter)
                e.record(stream)
            torch.cuda.synchronize()
            out[name] = (gib << 30) / (statistics.mean(a.elapsed_time(e) for a, e in ev) * 1e-3) / 1e9
    del src
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0,
                    help="attention calls per step; default: 32 (Llama-3-8B depth), 80 for workload 4 (70B depth)")
    ap.add_argument("--workload", type=int, default=2, choices=[2, 3, 4, 5],
                    help="workload configuration; 2 (the default) is the one the metric is quoted on, the others "
                         "run the same one-shot step at their batch shapes")
    ap.add_argument("--chunked", action="store_true",
                    help="workloads 4 and 5: run the configuration's own chunked schedule (two chunks / frontiers of two "
                         "drafts with accept and row pruning after each) instead of the one-shot step")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-plan", action="store_true",
                    help="every attention launch rebuilds the step's schedule itself (fsr_verify_attention) instead of "
                         "reading the per-step plan (fsr_attn_plan + fsr_verify_attention_planned)")
    ap.add_argument("--overlap", type=int, default=0, metavar="N",
                    help="also measure the step's attention on a stream that owns all but N compute units next to a "
                         "stand-in drafter on a stream that owns those N (adds an \"overlap\" object to the JSON line)")
    ap.add_argument("--logits", action="store_true",
                    help="also time spec_accept in LOGITS mode on the step's rows (reported under kernels.spec_accept_logits)")
    ap.add_argument("--variants", action="store_true",
                    help="also time the other forms of the kernels on the step's shapes: attention over 8-bit caches, "
                         "K/V append, greedy acceptance, row restore (reported under kernels)")
    ap.add_argument("--probe", action="store_true", help="time only the plain-read probe (three access patterns) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that hardware byte counters of a "
                         "profiled run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.chunked and args.workload not in (4, 5):
        print("bench.py: --chunked is the schedule of workloads 4 and 5", file=sys.stderr)
        sys.exit(2)
    if args.layers <= 0:
        args.layers = 80 if args.workload == 4 else N_LAYERS

    import torch
    import paper_2604_20503_amd as fsr
    import workloads

    fsr.load_library()  # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    b = workloads.make_batch(args.workload, keep_logits=True) if args.logits else workloads.make_batch(args.workload)
    drafts = int(b.spec_lens.sum())
    attn_kernel = "attn_stream_kernel" if args.no_plan else "attn_planned_kernel"

    if args.probe:
        print(json.dumps(probe_table(fsr, torch)))
        return

    if args.calibrate_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.chunked:
        ms_per_step, table, res, st, chunks = chunked_run(args, fsr, torch, workloads, b)
        attn_bytes = sum(t["attention_bytes_per_layer"] for t in table)
        attn_us = sum(t["attention_us_per_layer"] for t in table)
        achieved = attn_bytes / attn_us / 1e3
        one_shot_bytes = b.attention_bytes()
        result = {
            "metric": "verified_draft_tokens_per_s", "value": drafts / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": WORKLOADS[args.workload].replace(", one-shot", "").replace(" shapes, one-shot", ""),
                       "schedule": f"chunked: {len(chunks)} chunks, accept + row pruning after each",
                       "layers_per_step": args.layers, "rows": b.N, "drafts_per_step": drafts,
                       "launch": "eager" if args.no_graph else "hip_graph", "seed": b.seed,
                       "distinct_kv_caches": st["n_caches"], "kv_cache_bytes": st["kv_bytes"],
                       "rows_computed": sum(t["rows"] for t in table),
                       "kv_bytes_read_vs_one_shot": attn_bytes / one_shot_bytes, "chunks": table},
            "roofline": {"bound": "hbm", "kernel": f"{attn_kernel} (verify_attention, one launch per layer and chunk; all chunks)",
                         "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                         "traffic": None, "algorithmic_bytes_per_launch": attn_bytes / len(table),
                         "launch_us": attn_us / len(table), **plain_read_rates(fsr, torch)},
        }
        if not args.no_cpu_baseline:
            base, ref = cpu_baseline(b, args.layers)
            result["cpu_baseline"] = base
            result["cpu_baseline"]["sample"] += "; the oracle's one-shot step (the chunked schedule emits the same tokens)"
            result["config"]["accept_matches_oracle"] = bool(
                np.array_equal(res["accepted_len"].cpu().numpy(), ref["accepted_len"]) and
                np.array_equal(res["n_emitted"].cpu().numpy(), ref["n_emitted"]))
            result["config"]["accepted_drafts_per_step"] = int(ref["accepted_len"].sum())
        print(json.dumps(result))
        return

    step, attn_only, tail, st = build_step(fsr, torch, b, args.layers, seed=2002, use_plan=not args.no_plan,
                                           variants=args.variants)
    stream = torch.cuda.Stream()
    graph = None
    with torch.cuda.stream(stream):
        for _ in range(max(1, args.warmup)):
            step()
        stream.synchronize()
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                step()
            graph.replay()
            stream.synchronize()
        run = graph.replay if graph is not None else step
        for _ in range(args.warmup):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        t1 = time.perf_counter()

        # Per-call figures: HIP events on the launch stream around a graph (or eager run) of that call alone,
        # once per timed repetition.  Dominant: attention, the layer loop divided by the layer count (with a
        # plan, the step's one plan launch is inside that figure).
        def timed(fn):
            runner = fn
            if graph is not None:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    fn()
                runner = g.replay
            runner()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for a, e in ev:
                a.record(stream)
                runner()
                e.record(stream)
            torch.cuda.synchronize()
            return statistics.mean(a.elapsed_time(e) for a, e in ev)

        attn_ms = timed(attn_only) / args.layers
        tail_ms = timed(tail)
        call_us = {name: timed(fn) * 1e3 for name, fn in st["calls"].items()}
        run()  # leave the step's own outcome in the buffers (the rank check above reuses the mask buffer)
        torch.cuda.synchronize()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = drafts / (ms_per_step * 1e-3)
    attn_bytes = b.attention_bytes()
    achieved = attn_bytes / (attn_ms * 1e-3) / 1e9
    traffic, traffic_src = measured_traffic(attn_kernel, args.workload)

    result = {
        "metric": "verified_draft_tokens_per_s", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.workload], "schedule": "one-shot",
                   "layers_per_step": args.layers, "rows": b.N, "drafts_per_step": drafts,
                   "kv_tokens": b.kv_tokens(), "launch": "hip_graph" if graph is not None else "eager",
                   "attention_ms_per_layer": attn_ms, "accept_prune_ms": tail_ms, "seed": b.seed,
                   "distinct_kv_caches": st["n_caches"], "kv_cache_bytes": st["kv_bytes"]},
        "roofline": {"bound": "hbm", "kernel": f"{attn_kernel} (verify_attention, one launch per layer call"
                                               + ("" if args.no_plan else "; the step's one attn_plan_kernel launch is inside the figure") + ")",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_src, "algorithmic_bytes_per_launch": attn_bytes,
                     "launch_us": attn_ms * 1e3, **plain_read_rates(fsr, torch)},
        "kernels": kernel_figures(b, st, call_us),
    }
    if args.overlap > 0:
        result["overlap"] = overlap_measure(fsr, torch, workloads, b, args.layers, args.overlap)
    if not args.no_cpu_baseline:
        base, ref = cpu_baseline(b, args.layers)
        result["cpu_baseline"] = base
        result["config"]["accept_matches_oracle"] = bool(
            np.array_equal(st["acc"].cpu().numpy(), ref["accepted_len"]) and
            np.array_equal(st["nem"].cpu().numpy(), ref["n_emitted"]))
        result["config"]["accepted_drafts_per_step"] = int(ref["accepted_len"].sum())
        result["config"]["paper_context"] = "paper reports up to +53% throughput / 1.92x lower latency end to end on H100 (context only)"
    print(json.dumps(result))


if __name__ == "__main__":
    main()
