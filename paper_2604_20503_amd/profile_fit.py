"""Offline profiling (Sec. 3.4) on this machine: time the verification kernels over batch size b, speculative
length s and compute-unit share, and fit the latency models of Eqs. 12-14 to the measurements.

    python -m paper_2604_20503_amd.profile_fit [--reps 10] [--out FILE]

Target side (Eq. 12): one layer's ``verify_attention`` over b requests with s drafted tokens each, on a stream
that owns a (1 - r) share of the compute units.  Early-exit check (Eq. 13): ``topk_rank_check`` over the b s
drafted rows, same share.  Pruning (Eq. 14): ``prune_compact`` with a hidden-state payload, on the r share.
Inputs are synthetic (random caches, context lengths 1-4 K tokens); the drafter's model (Eq. 11) needs a draft
model and is not measured here.  Prints one JSON object with the fitted parameters and the relative error.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--out", default=None)
    ap.add_argument("--batches", default="16,64,128")
    ap.add_argument("--lengths", default="2,4,8")
    ap.add_argument("--shares", default="0.25,0.5,0.75,1.0", help="share of the compute units the timed side owns")
    args = ap.parse_args(argv)

    import torch

    import paper_2604_20503_amd as fsr
    from paper_2604_20503_amd import controller as ctl
    from paper_2604_20503_amd.streams import MaskedStream

    if not torch.cuda.is_available():
        print("profile_fit needs a GPU", file=sys.stderr)
        return 2
    fsr.load_library()
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    H_q, H_kv, D, P, V, hidden = 32, 8, 128, 16, 128256, 4096
    batches = [int(v) for v in args.batches.split(",")]
    lengths = [int(v) for v in args.lengths.split(",")]
    shares = [float(v) for v in args.shares.split(",")]
    rng = np.random.default_rng(0)
    streams = {x: MaskedStream(range(max(1, round(x * n_cus)))) for x in shares}

    def timed(stream, fn):
        with torch.cuda.stream(stream):
            fn()
            stream.synchronize()
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(args.reps):
                fn()
            e.record(stream)
            e.synchronize()
        return a.elapsed_time(e) / args.reps * 1e3  # us

    points = {"target": [], "exit": [], "prune": []}
    for b in batches:
        ctx = rng.integers(1024, 4096, size=b).astype(np.int32)
        for s in lengths:
            q_len = s + 1
            pages_per = (ctx + q_len + P - 1) // P
            max_pages, n_pages = int(pages_per.max()), int(pages_per.sum())
            perm = rng.permutation(n_pages).astype(np.int32)
            bt = np.zeros((b, max_pages), np.int32)
            o = 0
            for i in range(b):
                bt[i, :pages_per[i]] = perm[o:o + pages_per[i]]
                o += pages_per[i]
            N = b * q_len
            cu_q = torch.arange(0, N + 1, q_len, dtype=torch.int32, device="cuda")
            cu_d = torch.arange(0, b * s + 1, s, dtype=torch.int32, device="cuda")
            q = torch.randn(N, H_q, D, device="cuda").to(torch.bfloat16)
            # two cache sets, alternated, so that a repetition does not find the previous one's lines in the last-level cache
            kv = [(torch.randn(n_pages, H_kv, P, D, device="cuda").to(torch.bfloat16),
                   torch.randn(n_pages, H_kv, P, D, device="cuda").to(torch.bfloat16)) for _ in range(2)]
            bt_d, ctx_d = torch.from_numpy(bt).cuda(), torch.from_numpy(ctx).cuda()
            spec_d = torch.full((b,), s, dtype=torch.int32, device="cuda")
            out = torch.empty_like(q)
            ws = torch.empty(max(256, fsr.attn_workspace_bytes(B=b, N_cap=N, H_q=H_q, H_kv=H_kv, D=D, P=P, max_pages=max_pages,
                                                               n_pages=n_pages, dtype=torch.bfloat16, out_dtype=torch.bfloat16,
                                                               max_q_len=q_len)), dtype=torch.uint8, device="cuda")
            logits = torch.randn(N, V, device="cuda").to(torch.bfloat16)
            drafts = torch.randint(0, V, (b * s,), dtype=torch.int32, device="cuda")
            rank = torch.empty(b * s, dtype=torch.int32, device="cuda")
            keep = torch.empty(N, dtype=torch.uint8, device="cuda")
            keep_in = (torch.rand(N, device="cuda") < 0.7).to(torch.uint8)
            payload = torch.randn(N, hidden, device="cuda").to(torch.bfloat16)
            payload_out = torch.empty_like(payload)
            flip = [0]

            for x in shares:
                st = streams[x]
                n_wg = st.n_cus

                def attention():
                    k, v = kv[flip[0] & 1]
                    flip[0] += 1
                    fsr.verify_attention(q, k, v, bt_d, ctx_d, spec_d, cu_q, scale=D ** -0.5, out=out, workspace=ws,
                                         max_q_len=q_len, max_workgroups=n_wg)

                t = timed(st.stream, attention)
                points["target"].append((b, s, 1.0 - x, t))
                t = timed(st.stream, lambda: fsr.topk_rank_check(logits, drafts, cu_q, cu_d, K=10, rank=rank, keep_mask=keep))
                points["exit"].append((b, s, 1.0 - x, t))
                t = timed(st.stream, lambda: fsr.prune_compact(keep_in, cu_q, payload=payload, payload_out=payload_out))
                points["prune"].append((b, s, x, t))
            print(f"profiled b={b} s={s}", file=sys.stderr, flush=True)

    # the attention call is fitted twice: with Eq. 12's base and with the base that has a term in b alone
    points["target_kv"] = points["target"]
    forms = {"target": ctl.LAT_TARGET, "target_kv": ctl.LAT_KV, "exit": ctl.LAT_EXIT, "prune": ctl.LAT_PRUNE}
    result = {"device_compute_units": n_cus, "reps": args.reps, "unit": "us", "models": {}}
    for name, pts in points.items():
        b_, s_, r_, T_ = (list(v) for v in zip(*pts))
        model, rms = ctl.latency_fit(forms[name], b_, s_, r_, T_)
        pred = np.array([ctl.latency_eval(model, *p[:3]) for p in pts])
        rel = np.abs(pred - np.array(T_)) / np.array(T_)
        result["models"][name] = {
            "a1": model.a1, "g1": model.g1, "a2": model.a2, "g2": model.g2, "knee": model.knee,
            "alpha": model.alpha, "beta": model.beta, "c": model.c, "rms_us": rms,
            "mean_rel_err": float(rel.mean()), "max_rel_err": float(rel.max()),
            "points": [[int(p[0]), int(p[1]), round(p[2], 4), round(p[3], 2)] for p in pts],
        }
    text = json.dumps(result)
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
