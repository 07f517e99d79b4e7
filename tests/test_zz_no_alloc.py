"""GPU parity of fsr_verify_attention_static (the entry point that allocates nothing: its partial slots and
arrival words live in a buffer built into the library) against fsr_verify_attention, through the C ABI, on
two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_attention

pytestmark = pytest.mark.gpu


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else 0)


def test_static_scratch_entry_point_matches_workspace_entry_point(oracle):
    from paper_2604_20503_amd import binding as B
    lib = B.load_library()
    assert 16 << 20 < lib.fsr_static_scratch_bytes() < 32 << 20
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    cases = [dict(rep=41, ctx_lens=[1500, 45, 513, 128, 3000, 77, 2047, 900, 1, 0, 4000, 333], spec_lens=[8, 3, 6, 0, 2, 5, 8, 1, 4, 2, 7, 8]),
             dict(rep=42, ctx_lens=[700, 31, 260], spec_lens=[2, 0, 5])]          # second call: smaller input
    for n_call, kw in enumerate(cases):
        announce(f"fsr_verify_attention_static call {n_call}: B={len(kw['ctx_lens'])}")
        b = workloads.make_batch(2, with_probs=False, **kw)
        d = DeviceBatch(b, probs=False)
        p = B.AttnParams(B=b.B, N_cap=b.N, H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, max_pages=b.max_pages, n_pages=b.n_pages,
                         dtype=B.BF16, out_dtype=B.BF16, scale=float(b.scale), max_q_len=b.S_max + 1, max_workgroups=0, kv_layout=0)
        need = ctypes.c_size_t(0)
        assert lib.fsr_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(need)) == 0
        ws = torch.empty(need.value, dtype=torch.uint8, device="cuda")
        outs, lses = [], []
        for static in (False, True):
            out = torch.full((b.N, b.H_q, b.D), float("nan"), dtype=torch.bfloat16, device="cuda")
            lse = torch.full((b.N, b.H_q), float("nan"), dtype=torch.float32, device="cuda")
            if static:
                rc = lib.fsr_verify_attention_static(_ptr(d.q), _ptr(d.k_cache), _ptr(d.v_cache), _ptr(d.block_tables),
                                                     _ptr(d.ctx_lens), _ptr(d.cu_q), _ptr(out), _ptr(lse), ctypes.byref(p), stream)
            else:
                rc = lib.fsr_verify_attention(_ptr(d.q), _ptr(d.k_cache), _ptr(d.v_cache), _ptr(d.block_tables), _ptr(d.ctx_lens),
                                              None, _ptr(d.cu_q), _ptr(out), _ptr(lse), ctypes.byref(p), _ptr(ws),
                                              ctypes.c_size_t(need.value), stream)
            assert rc == 0, lib.fsr_last_error()
            torch.cuda.synchronize()
            outs.append(out)
            lses.append(lse)
        assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
        assert torch.equal(lses[0].view(torch.int32), lses[1].view(torch.int32))
        o_ref, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv,
                                           D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
        check_attention(outs[1], o_ref, "bf16", b.N)
    # shapes whose scratch would not fit are refused before any launch... none exist for the built kernels:
    # every stream-kernel shape needs at most the built-in size; the generic path needs no scratch
    g = B.AttnParams(B=2, N_cap=4, H_q=8, H_kv=2, D=64, P=16, max_pages=4, n_pages=8, dtype=B.F32, out_dtype=B.F32, scale=0.1,
                     max_q_len=2, max_workgroups=0, kv_layout=0)
    assert lib.fsr_verify_attention_static(None, None, None, None, None, None, None, None, ctypes.byref(g), stream) == -1
