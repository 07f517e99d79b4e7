"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
and reports host-detectable errors before launching anything (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2604_20503_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2604_20503_amd.build import build
        build()
    return binding.load_library()


def declared_symbols(header="faser_verify.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fsr_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2604_20503_amd import binding, controller
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == names
    ctl_names = declared_symbols("faser_controller.h")
    assert len(ctl_names) == 14
    for n in ctl_names:
        assert hasattr(lib, n), n
    assert sorted(controller.CTL_SYMBOLS) == ctl_names
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["faser_controller.h", "faser_verify.h"]


def test_struct_layouts_match_header():
    from paper_2604_20503_amd import binding
    assert ctypes.sizeof(binding.AttnParams) == 14 * 4
    assert ctypes.sizeof(binding.AcceptParams) == 32 and binding.AcceptParams.temperature.offset == 16
    assert ctypes.sizeof(binding.PruneParams) == 16
    assert ctypes.sizeof(binding.RankParams) == 7 * 4
    from paper_2604_20503_amd import controller
    assert ctypes.sizeof(controller.CtlConfig) == 4 * 19 + 4 + 6 * 8 and controller.CtlConfig.eps.offset == 80
    assert ctypes.sizeof(controller.LatencyModel) == 8 + 8 * 8


def test_host_detectable_errors(lib):
    from paper_2604_20503_amd import binding as b
    out = ctypes.c_size_t(0)
    ok = b.AttnParams(B=2, N_cap=8, H_q=32, H_kv=8, D=128, P=16, max_pages=4, n_pages=16, dtype=1, out_dtype=1,
                      scale=0.1, max_q_len=4, max_workgroups=0, kv_layout=0)
    assert lib.fsr_attn_workspace_bytes(ctypes.byref(ok), ctypes.byref(out)) == 0 and out.value > 0
    assert lib.fsr_attn_workspace_bytes(None, ctypes.byref(out)) == -1
    bad = b.AttnParams.from_buffer_copy(ok); bad.H_kv = 5
    assert lib.fsr_attn_workspace_bytes(ctypes.byref(bad), ctypes.byref(out)) == -2
    assert b"multiple" in lib.fsr_last_error()
    bad = b.AttnParams.from_buffer_copy(ok); bad.D = 96
    assert lib.fsr_attn_workspace_bytes(ctypes.byref(bad), ctypes.byref(out)) == -3
    bad = b.AttnParams.from_buffer_copy(ok); bad.dtype = 0; bad.out_dtype = 1
    assert lib.fsr_attn_workspace_bytes(ctypes.byref(bad), ctypes.byref(out)) == -3
    # null tensors are refused before any launch
    assert lib.fsr_verify_attention(None, None, None, None, None, None, None, None, None, ctypes.byref(ok), None,
                                    ctypes.c_size_t(0), None) == -1
    one = ctypes.c_void_p(256)  # never dereferenced: the workspace check comes first
    assert lib.fsr_verify_attention(one, one, one, one, one, None, one, one, None, ctypes.byref(ok), None,
                                    ctypes.c_size_t(0), None) == -4
    # which kernel a shape takes, and the plan calls' host checks
    assert lib.fsr_attn_path(ctypes.byref(ok)) == 1
    gen = b.AttnParams.from_buffer_copy(ok); gen.D = 64
    assert lib.fsr_attn_path(ctypes.byref(gen)) == 0
    gen = b.AttnParams.from_buffer_copy(ok); gen.dtype = 0; gen.out_dtype = 0
    assert lib.fsr_attn_path(ctypes.byref(gen)) == 0
    assert lib.fsr_attn_path(None) == -1
    assert lib.fsr_attn_plan_bytes(ctypes.byref(ok), ctypes.byref(out)) == 0 and out.value >= 33 * 128
    assert lib.fsr_attn_plan_bytes(ctypes.byref(gen), ctypes.byref(out)) == 0 and out.value == 0
    assert lib.fsr_attn_plan(one, one, one, ctypes.byref(gen), one, ctypes.c_size_t(1 << 20), None) == -3   # not the stream kernel
    assert lib.fsr_attn_plan(one, one, one, ctypes.byref(ok), one, ctypes.c_size_t(64), None) == -4         # buffer too small
    assert lib.fsr_attn_plan(one, one, None, ctypes.byref(ok), one, ctypes.c_size_t(1 << 20), None) == -1   # cu_q null
    ws = ctypes.c_size_t(0)
    assert lib.fsr_attn_workspace_bytes(ctypes.byref(ok), ctypes.byref(ws)) == 0
    assert lib.fsr_verify_attention_planned(one, one, one, one, one, one, one, None, ctypes.byref(ok), None, one, ws, None) == -1
    # a buffer in which no plan was built is refused before the launch
    assert lib.fsr_verify_attention_planned(one, one, one, one, one, one, one, None, ctypes.byref(ok), ctypes.c_void_p(4096),
                                            one, ws, None) == -1
    assert b"no plan" in lib.fsr_last_error()
    acc = b.AcceptParams(B=4, V=0, S_max=2, mode=0, temperature=1.0, dtype=0, reserved2=0)
    assert lib.fsr_accept_workspace_bytes(ctypes.byref(acc), ctypes.byref(out)) == -1
    acc.V = 1000; acc.mode = 7
    assert lib.fsr_accept_workspace_bytes(ctypes.byref(acc), ctypes.byref(out)) == -3
    acc.mode = 1; acc.temperature = 0.0
    assert lib.fsr_accept_workspace_bytes(ctypes.byref(acc), ctypes.byref(out)) == -1
    acc.mode = 0
    assert lib.fsr_accept_workspace_bytes(ctypes.byref(acc), ctypes.byref(out)) == 0
    assert lib.fsr_spec_accept(None, None, None, None, None, None, None, None, None, None, None, None,
                               ctypes.byref(acc), None, ctypes.c_size_t(0), None) == -1
    pr = b.PruneParams(B=-1, N_cap=4, suffix_close=1, reserved=0)
    assert lib.fsr_prune_compact(None, None, None, None, None, None, None, None, None, None, ctypes.c_size_t(0),
                                 ctypes.byref(pr), None) == -1
    pr.B = 2
    assert lib.fsr_prune_compact(None, one, one, one, one, one, one, one, one, one, ctypes.c_size_t(6),
                                 ctypes.byref(pr), None) == -1   # keep_mask null
    assert lib.fsr_prune_compact(one, one, one, one, one, one, one, one, one, ctypes.c_void_p(512), ctypes.c_size_t(6),
                                 ctypes.byref(pr), None) == -2   # row_bytes not a multiple of 4
    assert lib.fsr_prune_restore(one, one, one, None, ctypes.c_size_t(6), 4, 0, None) == -2
    assert lib.fsr_frontier_init(None, None, None, None, None, None, 3, 4, None) == -1
    assert lib.fsr_kv_append(None, one, one, one, one, one, one, ctypes.byref(ok), None) == -1   # k_new null
    rk = b.RankParams(B=2, N_cap=8, D_cap=6, V=0, K=10, dtype=0, reserved=0)
    assert lib.fsr_topk_rank_check(one, one, one, one, one, one, ctypes.byref(rk), None) == -1      # V = 0
    rk.V = 100; rk.dtype = 5
    assert lib.fsr_topk_rank_check(one, one, one, one, one, one, ctypes.byref(rk), None) == -3
    rk.dtype = 0
    assert lib.fsr_topk_rank_check(None, one, one, one, one, one, ctypes.byref(rk), None) == -1     # logits null
    rk.D_cap = 70000
    assert lib.fsr_topk_rank_check(one, one, one, one, one, one, ctypes.byref(rk), None) == -3
    assert lib.fsr_version().startswith(b"faser_verify")


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2604_20503_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()
