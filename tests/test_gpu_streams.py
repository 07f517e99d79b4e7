"""GPU: verification attention on compute-unit-masked streams (Sec. 3.3: drafting and verification
share the device spatially): results are those of an ordinary launch, alone and with another
masked stream busy at the same time."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import DeviceBatch, announce, check_attention

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


def test_masked_streams_alone_and_concurrently(fsr, oracle):
    from paper_2604_20503_amd.streams import split_device
    announce("attention on compute-unit-masked streams")
    b = workloads.make_batch(2, rep=51, with_probs=False, ctx_lens=[700, 45, 513, 128, 1500, 77, 2048, 300],
                             spec_lens=[8, 3, 6, 0, 2, 5, 7, 1])
    d = DeviceBatch(b, probs=False)
    o_ref, _ = oracle.verify_attention(b.q, b.k_cache, b.v_cache, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q,
                                       H_kv=b.H_kv, D=b.D, P=b.P, dtype=b.dtype, scale=b.scale)
    plain, _ = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens, d.cu_q,
                                    scale=b.scale, max_q_len=b.S_max + 1)
    torch.cuda.synchronize()
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    small, large = split_device(n_cus // 4)
    outs = {}
    for name, ms in (("small", small), ("large", large)):
        with torch.cuda.stream(ms.stream):
            outs[name], _ = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens, d.spec_lens,
                                                 d.cu_q, scale=b.scale, max_q_len=b.S_max + 1, max_workgroups=ms.n_cus)
        ms.stream.synchronize()
        check_attention(outs[name], o_ref, b.dtype, b.N)
    # both shares busy at once, several calls each
    both = {}
    for rep in range(4):
        for name, ms in (("small", small), ("large", large)):
            with torch.cuda.stream(ms.stream):
                both[name], _ = fsr.verify_attention(d.q, d.k_cache, d.v_cache, d.block_tables, d.ctx_lens,
                                                     d.spec_lens, d.cu_q, scale=b.scale, max_q_len=b.S_max + 1,
                                                     max_workgroups=ms.n_cus)
    torch.cuda.synchronize()
    for name in ("small", "large"):
        assert torch.equal(both[name].view(torch.int16), outs[name].view(torch.int16))
    assert plain.shape == outs["large"].shape
