"""The plain-read probe (measurement aid of bench.py) reads every byte exactly once: the XOR of its
per-workgroup words equals the XOR of the buffer's 64-bit words folded the way the kernel folds them."""
import numpy as np
import pytest
import torch

from gpu_utils import announce

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsr():
    import paper_2604_20503_amd as f
    f.load_library()
    return f


@pytest.mark.parametrize("mib,scatter", [(3, False), (4, True)])
def test_probe_reads_every_byte_once(fsr, mib, scatter):
    announce(f"fsr_hbm_read_probe: {mib} MiB, 7 workgroups, scatter={scatter}")
    rng = np.random.default_rng(5)
    host = rng.integers(0, 2 ** 32, size=(mib << 20) // 4, dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).cuda()
    sink = fsr.hbm_read_probe(src.view(torch.uint8), workgroups=7, scatter_4k=scatter)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint64))
    w = host.reshape(-1, 4)                      # 16-byte loads: words 0^2 -> high half, 1^3 -> low half
    hi = np.bitwise_xor.reduce(w[:, 0] ^ w[:, 2])
    lo = np.bitwise_xor.reduce(w[:, 1] ^ w[:, 3])
    assert got == (np.uint64(hi) << np.uint64(32)) | np.uint64(lo)


def test_probe_refuses_bad_sizes(fsr):
    src = torch.zeros(1000, dtype=torch.uint8, device="cuda")
    with pytest.raises(fsr.FsrError):
        fsr.hbm_read_probe(src)
    with pytest.raises(fsr.FsrError):
        fsr.hbm_read_probe(torch.zeros(3 << 15, dtype=torch.uint8, device="cuda"), scatter_4k=True)
