"""The streaming probe (measurement helper of the benchmark): it reads what it is told to read and writes what
it is told to write, nothing else; and the register-only MFMA loop launches."""
import pytest
import torch

from paper_2401_04658_amd import bench_probe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.mark.parametrize("nts", [False, True])
@pytest.mark.parametrize("reads,writes", [(3, 1), (4, 2), (1, 1), (0, 2), (2, 0)])
def test_streams(reads, writes, nts):
    unit = 1 << 20
    src = torch.zeros(4 * unit // 4, dtype=torch.float32, device=DEV)
    for r in range(4):
        src[r * unit // 4:(r + 1) * unit // 4] = float(r + 1)
    guard = 4096
    dst = torch.full(((2 * unit + guard) // 4,), -7.0, dtype=torch.float32, device=DEV)
    bench_probe.stream_probe(reads, writes, src.view(torch.uint8), dst.view(torch.uint8), unit, nt_stores=nts)
    torch.cuda.synchronize()
    # every lane starts from (1, 2, 3, 4), adds one element of each stream read, scales by the output stream's index
    base = torch.tensor([1.0, 2.0, 3.0, 4.0], device=DEV).repeat(unit // 16) + float(sum(range(1, reads + 1)))
    for w in range(2):
        got = dst[w * unit // 4:(w + 1) * unit // 4]
        if w < writes:
            assert torch.equal(got, base * float(w + 1))
        else:
            assert torch.all(got == -7.0)
    assert torch.all(dst[2 * unit // 4:] == -7.0)


def test_mfma_peak_launches():
    sink = torch.zeros(16, dtype=torch.float32, device=DEV)
    flops = bench_probe.mfma_peak(64, 100, sink)
    torch.cuda.synchronize()
    assert flops == 64 * 4 * 100 * 16 * 32768
    assert torch.all(sink == 0)
