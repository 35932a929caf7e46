"""The diagnostic kernels behind bench.py's measured ceilings: the read stream must really read every byte
it is credited with (its per-wave XOR is checked against torch's), and both reject what they cannot run."""
import pytest
import torch

import paper_2401_14112_amd as pkg

pytestmark = pytest.mark.gpu


def _xor_over(t, dim):
    """XOR-reduce an int32 tensor along one dimension."""
    t = t.movedim(dim, -1)
    while t.shape[-1] > 1:
        h = t.shape[-1] // 2
        rest = t[..., 2 * h:]
        t = t[..., :h] ^ t[..., h:2 * h]
        if rest.shape[-1]:
            t = torch.cat([t, rest], dim=-1)
    return t[..., 0]


@pytest.mark.parametrize("mib", [16, 80, 129])
def test_read_stream_reads_every_byte(mib):
    g = torch.Generator(device="cuda").manual_seed(mib)
    buf = torch.randint(0, 256, ((mib << 20) + 4096,), dtype=torch.uint8, device="cuda", generator=g)[: mib << 20]
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    n = pkg.fp6_probe_read(buf, sink)
    assert n % (1024 * 16384) == 0 and n <= buf.numel() and buf.numel() - n < 1024 * 16384
    # pieces of 8 KB (2048 words); wave w reads pieces w, 1024 + w, ...
    want = _xor_over(_xor_over(buf[:n].view(torch.int32).view(n // (1024 * 8192), 1024, 2048), 2), 0)
    torch.cuda.synchronize()
    assert torch.equal(sink, want)


def test_read_stream_rejects_short_buffers():
    buf = torch.zeros((16 << 20) - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6_probe_read(buf)


def test_matrix_loop_runs_and_rejects_bad_counts():
    sink = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    assert pkg.fp6_probe_mfma(3, sink) == 4096.0 * 3 * 4 * 32768.0
    torch.cuda.synchronize()
    assert torch.isfinite(sink.view(torch.float32)[: 4096 * 64]).all()
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6_probe_mfma(0, sink)
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6_probe_mfma(3, torch.zeros(16, dtype=torch.uint8, device="cuda"))
