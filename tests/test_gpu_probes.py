"""The measurement probes of the library run and leave their buffers as documented (they carry none of the method's
arithmetic; bench.py quotes their timings as second denominators)."""
import pytest
import torch

import paper_2605_08587_amd as kla

pytestmark = pytest.mark.gpu


def test_inplace_probe_doubles_the_buffer():
    x = torch.full((1 << 16,), 1.5, dtype=torch.float32, device="cuda")
    kla.kla_debug_peak_probe(0, x, iters=1)
    kla.kla_debug_peak_probe(0, x, iters=0)
    torch.cuda.synchronize()
    assert torch.all(x == 6.0)


def test_read_probe_sums_the_buffer():
    x = torch.ones((1 << 16,), dtype=torch.float32, device="cuda")
    aux = torch.zeros(x.numel() * 4 // 16384, dtype=torch.float32, device="cuda")
    kla.kla_debug_peak_probe(1, x, aux)
    torch.cuda.synchronize()
    assert float(aux.sum()) == float(x.numel())


@pytest.mark.parametrize("n,depth", [(16, 1), (16, 2), (60, 1), (60, 2)])
def test_ring_copy_probe_runs_and_leaves_its_source_alone(n, depth):
    buf = torch.arange(n << 20, dtype=torch.int32, device="cuda")          # n x 4 MiB
    ref = buf.clone()
    kla.kla_debug_peak_probe(3, buf, iters=n + 256 * (depth - 1))
    torch.cuda.synchronize()
    assert torch.equal(buf, ref)
    with pytest.raises(kla.KlaError):
        kla.kla_debug_peak_probe(3, buf[: buf.numel() // 2], iters=n + 256 * (depth - 1))
