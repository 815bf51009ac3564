"""GPU: the device-ceiling diagnostics run, the copy is bit-exact, and the matrix-instruction probe reports the
operation count its launch shape implies.  No rate is asserted here (the bench reports the rates)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_probe_copy_is_bit_exact_with_ragged_tail(gpu_lib):
    n = 16 * (4 * 256 * 3 + 5)                      # three whole workgroups of vectors and a partial one
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.full((n + 64,), 7, dtype=torch.uint8, device="cuda")
    gpu_lib.probe_copy(dst[:n], src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and bool((dst[n:] == 7).all())


def test_probe_read_and_mfma_run(gpu_lib):
    src = torch.randint(0, 256, (1 << 20,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros((4,), dtype=torch.float32, device="cuda")
    gpu_lib.probe_read(src, sink)
    for kind in (0, 1):
        flops = gpu_lib.probe_mfma_bf16(10, kind, sink)
        assert flops == 2 * 256 * 4 * 10 * 8 * (2 * 16 * 16 * 32)
    torch.cuda.synchronize()
    assert bool((sink == 0).all())
