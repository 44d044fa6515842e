"""GPU: the measurement library (libskiparse_probe.so): the MFMA-only kernel runs, reports its FLOP count and writes the sums of its accumulators."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_mfma_probe_runs_and_counts_flop():
    from paper_2605_28691_amd import probe

    ops = torch.zeros(8192, dtype=torch.bfloat16, device="cuda")
    ops[:] = 1.0  # every product is 1: an accumulator element after n MFMAs of depth 16 is 16 n
    sink = torch.full((16 * 256,), -1.0, dtype=torch.float32, device="cuda")
    flop = probe.mfma_probe(ops, sink, False, 16, 3)
    torch.cuda.synchronize()
    assert flop == 2.0 * 32 * 32 * 16 * 4 * 3 * 4 * 16
    # each thread sums 4 accumulators x 16 registers, every register = 16 * 3
    assert bool((sink == 4 * 16 * 16 * 3).all())
    # fp8: 0x38 is 1.0 in E4M3; depth 64
    ops8 = torch.full((16384,), 0x38, dtype=torch.uint8, device="cuda")
    flop8 = probe.mfma_probe(ops8, sink, True, 16, 2)
    torch.cuda.synchronize()
    assert flop8 == 2.0 * 32 * 32 * 64 * 4 * 2 * 4 * 16
    assert bool((sink == 4 * 16 * 64 * 2).all())


def test_mfma_valu_probe_runs():
    from paper_2605_28691_amd import probe

    ops = torch.zeros(8192, dtype=torch.bfloat16, device="cuda")
    sink = torch.full((8 * 256,), -1.0, dtype=torch.float32, device="cuda")
    for n in (0, 2, 4, 6, 8):
        flop = probe.mfma_valu_probe(ops, sink, n, 8, 5)
        assert flop == 2.0 * 32 * 32 * 16 * 2 * 5 * 4 * 8
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())


def test_mfma_lds_probe_runs_and_counts_flop():
    from paper_2605_28691_amd import probe

    ops = torch.ones(8192, dtype=torch.bfloat16, device="cuda")  # every product is 1
    sink = torch.full((8 * 256,), -1.0, dtype=torch.float32, device="cuda")
    flop = probe.mfma_lds_probe(ops, sink, 8, 6)
    torch.cuda.synchronize()
    assert flop == 2.0 * 32 * 32 * 16 * 8 * 6 * 4 * 8
    # 8 MFMAs of depth 16 per iteration spread over 4 accumulators: every register = 16 * 2 * 6; a thread sums 4 x 16 registers
    assert bool((sink == 4 * 16 * 16 * 2 * 6).all())


def test_device_info_reports_the_mi355x():
    from paper_2605_28691_amd import probe

    cu, khz = probe.device_info(0)
    assert cu == torch.cuda.get_device_properties(0).multi_processor_count
    assert 1_000_000 <= khz <= 3_000_000  # nominal engine clock in kHz (2.4 GHz on MI355X)


def test_lds_read_probe_runs_and_counts_bytes():
    from paper_2605_28691_amd import probe

    ops = torch.ones(8192, dtype=torch.bfloat16, device="cuda")
    sink = torch.full((4 * 512,), -1.0, dtype=torch.float32, device="cuda")
    for kind, per_read in ((0, 1024), (1, 512), (2, 512)):
        nbytes = probe.lds_read_probe(ops, sink, kind, 4, 3)
        assert nbytes == per_read * 16 * 3 * 8 * 4
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all()) and bool((sink >= 0).all())


def test_mfma8_valu_probe_runs():
    from paper_2605_28691_amd import probe

    ops = torch.zeros(16384, dtype=torch.uint8, device="cuda")
    sink = torch.full((8 * 256,), -1.0, dtype=torch.float32, device="cuda")
    for n in (0, 4, 8, 12, 16):
        assert probe.mfma8_valu_probe(ops, sink, n, 8, 5) == 2.0 * 32 * 32 * 64 * 2 * 5 * 4 * 8
    for chain in (1, 2, 4, 8):
        assert probe.mfma_chain_probe(ops.view(torch.bfloat16), sink, chain, 8, 5) == 2.0 * 32 * 32 * 16 * 4 * chain * 5 * 4 * 8
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())
