"""The MFMA-ceiling diagnostic runs, reports the flop it executes and leaves its operands alone."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_probe_runs_and_counts_flop():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    data = torch.randn(1 << 16, dtype=torch.bfloat16, device=dev)
    keep = data.clone()
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    ncu = torch.cuda.get_device_properties(dev).multi_processor_count
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.mlt_probe_mfma(64, data, sink)
    e0.record()
    flop = binding.mlt_probe_mfma(512, data, sink)
    e1.record()
    torch.cuda.synchronize()
    assert flop == ncu * 8 * 512 * 32 * 32768.0
    assert binding.mlt_last_kernel() == "mfma_rate_probe"
    assert torch.equal(data, keep)
    tflops = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    print("   probe: %.0f TFLOP/s on N(0,1) operands" % tflops, flush=True)
    assert 200.0 < tflops < 2600.0          # a loose sanity window around the chip's peak
    with pytest.raises(ValueError):
        binding.mlt_probe_mfma(16, data[:100], sink)
