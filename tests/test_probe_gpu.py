"""The ceiling diagnostics run, report the work they do and leave their inputs alone."""
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
    # the 16x16x32 form executes the same flop count
    assert binding.mlt_probe_mfma16(512, data, sink) == flop
    assert binding.mlt_last_kernel() == "mfma16_rate_probe"
    torch.cuda.synchronize()
    assert torch.equal(data, keep)


def test_hbm_read_probe_runs():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    # 1 GiB + a ragged tail of 16-byte words: far beyond L2 and the 256 MiB last-level cache
    data = torch.randint(0, 2 ** 31 - 1, ((1 << 28) + 4 * 37,), dtype=torch.int32, device=dev)
    head = data[:4096].clone()
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.mlt_probe_hbm_read(data, sink)
    e0.record()
    nbytes = binding.mlt_probe_hbm_read(data, sink)
    e1.record()
    torch.cuda.synchronize()
    assert nbytes == data.numel() * 4
    assert binding.mlt_last_kernel() == "hbm_read_probe"
    assert torch.equal(data[:4096], head) and int(sink.abs().sum()) == 0
    gbs = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    print("   probe: %.0f GB/s read" % gbs, flush=True)
    assert 500.0 < gbs < 8200.0             # a loose sanity window below the 8 TB/s peak
    binding.mlt_probe_hbm_read(data[:4], sink)                    # a single 16-byte word
    with pytest.raises(binding.MltError):
        binding.mlt_probe_hbm_read(data[:3], sink)                # 12 bytes
