"""The entry points enqueue on the stream they are given and nothing else: results on a side stream
are those of the default stream, and a captured step (GEMM, attention forward, paged decode)
replays to the eager result every time."""
import math

import numpy as np
import pytest
import torch

from paper_2503_14985_amd import inputs
import parity_util as pu

pytestmark = pytest.mark.gpu
BF16 = inputs.BF16


@pytest.fixture(autouse=True)
def _announce(request):
    print("\n[case] %s" % request.node.name, flush=True)
    yield


def _problem(dev, seed):
    """One small problem per entry point, each big enough for several workgroups and tiles."""
    A_h, B_h = inputs.gemm_inputs(520, 776, 320, BF16, seed)
    Q_h, K_h, V_h = inputs.mha_inputs(2, 3, 300, 455, 128, BF16, seed)
    lens = [1, 37, 300, 130]
    q_h, kc_h, vc_h, table, seq_lens, _, _ = inputs.paged_inputs(4, 2, 128, 16, lens, BF16, seed)
    t = lambda x: inputs.bits_to_torch(x, BF16, dev)
    return {
        "host": (A_h, B_h, Q_h, K_h, V_h),
        "A": t(A_h), "B": t(B_h), "Q": t(Q_h), "K": t(K_h), "V": t(V_h),
        "q": t(q_h), "kc": t(kc_h), "vc": t(vc_h),
        "table": torch.from_numpy(table).to(dev), "lens": torch.from_numpy(seq_lens).to(dev),
    }


def _run(binding, p, out):
    binding.mlt_gemm(p["A"], p["B"], C=out["C"])
    binding.mlt_mha_fwd(p["Q"], p["K"], p["V"], 1.0 / math.sqrt(128), causal=True, O=out["O"])
    binding.mlt_paged_attn_decode(p["q"], p["kc"], p["vc"], p["table"], p["lens"], 1.0 / math.sqrt(128),
                                  O=out["o"])


def _outputs(p):
    return {"C": torch.empty((p["A"].shape[0], p["B"].shape[1]), dtype=torch.bfloat16, device=p["A"].device),
            "O": torch.empty_like(p["Q"]), "o": torch.empty_like(p["q"])}


def _same(a, b):
    return all(torch.equal(a[k].view(torch.int16), b[k].view(torch.int16)) for k in a)


def test_side_stream_matches_default_stream():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    p = _problem(dev, 3)
    ref = _outputs(p)
    _run(binding, p, ref)
    torch.cuda.synchronize()
    # parity of the default-stream result with the oracle (the GEMM and the attention forward)
    A_h, B_h, Q_h, K_h, V_h = p["host"]
    pu.check_gemm(A_h, B_h, ref["C"], BF16, False, seed=3)
    pu.check_mha(Q_h, K_h, V_h, ref["O"], 1.0 / math.sqrt(128), True, BF16, seed=3)

    side = torch.cuda.Stream(device=dev)          # default priority
    out = _outputs(p)
    for k in out:
        out[k].fill_(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        _run(binding, p, out)                     # the binding takes torch's current stream
        done = torch.cuda.Event()
        done.record(side)
    done.synchronize()                            # only the side stream's work is waited for
    assert _same(out, ref)
    # an explicit stream argument (GEMM and attention take one)
    out2 = _outputs(p)
    binding.mlt_gemm(p["A"], p["B"], C=out2["C"], stream=side)
    binding.mlt_mha_fwd(p["Q"], p["K"], p["V"], 1.0 / math.sqrt(128), causal=True, O=out2["O"], stream=side)
    side.synchronize()
    assert torch.equal(out2["C"].view(torch.int16), ref["C"].view(torch.int16))
    assert torch.equal(out2["O"].view(torch.int16), ref["O"].view(torch.int16))


def test_captured_step_replays_to_the_eager_result():
    """Capture one step into a HIP graph (on these shapes the entry points launch only kernels and
    need no scratch of the library's own; the captured form of a call that does is
    mlt_gemm_noalloc, tested with its own file), replay it several times with eager work and synchronisations in between and with new
    input contents, and compare every replay with the eager result on the same contents."""
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    p = _problem(dev, 5)
    eager = _outputs(p)
    _run(binding, p, eager)                       # also the warm-up: per-kernel attributes are set here
    torch.cuda.synchronize()

    static = _outputs(p)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _run(binding, p, static)
    other = _problem(dev, 6)
    for rep in range(4):
        if rep == 2:
            # new contents in the captured input buffers
            for k in ("A", "B", "Q", "K", "V", "q", "kc", "vc"):
                p[k].copy_(other[k])
            _run(binding, p, eager)
            torch.cuda.synchronize()
        for k in static:
            static[k].fill_(0)
        graph.replay()
        # eager work of the program's own between the replays
        scratch = _outputs(other)
        _run(binding, other, scratch)
        torch.cuda.synchronize()
        assert _same(static, eager), "replay %d differs from the eager result" % rep


def test_capture_on_a_stream_without_scratch_does_not_allocate():
    """A GEMM that would split K across workgroups, captured on a stream the library has no scratch
    buffer for: the call must not allocate in the middle of the capture; it runs without the split
    (the kernel name says so) and the replays meet the oracle bound."""
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    M, N, K = 64, 2048, 64 * 160
    A_h, B_h = inputs.gemm_inputs(M, N, K, BF16, 9, transB=True, std=0.02)
    A, B = inputs.bits_to_torch(A_h, BF16, dev), inputs.bits_to_torch(B_h, BF16, dev)
    eager = binding.mlt_gemm(A, B, transB=True)
    assert "splitk" in binding.mlt_last_kernel()
    torch.cuda.synchronize()
    static = torch.empty_like(eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                   # records on a fresh side stream
        binding.mlt_gemm(A, B, C=static, transB=True)
        captured_name = binding.mlt_last_kernel()
    assert "splitk" not in captured_name, captured_name
    for rep in range(3):
        static.fill_(0)
        graph.replay()
        binding.mlt_gemm(A, B, transB=True)          # eager work between the replays
        torch.cuda.synchronize()
        pu.check_gemm(A_h, B_h, static, BF16, True, seed=9)
