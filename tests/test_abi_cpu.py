"""Host-only checks of the C ABI: the library loads, exports what include/mlt.h declares, rejects
bad arguments before touching a device, and answers the host-side tiling query. No kernel runs."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mlt.h")
DIAG_HEADER = os.path.join(ROOT, "include", "mlt_diag.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2503_14985_amd import binding as b
    return b


def declared_functions(header):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mlt_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(binding):
    names = declared_functions(HEADER)
    assert {"mlt_gemm", "mlt_mha_fwd", "mlt_status_string", "mlt_version"} <= set(names)
    diag = declared_functions(DIAG_HEADER)
    # the operations' header carries no diagnostics
    assert not [n for n in names if "probe" in n or "diag" in n or "timing" in n or "query" in n]
    lib = binding.raw()
    for n in names + diag:
        assert hasattr(lib, n), "libmlt.so does not export %s" % n
    assert sorted(binding.EXPORTS) == names
    assert sorted(binding.DIAG_EXPORTS) == diag


def test_kernel_choice_overrides(binding):
    """mlt_diag_force_variant: host-side state only; unknown names are rejected and change nothing;
    the tiling query reports the MFMA shape of the attention variant in force."""
    try:
        binding.mlt_diag_force_variant(mha="pp16")
        assert binding.mlt_query_tiling(1, (4096, 4096, 128, 0), 0)[6:9] == [16, 16, 32]
        with pytest.raises(binding.MltError):
            binding.mlt_diag_force_variant(mha="no-such-kernel")
        assert binding.mlt_query_tiling(1, (4096, 4096, 128, 0), 0)[6:9] == [16, 16, 32]
        binding.mlt_diag_force_variant(mha="auto")
        assert binding.mlt_query_tiling(1, (4096, 4096, 128, 0), 0)[6:9] == [32, 32, 16]
        binding.mlt_diag_force_variant(gemm="64k4")
        assert binding.mlt_query_tiling(0, (8192, 8192, 8192, 0), 0)[0:2] == [64, 64]
        with pytest.raises(binding.MltError):
            binding.mlt_diag_force_variant(gemm="256pp")        # retired name
        with pytest.raises(binding.MltError):
            binding.mlt_diag_set_persistent_grid(-1)
    finally:
        binding.mlt_diag_force_variant(gemm="auto", mha="auto")
        binding.mlt_diag_set_persistent_grid(0)
    assert binding.mlt_query_tiling(0, (8192, 8192, 8192, 0), 0)[0:2] == [256, 256]


def test_status_strings_and_version(binding):
    assert binding.mlt_status_string(0) == "ok"
    seen = {binding.mlt_status_string(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5
    assert binding.mlt_status_string(-99) == "unknown status"
    assert re.fullmatch(r"\d+\.\d+\.\d+", binding.mlt_version())


def test_gemm_argument_validation_without_device(binding):
    lib = binding.raw()
    p = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    null = ctypes.c_void_p(0)
    g = lib.mlt_gemm
    assert g(-1, 8, 8, p, 8, p, 8, 0, p, 8, 0, None) == binding.MLT_ERR_INVALID_ARG
    assert g(8, 8, 8, p, 8, p, 8, 0, p, 8, 7, None) == binding.MLT_ERR_INVALID_ARG      # dtype
    assert g(8, 8, 8, null, 8, p, 8, 0, p, 8, 0, None) == binding.MLT_ERR_INVALID_ARG   # A null
    assert g(8, 8, 8, p, 8, p, 8, 0, null, 8, 0, None) == binding.MLT_ERR_INVALID_ARG   # C null
    assert g(8, 8, 16, p, 8, p, 8, 0, p, 8, 0, None) == binding.MLT_ERR_INVALID_ARG     # lda < K
    assert g(8, 16, 8, p, 8, p, 8, 0, p, 16, 0, None) == binding.MLT_ERR_INVALID_ARG    # ldb < N
    assert g(8, 16, 8, p, 8, p, 4, 1, p, 16, 0, None) == binding.MLT_ERR_INVALID_ARG    # ldb < K (transB)
    assert g(8, 16, 8, p, 8, p, 16, 0, p, 8, 0, None) == binding.MLT_ERR_INVALID_ARG    # ldc < N
    assert g(0, 16, 8, null, 8, null, 16, 0, null, 16, 0, None) == binding.MLT_OK       # M = 0: no-op
    assert g(8, 0, 8, null, 8, null, 16, 0, null, 16, 1, None) == binding.MLT_OK        # N = 0: no-op


def test_tiling_hint_argument_validation_without_device(binding):
    lib = binding.raw()
    p = ctypes.c_void_p(0x1000)
    t = lib.mlt_gemm_tiled
    assert t(8, 8, 8, p, 8, p, 8, 0, p, 8, 0, 4, None) == binding.MLT_ERR_INVALID_ARG     # unknown tiling
    assert t(8, 8, 8, p, 8, p, 8, 0, p, 8, 0, -1, None) == binding.MLT_ERR_INVALID_ARG
    assert t(8, 8, 8, None, 8, p, 8, 0, p, 8, 0, 1, None) == binding.MLT_ERR_INVALID_ARG  # A null
    assert t(0, 8, 8, None, 8, None, 8, 0, None, 8, 0, 2, None) == binding.MLT_OK         # M = 0: no-op


def test_probe_argument_validation_without_device(binding):
    lib = binding.raw()
    p = ctypes.c_void_p(0x1000)
    flop = ctypes.c_double()
    f = lib.mlt_probe_mfma
    assert f(0, p, p, ctypes.byref(flop), None) == binding.MLT_ERR_INVALID_ARG          # iters < 1
    assert f(1 << 21, p, p, ctypes.byref(flop), None) == binding.MLT_ERR_INVALID_ARG    # iters too large
    assert f(16, None, p, ctypes.byref(flop), None) == binding.MLT_ERR_INVALID_ARG      # data null
    assert f(16, p, None, ctypes.byref(flop), None) == binding.MLT_ERR_INVALID_ARG      # sink null
    assert f(16, p, p, None, None) == binding.MLT_ERR_INVALID_ARG                       # flop null
    assert lib.mlt_probe_mfma16(0, p, p, ctypes.byref(flop), None) == binding.MLT_ERR_INVALID_ARG
    assert lib.mlt_probe_mfma16(16, None, p, ctypes.byref(flop), None) == binding.MLT_ERR_INVALID_ARG
    r = lib.mlt_probe_hbm_read
    assert r(None, 1024, p, None) == binding.MLT_ERR_INVALID_ARG                        # data null
    assert r(p, 1024, None, None) == binding.MLT_ERR_INVALID_ARG                        # sink null
    assert r(p, 0, p, None) == binding.MLT_ERR_INVALID_ARG                              # empty
    assert r(p, 1000, p, None) == binding.MLT_ERR_INVALID_ARG                           # not a multiple of 16
    assert r(ctypes.c_void_p(0x1008), 1024, p, None) == binding.MLT_ERR_INVALID_ARG     # misaligned


def test_skinny_shapes_are_routed_by_the_tiling_query(binding):
    # M <= 64 with B stored N x K and enough columns: 16-column workgroups, 16x16x32 MFMA
    t = binding.mlt_query_tiling(0, (16, 4096, 4096, 1), 0)
    assert list(t[:2]) == [16, 16] and list(t[6:9]) == [16, 16, 32]
    t = binding.mlt_query_tiling(0, (16, 4096, 4096, 0), 0)      # row-major B: the tile kernels
    assert list(t[6:9]) == [32, 32, 16]


def test_mha_argument_validation_without_device(binding):
    lib = binding.raw()
    p = ctypes.c_void_p(0x1000)
    f = lib.mlt_mha_fwd
    assert f(1, 1, 4, 4, 96, p, p, p, p, 1.0, 0, 0, None) == binding.MLT_ERR_UNSUPPORTED   # D
    assert f(1, 1, 4, 0, 64, p, p, p, p, 1.0, 0, 0, None) == binding.MLT_ERR_INVALID_ARG   # Sk = 0
    assert f(1, 1, 4, 4, 64, p, p, p, p, float("nan"), 0, 0, None) == binding.MLT_ERR_INVALID_ARG
    assert f(1, 1, 4, 4, 64, p, p, p, p, float("inf"), 0, 0, None) == binding.MLT_ERR_INVALID_ARG
    assert f(1, 1, 4, 4, 64, p, p, p, p, 1.0, 0, 5, None) == binding.MLT_ERR_INVALID_ARG   # dtype
    assert f(1, 1, 4, 4, 64, ctypes.c_void_p(0), p, p, p, 1.0, 0, 0, None) == binding.MLT_ERR_INVALID_ARG
    assert f(1, 1, 4, 4, 64, ctypes.c_void_p(0x1008), p, p, p, 1.0, 0, 0, None) == binding.MLT_ERR_INVALID_ARG  # alignment
    assert f(0, 1, 4, 4, 64, p, p, p, p, 1.0, 0, 0, None) == binding.MLT_OK                # B = 0
    assert f(1, 1, 0, 4, 128, p, p, p, p, 1.0, 1, 1, None) == binding.MLT_OK               # Sq = 0


def test_tiling_query_is_the_papers_partition_rule(binding):
    """The kernels' fixed layouts follow the paper's encoding rule (Section 2.1):
    sizePerWarp = workgroupSize / warpsPerCTA, GEMM partitioned over both dimensions of the tile,
    attention along the rows only (Section 2.5: warpsPerCTA = [numWarps, 1])."""
    t = binding.mlt_query_tiling(0, (8192, 8192, 8192, 0), 0)
    wg, waves, per_wave, mfma = t[0:2], t[2:4], t[4:6], t[6:9]
    assert wg == [256, 256] and waves[0] * waves[1] == 8
    assert per_wave == [wg[0] // waves[0], wg[1] // waves[1]]
    # the hardware dot of the big-tile kernel is the 16x16x32 MFMA (the lower-power shape)
    assert mfma == [16, 16, 32] and per_wave[0] % 16 == 0 and per_wave[1] % 16 == 0
    # small problems get smaller workgroup tiles, chosen by time per K step over the whole grid
    small = binding.mlt_query_tiling(0, (512, 512, 512, 1), 1)
    assert small[0:2] == [64, 64] and small[2:4] == [2, 2] and small[4:6] == [32, 32]   # (x 4 K groups)
    mid = binding.mlt_query_tiling(0, (2048, 2048, 2048, 0), 0)
    assert mid[0:2] == [128, 128] and mid[2:4] == [2, 4] and mid[4:6] == [64, 32]
    a = binding.mlt_query_tiling(1, (4096, 4096, 128, 0), 0)
    assert a[2:4] == [8, 1] and a[4] == a[0] // 8 and a[5] == 128 and a[9] == 64
    with pytest.raises(binding.MltError):
        binding.mlt_query_tiling(1, (4096, 4096, 80, 0), 0)


def test_bench_refuses_more_than_one_gpu():
    """Everything here runs on one GPU; bench.py says so instead of pretending to scale."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_bench_offers_the_shape_sweeps():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--help"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "--sweep" in r.stdout and "fa2" in r.stdout


def test_bench_reads_measured_traffic_from_the_committed_table():
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    assert bench.median([3.0, 1.0, 2.0]) == 2.0 and bench.median([4.0, 1.0, 2.0, 3.0]) == 2.5
    known = bench.measured_traffic("gemm_nn_256x256x64_w2x4_pp16", 384 << 20)
    assert known["traffic"] == known["traffic_fetch"] + known["traffic_write"] > 384 << 20
    assert "commit" in known["traffic_source"] and known["traffic_ratio"] > 1.0
    unknown = bench.measured_traffic("no_such_kernel", 1)
    assert unknown["traffic"] is None and unknown["traffic_source"] is None
