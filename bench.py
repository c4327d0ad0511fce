#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: one step = one bf16 GEMM 8192^3 (row-major A and B,
fp32 accumulate) followed by one non-causal bf16 attention forward B4 H32 S4096 D128, both through
the C ABI. Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]
  python bench.py --sweep gemm [--torch] [--cold] [--sweep-dtype fp16]   markdown table over the GEMM shape families
  python bench.py --sweep fa2                                    markdown table over the paper's FlashAttention-2 sweep

`value` is the whole step's TFLOP/s (2*M*N*K + 4*B*H*Sq*Sk*D flop per step) with all inputs
resident in HBM. Each kernel is also timed on its own with HIP events recorded on the launch
stream inside the timed region; the `roofline` object is for the kernel that takes the larger
share of the step. `cpu_baseline` times the fp64 oracle on a bounded sample of the same
workload on the host cores (a reported baseline, not a target).
"""
import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0          # MI355X dense bf16/fp16: 256 CUs x 2.4 GHz x 4096 flop/clk/CU
# HBM-side bytes per launch (fetched, written) of the step's kernels, as the rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs measured them (counter x the factor that a plain copy of known size
# gives): a committed text table, one line per kernel name, each with the commit the counters were
# taken at. A kernel that is not in the table has no measured traffic (null in the JSON line).
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
GEMM_MNK = (8192, 8192, 8192)
MHA_SHAPE = (4, 32, 4096, 4096, 128)   # B, H, Sq, Sk, D


def measured_traffic(kernel, algorithmic_bytes):
    """{traffic, traffic_source, traffic_ratio} of one kernel from the committed counter table."""
    none = {"traffic": None, "traffic_source": None, "traffic_ratio": None,
            "algorithmic_bytes": algorithmic_bytes}
    try:
        with open(TRAFFIC_TABLE) as f:
            lines = [ln.strip() for ln in f if ln.strip() and not ln.lstrip().startswith("#")]
    except OSError:
        return none
    for ln in lines:
        cols = [c.strip() for c in ln.split("|")]
        if len(cols) >= 5 and cols[0] == kernel:
            fetch, write = int(cols[2]), int(cols[3])
            return {"traffic": fetch + write, "traffic_fetch": fetch, "traffic_write": write,
                    "traffic_source": "profiles/hbm_traffic.txt: %s, counters taken at commit %s"
                                      % (cols[1], cols[4]),
                    "traffic_ratio": (fetch + write) / algorithmic_bytes,
                    "algorithmic_bytes": algorithmic_bytes}
    return none


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


class HipEvents:
    """Raw hipEvent_t pairs (ctypes on the HIP runtime torch already loaded) for per-kernel timing
    on the stream the library launches on."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return ev

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return ms.value


def cpu_baseline(A, B, Q, K, V, scale):
    """The oracle as it stands, on the host cores: the two headline problems on a bounded sample
    (random C entries at K = 8192, whole attention rows) with the time of the full problem
    extrapolated from it, and two small problems computed in full (GEMM 512^3 with one thread and
    with all of them, attention B1 H1 S1024 D128)."""
    import numpy as np
    import oracle
    from paper_2503_14985_amd import inputs
    rng = np.random.default_rng(123)
    nt = oracle.num_threads()               # all host threads; passed explicitly from here on
    M, Kd = A.shape
    N = B.shape[1]
    ns = 4_000_000
    r, c = rng.integers(0, M, ns), rng.integers(0, N, ns)
    Bt = np.ascontiguousarray(B.T)          # same matrix, k-contiguous storage for the inner loop
    t0 = time.perf_counter()
    oracle.gemm_sampled(A, Bt, r, c, inputs.BF16, transB=True, nthreads=nt)
    t_gemm = time.perf_counter() - t0
    f_gemm = 2.0 * Kd * ns
    Bq, H, Sq, D = Q.shape
    Sk = K.shape[2]
    nrows = 49_152
    bs, hs, qs = rng.integers(0, Bq, nrows), rng.integers(0, H, nrows), rng.integers(0, Sq, nrows)
    t0 = time.perf_counter()
    oracle.mha_fwd_rows(Q, K, V, bs, hs, qs, scale, False, inputs.BF16, nthreads=nt)
    t_mha = time.perf_counter() - t0
    f_mha = 4.0 * D * Sk * nrows

    # small problems in full
    a5, b5 = inputs.gemm_inputs(512, 512, 512, inputs.BF16, seed=1)
    f5 = 2.0 * 512 ** 3
    t0 = time.perf_counter()
    oracle.gemm(a5, b5, inputs.BF16, nthreads=1)
    t5_one = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.gemm(a5, b5, inputs.BF16, nthreads=nt)
    t5_all = time.perf_counter() - t0
    q1, k1, v1 = inputs.mha_inputs(1, 1, 1024, 1024, 128, inputs.BF16, seed=1)
    fm = 4.0 * 1024 * 1024 * 128
    t0 = time.perf_counter()
    oracle.mha_fwd(q1, k1, v1, 1.0 / math.sqrt(128), False, inputs.BF16, nthreads=nt)
    tm = time.perf_counter() - t0
    return {
        "value": (f_gemm + f_mha) / (t_gemm + t_mha) / 1e12, "unit": "TFLOP/s",
        "cores": nt, "kind": "oracle",
        "sample": "%d random C entries of the 8192^3 GEMM (%.1f s) + %d random query rows of the "
                  "B4 H32 S4096 D128 attention (%.1f s), fp64" % (ns, t_gemm, nrows, t_mha),
        "gemm_gflops": f_gemm / t_gemm / 1e9, "mha_gflops": f_mha / t_mha / 1e9,
        "full_problem_seconds_extrapolated": {
            "gemm_8192^3": t_gemm * (float(M) * N / ns),
            "mha_b4_h32_s4096_d128": t_mha * (float(Bq) * H * Sq / nrows),
            "note": "sample time x (outputs of the full problem / outputs sampled); not run in full"},
        "small_problems_in_full": {
            "gemm_512^3_1_thread": {"seconds": t5_one, "gflops": f5 / t5_one / 1e9},
            "gemm_512^3_all_threads": {"seconds": t5_all, "gflops": f5 / t5_all / 1e9,
                                       "threads": nt},
            "mha_b1_h1_s1024_d128_all_threads": {"seconds": tm, "gflops": fm / tm / 1e9}},
    }


PAGED_SHAPE = (64, 32, 4096, 128, 16)   # sequences, heads, keys per sequence, head dim, block size
PAGED_SHAPE_FEW = (1, 8, 32768, 128, 16)   # too few (sequence, head) pairs for the chip: keys split over workgroups


def paged_decode(binding, ev, dev, shape=PAGED_SHAPE):
    """The paged-attention decode kernel (paper Section 3.2) on a bf16 cache of B x H x S keys in
    shuffled 16-key blocks (N(0,1), torch seed 0, generated on the device): HBM-bound, reported in
    GB/s of algorithmic bytes (K and V cache read once, Q and O) against the 8 TB/s peak."""
    import torch
    Bp, Hp, Sp, Dp, bs = shape
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    nb = Bp * (Sp // bs)
    kc = torch.randn((nb, Hp, bs, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    vc = torch.randn((nb, Hp, bs, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    q = torch.randn((Bp, Hp, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    table = torch.randperm(nb, generator=g, device=dev).to(torch.int32).reshape(Bp, -1).contiguous()
    lens = torch.full((Bp,), Sp, dtype=torch.int32, device=dev)
    o = torch.empty_like(q)
    scale = 1.0 / math.sqrt(Dp)
    for _ in range(3):
        binding.mlt_paged_attn_decode(q, kc, vc, table, lens, scale, O=o)
    reps = 10
    e0, e1 = ev.create(), ev.create()
    binding.mlt_set_timing_events(e0, None)
    binding.mlt_paged_attn_decode(q, kc, vc, table, lens, scale, O=o)
    binding.mlt_set_timing_events(None, None)
    for _ in range(reps - 2):
        binding.mlt_paged_attn_decode(q, kc, vc, table, lens, scale, O=o)
    binding.mlt_set_timing_events(None, e1)
    binding.mlt_paged_attn_decode(q, kc, vc, table, lens, scale, O=o)
    binding.mlt_set_timing_events(None, None)
    torch.cuda.synchronize()
    ms = ev.elapsed_ms(e0, e1) / reps
    nbytes = 2.0 * Bp * Hp * Sp * Dp * 2 + 2.0 * Bp * Hp * Dp * 2 + table.numel() * 4
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": binding.mlt_last_kernel(), "avg_ms": ms, "GB_per_s": gbs,
            "frac_hbm_peak": gbs / 8000.0, "bytes_per_launch": nbytes,
            "workload": "B=%d H=%d S=%d D=%d block=%d bf16, shuffled blocks" % shape}


def hbm_ceiling(binding, ev, dev):
    """Rate of a read-only streaming kernel (mlt_probe_hbm_read) over 2 GiB: the practical HBM
    read rate, context for the memory-bound kernels (`paged_decode`), whose fractions stay
    quoted against the nominal 8 TB/s."""
    import torch
    data = torch.empty(1 << 29, dtype=torch.int32, device=dev).random_(0, 2 ** 31 - 1)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    reps = 10
    for _ in range(3):
        binding.mlt_probe_hbm_read(data, sink)
    e0, e1 = ev.create(), ev.create()
    binding.mlt_set_timing_events(e0, None)
    nbytes = binding.mlt_probe_hbm_read(data, sink)
    binding.mlt_set_timing_events(None, None)
    for _ in range(reps - 2):
        binding.mlt_probe_hbm_read(data, sink)
    binding.mlt_set_timing_events(None, e1)
    binding.mlt_probe_hbm_read(data, sink)
    binding.mlt_set_timing_events(None, None)
    torch.cuda.synchronize()
    gbs = nbytes * reps / (ev.elapsed_ms(e0, e1) * 1e-3) / 1e9
    return {"read_GB_per_s": gbs, "frac_hbm_peak": gbs / 8000.0,
            "note": "read-only streaming kernel over 2 GiB, 16-byte loads, 32 KB pieces round-robin over 8 workgroups per CU"}


def sustained(torch, fn, flop_per_call, secs=1.5, batch=25):
    """fn launched back to back for `secs` seconds; rate, board power and shader clock over the
    second half of the run."""
    ps = PowerSampler()
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    ps.start()
    t0 = time.perf_counter()
    n, t_half, n_half = 0, None, 0
    while True:
        for _ in range(batch):
            fn()
        torch.cuda.synchronize()
        n += batch
        now = time.perf_counter()
        if t_half is None and now - t0 >= secs / 2:
            t_half, n_half = now, n
        if now - t0 >= secs:
            break
    watts, mhz = ps.stop(t_half)
    tf = flop_per_call * (n - n_half) / (now - t_half) / 1e12
    return {"tflops": tf, "avg_w": None if watts is None else round(watts, 1),
            "sclk_mhz": None if mhz is None else round(mhz, 1),
            "pj_per_flop": None if watts is None else round(watts / tf, 4),
            "frac_mfma_peak": tf / MFMA_PEAK_TFLOPS,
            "frac_mfma_peak_at_observed_clock":
                None if not mhz else tf / (MFMA_PEAK_TFLOPS * mhz / 2400.0)}


def mfma_ceiling(binding, ev, A, dev):
    """Rate, board power and clock of a register-only MFMA loop over the whole chip
    (mlt_probe_mfma), each run for a second: on all-zero operands, and on the GEMM's own N(0,1)
    operand values through both MFMA shapes. The N(0,1) figures are what the chip's power
    management leaves of the nominal peak for such data before any memory traffic; board power
    over rate is the energy per flop of the multipliers alone, to set beside the kernels' own
    (`power`). Context for `roofline`, whose `peak` stays the nominal one."""
    import torch
    sink = torch.zeros(16, dtype=torch.float32, device=dev)
    res = {}
    for name, data, size in (("zeros", torch.zeros(1 << 16, dtype=torch.bfloat16, device=dev), 32),
                             ("zeros_16x16x32", torch.zeros(1 << 16, dtype=torch.bfloat16, device=dev), 16),
                             ("n01", A.reshape(-1)[: 1 << 16].contiguous(), 32),
                             ("n01_16x16x32", A.reshape(-1)[: 1 << 16].contiguous(), 16)):
        iters = 2048
        flop = binding.mlt_probe_mfma(iters, data, sink, size)
        r = sustained(torch, lambda: binding.mlt_probe_mfma(iters, data, sink, size), flop, secs=1.0, batch=10)
        res[name + "_tflops"] = r["tflops"]
        res[name] = r
    res["note"] = ("register-only bf16 MFMA loop, 8 wavefronts per CU, launched back to back for 1 s "
                   "(rate, board power, shader clock over the second half); zeros / n01: 32x32x16 "
                   "MFMAs on all-zero operands / on operands taken from the GEMM's A matrix; "
                   "_16x16x32: the same through 16x16x32 MFMAs (the GEMM kernel's shape)")
    return res


class PowerSampler:
    """Board power from the amdgpu hwmon files (microwatts), sampled by a thread while kernels run.
    With several cards in sysfs the one drawing the most is taken: it is the one being driven."""

    def __init__(self):
        import glob
        self.inputs = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") or
                             glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))
        self.sclk_files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.samples, self.clocks, self._stop, self._th = [], [], False, None

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return int(f.read().strip())
        except (OSError, ValueError):
            return None

    @staticmethod
    def _current_mhz(path):
        """The level marked as current in an amdgpu pp_dpm_sclk file ('1: 1650Mhz *')."""
        try:
            with open(path) as f:
                for ln in f:
                    if ln.rstrip().endswith("*"):
                        return float(ln.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError):
            pass
        return None

    def cap_w(self):
        caps = [self._read(os.path.join(os.path.dirname(p), "power1_cap")) for p in self.inputs]
        caps = [c for c in caps if c]
        return max(caps) / 1e6 if caps else None

    def _poll(self):
        while not self._stop:
            vals = [v for v in (self._read(p) for p in self.inputs) if v is not None]
            now = time.perf_counter()
            if vals:
                self.samples.append((now, max(vals) / 1e6))
                # the card being driven is the one drawing the most: take its clock
                card = self.inputs[vals.index(max(vals))].split("/device/")[0]
                mhz = self._current_mhz(card + "/device/pp_dpm_sclk")
                if mhz:
                    self.clocks.append((now, mhz))
            time.sleep(0.02)

    def start(self):
        import threading
        self.samples, self.clocks, self._stop = [], [], False
        self._th = threading.Thread(target=self._poll, daemon=True)
        self._th.start()

    def stop(self, since):
        self._stop = True
        self._th.join()
        w = [v for (t, v) in self.samples if t >= since]
        c = [v for (t, v) in self.clocks if t >= since]
        return (sum(w) / len(w) if w else None), (sum(c) / len(c) if c else None)


def power_context(binding, A, B, C, Q, K, V, O, scale):
    """Why the fractions of the nominal peak are what they are: each of the two kernels launched
    back to back for about 1.5 s, once on the benchmark's N(0,1) operands and once on all-zero
    operands of the same shapes (same instructions, same memory traffic, no switching in the
    multipliers), with the board power sampled meanwhile (second half of each run). On the N(0,1)
    operands the board sits at its power cap and the clock is what the cap leaves; on zeros it does
    not, and the rate is what the kernel's schedule reaches at full clock."""
    import torch
    ps = PowerSampler()
    M, N, Kd = GEMM_MNK
    Bq, H, Sq, Sk, D = MHA_SHAPE
    f_gemm, f_mha = 2.0 * M * N * Kd, 4.0 * Bq * H * Sq * Sk * D
    Az, Bz = torch.zeros_like(A), torch.zeros_like(B)
    Qz, Kz, Vz = torch.zeros_like(Q), torch.zeros_like(K), torch.zeros_like(V)
    runs = (("gemm_n01", lambda: binding.mlt_gemm(A, B, C=C), f_gemm),
            ("gemm_zeros", lambda: binding.mlt_gemm(Az, Bz, C=C), f_gemm),
            ("mha_n01", lambda: binding.mlt_mha_fwd(Q, K, V, scale, causal=False, O=O), f_mha),
            ("mha_zeros", lambda: binding.mlt_mha_fwd(Qz, Kz, Vz, scale, causal=False, O=O), f_mha))
    res = {"cap_w": ps.cap_w()}
    for name, fn, flop in runs:
        res[name] = sustained(torch, fn, flop)
    res["note"] = ("each kernel launched back to back for 1.5 s; rate, board power (hwmon "
                   "power1_input) and shader clock (the current level of pp_dpm_sclk) over the "
                   "second half; zeros = all-zero operands of the same shapes; the fraction at the "
                   "observed clock is against 256 CUs x 4096 flop/clk x that clock; pj_per_flop = "
                   "board power / rate")
    return res


GEMM_SWEEP_SHAPES = [
    # (M, N, K, B stored N x K): the square sweep, the LLM shapes with B stored N x K, mid-size
    # and decode (skinny) shapes
    (1024, 1024, 1024, False), (2048, 2048, 2048, False), (3072, 3072, 3072, False),
    (4096, 4096, 4096, False), (8192, 8192, 8192, False), (8192, 8192, 8192, True),
    (4096, 14336, 4096, True), (4096, 4096, 14336, True), (8192, 28672, 8192, True),
    (1024, 4096, 4096, True), (512, 4096, 4096, True), (256, 4096, 4096, True), (128, 4096, 4096, True),
    (512, 8192, 8192, True), (256, 8192, 8192, True), (256, 14336, 4096, True), (512, 4096, 14336, True),
    (64, 4096, 4096, True), (64, 14336, 4096, True), (64, 28672, 8192, True), (64, 8192, 28672, True),
    (64, 131072, 4096, True), (32, 28672, 8192, True), (32, 8192, 28672, True),
    (32, 16384, 8192, True), (32, 32768, 4096, True), (32, 65536, 2048, True),
    (16, 4096, 4096, True), (16, 28672, 8192, True), (16, 8192, 28672, True), (16, 131072, 4096, True),
    (16, 4096, 4096, False), (32, 28672, 8192, False), (1, 28672, 8192, True),
]


def _time_back_to_back(torch, fn, n):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def sweep_gemm(torch, binding, dev, with_torch, dt, with_cold=False):
    """Markdown table of mlt_gemm over the shape families. Each shape is launched back to back
    (best of two runs of n launches; the library launches on torch's current stream here, so
    torch's events see it) on torch.randn inputs: N(0,1) for the square shapes, N(0, 0.02^2) for
    the shapes with B stored N x K. Times below about 12 us are bounded by the Python call.
    with_cold: the decode shapes (M <= 64, B stored N x K) once more with B rotating over copies
    of more than 800 MB in total, so that no launch finds B in the 256 MiB last-level cache, as
    in a decoder, where every weight matrix is read once per token."""
    head = "| M x N x K | B stored | kernel | us | TFLOP/s | GB/s (A+B+C once) |"
    print(head + (" torch us |" if with_torch else "") +
          ((" cold B: us |" + (" torch us |" if with_torch else "")) if with_cold else ""))
    print("|---|---|---|---|---|---|" + ("---|" if with_torch else "") +
          (("---|" + ("---|" if with_torch else "")) if with_cold else ""))
    for (M, N, K, tb) in GEMM_SWEEP_SHAPES:
        std = 0.02 if (tb or M <= 64) else 1.0
        A = (torch.randn(M, K, device=dev, dtype=torch.float32) * std).to(dt)
        B = (torch.randn((N, K) if tb else (K, N), device=dev, dtype=torch.float32) * std).to(dt)
        C = torch.empty(M, N, device=dev, dtype=dt)
        n = 20 if M * N * K > 1e11 else 100
        ms = min(_time_back_to_back(torch, lambda: binding.mlt_gemm(A, B, C=C, transB=tb), n) for _ in range(2))
        line = "| %d x %d x %d | %s | `%s` | %.1f | %.0f | %.0f |" % (
            M, N, K, "N x K" if tb else "K x N", binding.mlt_last_kernel(), ms * 1e3,
            2.0 * M * N * K / ms / 1e9, 2.0 * (M * K + N * K + M * N) / ms / 1e6)
        if with_torch:
            tms = min(_time_back_to_back(torch, lambda: torch.matmul(A, B.t() if tb else B, out=C), n)
                      for _ in range(2))
            line += " %.1f |" % (tms * 1e3)
        if with_cold:
            if M <= 64 and tb:
                copies = [B] + [(torch.randn((N, K), device=dev, dtype=torch.float32) * std).to(dt)
                                for _ in range(max(1, int(800e6 // (N * K * 2))))]
                turn = [0]

                def rotating(f):
                    def call():
                        turn[0] += 1
                        f(copies[turn[0] % len(copies)])
                    return call
                cms = min(_time_back_to_back(
                    torch, rotating(lambda b: binding.mlt_gemm(A, b, C=C, transB=True)), n) for _ in range(2))
                line += " %.1f |" % (cms * 1e3)
                if with_torch:
                    ctms = min(_time_back_to_back(
                        torch, rotating(lambda b: torch.matmul(A, b.t(), out=C)), n) for _ in range(2))
                    line += " %.1f |" % (ctms * 1e3)
                del copies
            else:
                line += " |" + (" |" if with_torch else "")
        print(line, flush=True)


def sweep_fa2(torch, binding, dev):
    """Markdown table of mlt_mha_fwd over the shapes of the paper's FlashAttention-2 evaluation
    (Section 4.2: 32k tokens in total, hidden size 2048 as 32 heads of 64 or 16 heads of 128,
    with and without the causal mask), N(0,1) inputs; causal rates count visible pairs only."""
    print("| heads x D | seq | batch | causal | dtype | kernel | ms | TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|")
    for (H, D) in [(32, 64), (16, 128)]:
        for S in [1024, 2048, 4096, 8192, 16384, 32768]:
            B = 32768 // S
            for causal in (False, True):
                for dt in (torch.float16, torch.bfloat16):
                    if dt == torch.bfloat16 and S not in (4096, 32768):
                        continue
                    q = torch.randn(B, H, S, D, device=dev, dtype=dt)
                    k, v = torch.randn_like(q), torch.randn_like(q)
                    o = torch.empty_like(q)
                    flop = 4.0 * B * H * D * (S * (S + 1) / 2 if causal else S * S)
                    ms = min(_time_back_to_back(
                        torch, lambda: binding.mlt_mha_fwd(q, k, v, 1 / math.sqrt(D), causal, O=o), 10)
                        for _ in range(2))
                    print("| %d x %d | %d | %d | %d | %s | `%s` | %.3f | %.0f |" % (
                        H, D, S, B, int(causal), "fp16" if dt == torch.float16 else "bf16",
                        binding.mlt_last_kernel(), ms, flop / ms / 1e9), flush=True)


def cold_cache_gemm(binding, ev, dev, sets=3, reps=12):
    """The 8192^3 GEMM on operand sets that rotate from launch to launch (3 sets of A, B and C,
    384 MiB each: more than the 256 MiB last-level cache between two uses of the same bytes), so
    that no launch finds its operands cached by the previous one."""
    import torch
    M, N, Kd = GEMM_MNK
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    abc = [(torch.randn((M, Kd), generator=g, device=dev, dtype=torch.bfloat16),
            torch.randn((Kd, N), generator=g, device=dev, dtype=torch.bfloat16),
            torch.empty((M, N), device=dev, dtype=torch.bfloat16)) for _ in range(sets)]
    for i in range(sets):
        binding.mlt_gemm(abc[i][0], abc[i][1], C=abc[i][2])
    evs = [(ev.create(), ev.create()) for _ in range(reps)]
    for i in range(reps):
        a, b, c = abc[i % sets]
        binding.mlt_set_timing_events(evs[i][0], evs[i][1])
        binding.mlt_gemm(a, b, C=c)
    binding.mlt_set_timing_events(None, None)
    torch.cuda.synchronize()
    ms = [ev.elapsed_ms(a, b) for (a, b) in evs]
    flop = 2.0 * M * N * Kd
    return {"median_ms": median(ms), "min_ms": min(ms), "tflops_median": flop / median(ms) / 1e9,
            "frac_mfma_peak": flop / median(ms) / 1e9 / MFMA_PEAK_TFLOPS, "launches": reps,
            "note": "%d operand sets of 384 MiB used in rotation" % sets}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle timing (used when profiling)")
    ap.add_argument("--only", choices=["gemm", "mha", "paged"], default=None,
                    help="run only one kernel (for counter runs of that kernel): one of the two of "
                         "the step, or the paged-attention decode kernel")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the context measurements (MFMA and HBM ceilings, paged decode, power)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed steps also run plain device copies of 256 MiB, so a "
                         "counter run (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) can be scaled by "
                         "what the same counter reads for a copy of known size")
    ap.add_argument("--sweep", choices=["gemm", "fa2"], default=None,
                    help="instead of the step, time the library over a family of shapes and print "
                         "a markdown table: the GEMM shape families, or the paper's "
                         "FlashAttention-2 sweep (Section 4.2)")
    ap.add_argument("--torch", action="store_true", help="--sweep gemm: add torch.matmul on the same tensors")
    ap.add_argument("--sweep-dtype", choices=["bf16", "fp16"], default="bf16", help="--sweep gemm: element type")
    ap.add_argument("--cold", action="store_true",
                    help="--sweep gemm: time the decode shapes once more with B rotating over more than the last-level cache holds")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (kernels on one GPU's share of the "
                 "work); --gpus %d is not supported" % args.gpus)

    import numpy as np
    import torch
    from paper_2503_14985_amd import binding, inputs   # raises if libmlt.so is missing

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def copy_calibration():
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 256 MiB, writes 256 MiB per launch
        torch.cuda.synchronize()

    if args.sweep is not None:
        torch.manual_seed(0)
        if args.sweep == "gemm":
            sweep_gemm(torch, binding, dev, args.torch,
                       torch.bfloat16 if args.sweep_dtype == "bf16" else torch.float16, args.cold)
        else:
            sweep_fa2(torch, binding, dev)
        return

    if args.only == "paged":
        for shape in (PAGED_SHAPE, PAGED_SHAPE_FEW):
            r = paged_decode(binding, HipEvents(), dev, shape)
            print("paged: %s (%s) avg %.4f ms, %.1f GB/s" % (r["kernel"], r["workload"], r["avg_ms"], r["GB_per_s"]))
        if args.copy_calibration:
            copy_calibration()
        return

    M, N, Kd = GEMM_MNK
    Bq, H, Sq, Sk, D = MHA_SHAPE
    scale = 1.0 / math.sqrt(D)
    A_h, B_h = inputs.gemm_inputs(M, N, Kd, inputs.BF16, seed=0)           # N(0,1), row-major
    Q_h, K_h, V_h = inputs.mha_inputs(Bq, H, Sq, Sk, D, inputs.BF16, seed=0)
    A, B = (inputs.bits_to_torch(x, inputs.BF16, dev) for x in (A_h, B_h))
    Q, K, V = (inputs.bits_to_torch(x, inputs.BF16, dev) for x in (Q_h, K_h, V_h))
    C = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    O = torch.empty_like(Q)
    torch.cuda.synchronize()

    ev = HipEvents()
    pairs = [(ev.create(), ev.create(), ev.create(), ev.create()) for _ in range(args.steps)]

    def step(p=None):
        gemm_name = mha_name = ""
        if args.only != "mha":
            if p is not None:
                binding.mlt_set_timing_events(p[0], p[1])
            binding.mlt_gemm(A, B, C=C)
            gemm_name = binding.mlt_last_kernel()
        if args.only != "gemm":
            if p is not None:
                binding.mlt_set_timing_events(p[2], p[3])
            binding.mlt_mha_fwd(Q, K, V, scale, causal=False, O=O)
            mha_name = binding.mlt_last_kernel()
        if p is not None:
            binding.mlt_set_timing_events(None, None)
        return gemm_name, mha_name

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        names = step(pairs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    if args.copy_calibration:
        copy_calibration()

    if args.only is not None:
        # counter / trace runs of a single kernel: no JSON line, just the kernel's own time
        which = 0 if args.only == "gemm" else 2
        ms = [ev.elapsed_ms(p[which], p[which + 1]) for p in pairs]
        print("%s: %s avg %.4f ms over %d launches" % (args.only, names[which // 2], sum(ms) / len(ms), len(ms)))
        return

    gemm_ms = [ev.elapsed_ms(p[0], p[1]) for p in pairs]
    mha_ms = [ev.elapsed_ms(p[2], p[3]) for p in pairs]
    gemm_avg, mha_avg = sum(gemm_ms) / len(gemm_ms), sum(mha_ms) / len(mha_ms)
    f_gemm = 2.0 * M * N * Kd
    f_mha = 4.0 * Bq * H * Sq * Sk * D
    ms_per_step = elapsed * 1e3 / args.steps
    value = (f_gemm + f_mha) / (ms_per_step * 1e-3) / 1e12
    gemm_tf, mha_tf = f_gemm / gemm_avg / 1e9, f_mha / mha_avg / 1e9
    # algorithmic HBM bytes per launch: every operand read once, the result written once
    b_gemm = 2 * (M * Kd + Kd * N + M * N)
    b_mha = 2 * Bq * H * D * (2 * Sq + 2 * Sk)
    t_gemm, t_mha = measured_traffic(names[0], b_gemm), measured_traffic(names[1], b_mha)

    # The kernel with the larger share of the step carries the roofline object.
    if mha_avg >= gemm_avg:
        dom = {"kernel": names[1], "achieved": mha_tf, "avg_ms": mha_avg, "median_ms": median(mha_ms),
               "flop_per_launch": f_mha, "t": t_mha}
    else:
        dom = {"kernel": names[0], "achieved": gemm_tf, "avg_ms": gemm_avg, "median_ms": median(gemm_ms),
               "flop_per_launch": f_gemm, "t": t_gemm}
    roofline = {"bound": "mfma", "achieved": dom["achieved"], "peak": MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["achieved"] / MFMA_PEAK_TFLOPS,
                "traffic": dom["t"]["traffic"], "traffic_source": dom["t"]["traffic_source"],
                "traffic_ratio": dom["t"]["traffic_ratio"], "kernel": dom["kernel"],
                "avg_kernel_ms": dom["avg_ms"], "median_kernel_ms": dom["median_ms"],
                "flop_per_launch": dom["flop_per_launch"],
                "launches": "the %d timed launches of the step (warm-ups not included), HIP events "
                            "around each on the launch stream" % args.steps}

    def kernel_line(name, ms, tf, flop, t):
        return {"kernel": name, "avg_ms": sum(ms) / len(ms), "median_ms": median(ms), "min_ms": min(ms),
                "tflops": tf, "tflops_median": flop / median(ms) / 1e9,
                "frac_mfma_peak": tf / MFMA_PEAK_TFLOPS, "hbm": t}

    out = {
        "metric": "TFLOP/s + % MFMA peak: bf16 GEMM 8192^3; MHA fwd B4*H32*S4096*D128",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "bf16 GEMM M=N=K=8192 row-major A,B (N(0,1), seed 0) + non-causal "
                               "MHA forward B=4 H=32 Sq=Sk=4096 D=128 bf16 (N(0,1), seed 0), "
                               "one of each per step"},
        "gemm": kernel_line(names[0], gemm_ms, gemm_tf, f_gemm, t_gemm),
        "mha": dict(kernel_line(names[1], mha_ms, mha_tf, f_mha, t_mha),
                    flop_convention="4*B*H*Sq*Sk*D",
                    # the second bound of this kernel: the softmax on the vector ALU. Per 64-key tile
                    # a wavefront (32 query rows) issues 32 v_exp_f32 (8.3 clk each, measured) and
                    # about 113 other vector instructions (5.1 clk) for 4*D*32*64 flop of MFMA work
                    valu_bound={"tflops": 1024 * 2.4e9 / (32 * 8.3 + 113 * 5.1) * 4 * D * 32 * 64 / 1e12,
                                "note": "1024 SIMDs x 2.4 GHz / (vector ALU clocks per key tile and "
                                        "wavefront) x MFMA flop per key tile and wavefront; above the "
                                        "MFMA peak for D = 128, below it (1.53 PFLOP/s) for D = 64"}),
        "roofline": roofline,
    }
    if not args.no_ceiling:
        out["mfma_ceiling"] = mfma_ceiling(binding, ev, A, dev)
        out["paged_decode"] = paged_decode(binding, ev, dev)
        out["paged_decode_few_pairs"] = paged_decode(binding, ev, dev, PAGED_SHAPE_FEW)
        out["hbm_ceiling"] = hbm_ceiling(binding, ev, dev)
        out["power"] = power_context(binding, A, B, C, Q, K, V, O, scale)
        # second number beside the nominal fraction: against what a register-only loop of the same
        # MFMA shape reaches on N(0,1) operands on this board (power management included)
        for k, ceil in (("gemm", "n01_16x16x32"), ("mha", "n01")):
            out[k]["frac_of_measured_mfma_ceiling"] = out[k]["tflops"] / out["mfma_ceiling"][ceil + "_tflops"]
            out[k]["measured_mfma_ceiling"] = "mfma_ceiling.%s_tflops" % ceil
        for k in ("gemm", "mha"):
            out[k]["frac_mfma_peak_at_observed_clock"] = out["power"][k + "_n01"]["frac_mfma_peak_at_observed_clock"]
            out[k]["observed_clock_note"] = ("from the back-to-back run of this kernel in `power` "
                                             "(its rate over 256 CUs x 4096 flop/clk x the sampled shader clock)")
        out["gemm_cold_cache"] = cold_cache_gemm(binding, ev, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(A_h, B_h, Q_h, K_h, V_h, scale)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
