#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: one step = one bf16 GEMM 8192^3 (row-major A and B,
fp32 accumulate) followed by one non-causal bf16 attention forward B4 H32 S4096 D128, both through
the C ABI. Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]

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
# HBM-side bytes per launch (fetched + written) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs summarised under profiles/ (counter x the factor a plain copy of known size gives).
# Keyed by kernel variant; None when a variant has not been measured.
MEASURED_TRAFFIC_BYTES = {
    "mha_fwd_d128_256x64_pp": int((2.0 * 196680 + 131072) * 1024),
    "gemm_nn_256x256x64_w2x4_pp16": int((2.0 * 786569 + 133228) * 1024),
}
GEMM_MNK = (8192, 8192, 8192)
MHA_SHAPE = (4, 32, 4096, 4096, 128)   # B, H, Sq, Sk, D


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
    """Oracle (as it stands) on a bounded sample: GEMM entries at K = 8192 and whole attention rows."""
    import numpy as np
    import oracle
    from paper_2503_14985_amd import inputs
    rng = np.random.default_rng(123)
    M, Kd = A.shape
    N = B.shape[1]
    ns = 4_000_000
    r, c = rng.integers(0, M, ns), rng.integers(0, N, ns)
    Bt = np.ascontiguousarray(B.T)          # same matrix, k-contiguous storage for the inner loop
    t0 = time.perf_counter()
    oracle.gemm_sampled(A, Bt, r, c, inputs.BF16, transB=True)
    t_gemm = time.perf_counter() - t0
    f_gemm = 2.0 * Kd * ns
    Bq, H, Sq, D = Q.shape
    Sk = K.shape[2]
    nrows = 49_152
    bs, hs, qs = rng.integers(0, Bq, nrows), rng.integers(0, H, nrows), rng.integers(0, Sq, nrows)
    t0 = time.perf_counter()
    oracle.mha_fwd_rows(Q, K, V, bs, hs, qs, scale, False, inputs.BF16)
    t_mha = time.perf_counter() - t0
    f_mha = 4.0 * D * Sk * nrows
    return {
        "value": (f_gemm + f_mha) / (t_gemm + t_mha) / 1e12, "unit": "TFLOP/s",
        "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "%d random C entries of the 8192^3 GEMM (%.1f s) + %d random query rows of the "
                  "B4 H32 S4096 D128 attention (%.1f s), fp64" % (ns, t_gemm, nrows, t_mha),
        "gemm_gflops": f_gemm / t_gemm / 1e9, "mha_gflops": f_mha / t_mha / 1e9,
    }


PAGED_SHAPE = (64, 32, 4096, 128, 16)   # sequences, heads, keys per sequence, head dim, block size


def paged_decode(binding, ev, dev):
    """The paged-attention decode kernel (paper Section 3.2) on a bf16 cache of B x H x S keys in
    shuffled 16-key blocks (N(0,1), torch seed 0, generated on the device): HBM-bound, reported in
    GB/s of algorithmic bytes (K and V cache read once, Q and O) against the 8 TB/s peak."""
    import torch
    Bp, Hp, Sp, Dp, bs = PAGED_SHAPE
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
            "workload": "B=%d H=%d S=%d D=%d block=%d bf16, shuffled blocks" % PAGED_SHAPE}


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


def mfma_ceiling(binding, ev, A, dev):
    """Rate of a register-only MFMA loop over the whole chip (mlt_probe_mfma) on all-zero operands
    and on the GEMM's own N(0,1) operand values: the second is what the chip's power management
    leaves of the nominal peak for such data, before any memory traffic. Context for `roofline`,
    whose `peak` stays the nominal one."""
    import torch
    sink = torch.zeros(16, dtype=torch.float32, device=dev)
    res = {}
    for name, data, size in (("zeros", torch.zeros(1 << 16, dtype=torch.bfloat16, device=dev), 32),
                             ("n01", A.reshape(-1)[: 1 << 16].contiguous(), 32),
                             ("n01_16x16x32", A.reshape(-1)[: 1 << 16].contiguous(), 16)):
        iters, reps = 2048, 12
        for _ in range(3):
            binding.mlt_probe_mfma(iters, data, sink, size)
        e0, e1 = ev.create(), ev.create()
        binding.mlt_set_timing_events(e0, None)
        flop = binding.mlt_probe_mfma(iters, data, sink, size)
        binding.mlt_set_timing_events(None, None)
        for _ in range(reps - 2):
            binding.mlt_probe_mfma(iters, data, sink, size)
        binding.mlt_set_timing_events(None, e1)
        binding.mlt_probe_mfma(iters, data, sink, size)
        binding.mlt_set_timing_events(None, None)
        torch.cuda.synchronize()
        res[name + "_tflops"] = flop * reps / (ev.elapsed_ms(e0, e1) * 1e-3) / 1e12
    res["note"] = ("register-only bf16 MFMA loop, 8 wavefronts per CU; zeros / n01: 32x32x16 MFMAs on "
                   "all-zero operands / on operands taken from the GEMM's A matrix; n01_16x16x32: the "
                   "same N(0,1) operands through 16x16x32 MFMAs (the GEMM kernel's shape)")
    return res


class PowerSampler:
    """Board power from the amdgpu hwmon files (microwatts), sampled by a thread while kernels run.
    With several cards in sysfs the one drawing the most is taken: it is the one being driven."""

    def __init__(self):
        import glob
        self.inputs = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") or
                             glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))
        self.samples, self._stop, self._th = [], False, None

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return int(f.read().strip())
        except (OSError, ValueError):
            return None

    def cap_w(self):
        caps = [self._read(os.path.join(os.path.dirname(p), "power1_cap")) for p in self.inputs]
        caps = [c for c in caps if c]
        return max(caps) / 1e6 if caps else None

    def _poll(self):
        while not self._stop:
            vals = [v for v in (self._read(p) for p in self.inputs) if v is not None]
            if vals:
                self.samples.append((time.perf_counter(), max(vals) / 1e6))
            time.sleep(0.02)

    def start(self):
        import threading
        self.samples, self._stop = [], False
        self._th = threading.Thread(target=self._poll, daemon=True)
        self._th.start()

    def stop(self, since):
        self._stop = True
        self._th.join()
        w = [v for (t, v) in self.samples if t >= since]
        return sum(w) / len(w) if w else None


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
    secs = 1.5
    for name, fn, flop in runs:
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        ps.start()
        t0 = time.perf_counter()
        n, t_half, n_half = 0, None, 0
        while True:
            for _ in range(25):
                fn()
            torch.cuda.synchronize()
            n += 25
            now = time.perf_counter()
            if t_half is None and now - t0 >= secs / 2:
                t_half, n_half = now, n
            if now - t0 >= secs:
                break
        watts = ps.stop(t_half)
        res[name] = {"tflops": flop * (n - n_half) / (now - t_half) / 1e12,
                     "avg_w": None if watts is None else round(watts, 1)}
    res["note"] = ("each kernel launched back to back for 1.5 s; rate and board power (hwmon "
                   "power1_input) over the second half; zeros = all-zero operands of the same shapes")
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
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

    if args.only == "paged":
        r = paged_decode(binding, HipEvents(), dev)
        if args.copy_calibration:
            copy_calibration()
        print("paged: %s avg %.4f ms, %.1f GB/s" % (r["kernel"], r["avg_ms"], r["GB_per_s"]))
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

    # The kernel with the larger share of the step carries the roofline object.
    if mha_avg >= gemm_avg:
        dom = {"kernel": names[1], "achieved": mha_tf, "avg_ms": mha_avg,
               "flop_per_launch": f_mha, "traffic": MEASURED_TRAFFIC_BYTES.get(names[1])}
    else:
        dom = {"kernel": names[0], "achieved": gemm_tf, "avg_ms": gemm_avg,
               "flop_per_launch": f_gemm, "traffic": MEASURED_TRAFFIC_BYTES.get(names[0])}
    roofline = {"bound": "mfma", "achieved": dom["achieved"], "peak": MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["achieved"] / MFMA_PEAK_TFLOPS,
                "traffic": dom["traffic"], "kernel": dom["kernel"], "avg_kernel_ms": dom["avg_ms"],
                "flop_per_launch": dom["flop_per_launch"]}

    out = {
        "metric": "TFLOP/s + % MFMA peak: bf16 GEMM 8192^3; MHA fwd B4*H32*S4096*D128",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "bf16 GEMM M=N=K=8192 row-major A,B (N(0,1), seed 0) + non-causal "
                               "MHA forward B=4 H=32 Sq=Sk=4096 D=128 bf16 (N(0,1), seed 0), "
                               "one of each per step"},
        "gemm": {"kernel": names[0], "avg_ms": gemm_avg, "min_ms": min(gemm_ms), "tflops": gemm_tf,
                 "frac_mfma_peak": gemm_tf / MFMA_PEAK_TFLOPS},
        "mha": {"kernel": names[1], "avg_ms": mha_avg, "min_ms": min(mha_ms), "tflops": mha_tf,
                "frac_mfma_peak": mha_tf / MFMA_PEAK_TFLOPS,
                "flop_convention": "4*B*H*Sq*Sk*D"},
        "roofline": roofline,
    }
    if not args.no_ceiling:
        out["mfma_ceiling"] = mfma_ceiling(binding, ev, A, dev)
        out["paged_decode"] = paged_decode(binding, ev, dev)
        out["hbm_ceiling"] = hbm_ceiling(binding, ev, dev)
        out["power"] = power_context(binding, A, B, C, Q, K, V, O, scale)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(A_h, B_h, Q_h, K_h, V_h, scale)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
