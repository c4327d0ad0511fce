"""Address and undefined-behaviour sanitizer runs of the code that executes on the host: the fp64
oracle (oracle/oracle.c) on small ragged problems with exactly-sized buffers, and the argument
validation and dispatch layer of the C ABI (csrc/mlt_api.hip, host side only) on calls it must
reject or accept as no-ops before anything touches a GPU. Each is a small program of its own under
tests/sanitize/, built here with the sanitizers linked in statically and run as a child process."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
CSRC = os.path.join(ROOT, "paper_2503_14985_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-3000:], r.stderr[-3000:])
    return r


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "san_oracle")
    _run([gcc, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-static-libasan", "-fopenmp", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "oracle.c"), "-lm"])
    r = _run([exe])
    assert r.stdout.strip().endswith("ok"), r.stdout + r.stderr


def test_host_side_of_the_abi_under_address_and_undefined_sanitizers(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    # the kernels' objects come from the regular build; only the API layer is rebuilt here
    others = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))
              if f.endswith(".o") and not f.endswith("_dbg.o") and f != "mlt_api.o"]
    if len(others) < 8:
        pytest.skip("library objects not built (run __graft_entry__.build_lib())")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    api, drv, exe = (str(tmp_path / n) for n in ("mlt_api_san.o", "abi_driver.o", "san_abi"))
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
          "-Xclang", "-packed-fp32-ops"] + san + ["-c", os.path.join(CSRC, "mlt_api.hip"), "-o", api])
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17"] + san +
         ["-x", "hip", "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv])
    _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
          "-o", exe, drv, api] + others)
    r = _run([exe])
    assert r.stdout.strip().endswith("ok"), r.stdout + r.stderr
