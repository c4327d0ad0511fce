"""A guard on one assumption the persistent attention kernel makes about the compiler.

mha_ps_kernel loads the next item's Q operand with inline-assembly loads straight into the
registers the MFMAs read, and only the schedule's own s_waitcnt knows when the data is there. That
is sound as long as the compiler does not touch those registers between the loads and the
q_finish step that follows the wait (a register copy there would copy data that has not arrived).
The GPU parity tests would catch such a copy; this test catches it without a GPU, by compiling
the file to assembly and reading the kernel."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _vregs(text):
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        regs |= set(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", text):
        regs.add(int(a))
    return regs


def test_persistent_attention_q_registers_are_left_alone_while_loading(tmp_path):
    import __graft_entry__ as entry
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc here")
    out = tmp_path / "mha_pp.s"
    flags = [f for f in entry.HIPCC_FLAGS if f != "-fPIC"]
    subprocess.check_call([hipcc] + flags + ["-S", "--cuda-device-only", "-o", str(out),
                                             os.path.join(entry.CSRC, "mha_pp.hip")],
                          stderr=subprocess.DEVNULL)
    asm = out.read_text()
    kernels = re.findall(r"^(_Z\S*mha_ps_kernel\S*):.*?\n(.*?)\.end_amdhsa_kernel", asm, re.S | re.M)
    assert len(kernels) == 2, "bf16 and fp16, D = 128"
    for name, body in kernels:
        lines = [l.strip() for l in body.split("\n")]
        nkk = 8 if "Li128E" in name else 4
        loads = [i for i, l in enumerate(lines) if l.startswith("global_load_dwordx4 ")]
        # two groups of nkk loads: the first item's (before the loop) and the next item's (in it)
        assert len(loads) == 2 * nkk, (name, len(loads))
        for group in (loads[:nkk], loads[nkk:]):
            dest = set()
            for i in group:
                dest |= _vregs(lines[i].split(",")[0])
            assert len(dest) == 4 * nkk
            # from the last load of the group to the first sign flip that reads one of them
            j = group[-1] + 1
            while not (lines[j].startswith("v_xor_b32") and _vregs(lines[j]) & dest):
                touched = _vregs(lines[j]) & dest
                # the loads of the group itself may interleave with address arithmetic, nothing else
                assert not touched, "%s: line %d touches a Q register in flight: %s" % (name[-30:], j, lines[j])
                j += 1
                assert j < len(lines), "no q_finish found"
            # and the wait that the schedule supplies sits in front of that first use
            back = [l for l in lines[group[-1]:j] if l.startswith("s_waitcnt") and "vmcnt" in l]
            assert back, "%s: no vmcnt wait between the Q loads and their first use" % name[-30:]


def _compile_to_asm(src, tmp_path):
    import __graft_entry__ as entry
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc here")
    out = tmp_path / (src + ".s")
    flags = [f for f in entry.HIPCC_FLAGS if f != "-fPIC"]
    subprocess.check_call([hipcc] + flags + ["-S", "--cuda-device-only", "-o", str(out),
                                             os.path.join(entry.CSRC, src)], stderr=subprocess.DEVNULL)
    return out.read_text()


def test_headline_kernels_keep_their_registers(tmp_path):
    """The two kernels of the benchmark step must not spill (no scratch memory) and must fit the
    occupancy their launch assumes: 8 wavefronts per CU = 2 per SIMD = at most 256 registers."""
    for src, pattern in (("gemm_pp.hip", r"gemm_pp_kernel\S*"), ("mha_pp.hip", r"mha_pp_kernelINS_\w+_tagELi128\S*")):
        asm = _compile_to_asm(src, tmp_path)
        found = 0
        for m in re.finditer(r"^(_Z\S*" + pattern + r"):.*?\n(.*?)\.end_amdhsa_kernel", asm, re.S | re.M):
            body, tail = m.group(2), asm[m.end():m.end() + 4000]
            scratch = int(re.search(r"; ScratchSize: (\d+)", tail).group(1))
            vgprs = int(re.search(r"\.amdhsa_next_free_vgpr (\d+)", body).group(1))
            assert scratch == 0, "%s spills %d bytes" % (m.group(1)[-40:], scratch)
            assert vgprs <= 256
            found += 1
        assert found >= 4, (src, found)
