"""Are the oracle's pins sharp? Plant one plausible mistake at a time in a COPY of oracle.c
(CPU only, never in the committed oracle), rebuild it, and require the pin suite to fail."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "oracle.c")

# (name, text in oracle.c, replacement)
MUTATIONS = [
    ("attention: scale dropped", "s[j] = scale * dot;", "s[j] = dot;"),
    ("attention: exponent sign", "s[j] = exp(s[j] - m);", "s[j] = exp(m - s[j]);"),
    ("attention: no normalisation", "double wj = s[j] / l;", "double wj = s[j];"),
    ("attention: causal excludes the diagonal", "(i + 1 < Sk ? i + 1 : Sk)", "(i < Sk ? i : Sk)"),
    ("attention: causal ignored", "int64_t nvis = causal ?", "int64_t nvis = 0 ?"),
    ("attention: V taken from head 0 of the batch",
     "const uint16_t* vbase = V + (b * H + h) * Sk * D;",
     "const uint16_t* vbase = V + (b * H) * Sk * D;"),
    ("attention: K used in place of V", "o[d] += wj * widen(vbase[j * D + d], dtype);",
     "o[d] += wj * widen(kbase[j * D + d], dtype);"),
    ("attention: query row ignored", "Q + ((b * H + h) * Sq + i) * D;",
     "Q + ((b * H + h) * Sq) * D;"),
    ("paged: slot taken from the block number", "+ p % block_size) * D;\n        double dot",
     "+ p / block_size) * D;\n        double dot"),
    ("paged: keys past seq_len included", "for (int64_t p = 0; p < len; ++p) {\n        s[p] = exp",
     "for (int64_t p = 0; p < cap; ++p) {\n        s[p] = exp"),
    ("paged: table row of sequence 0", "block_table[b * max_blocks + p / block_size];\n        const uint16_t* v",
     "block_table[p / block_size];\n        const uint16_t* v"),
    ("paged: head stride dropped for K", "Kc + ((pb * H + h) * block_size", "Kc + ((pb * H) * block_size"),
    ("paged: scale dropped", "s[p] = scale * dot;", "s[p] = dot;"),
    ("paged: weights not normalised", "const double wp = s[p] / l;", "const double wp = s[p];"),
    ("epilogue: bias taken by row", "const double bj = widen(bias[j], dtype);",
     "const double bj = widen(bias[i], dtype);"),
    ("epilogue: bias subtracted", "y += bj;", "y -= bj;"),
    ("epilogue: magnitude ignores the bias", "mag[i * ldx + j] += fabs(bj);", "mag[i * ldx + j] += 0.0;"),
    ("epilogue: relu keeps the negative side", "y = y > 0.0 ? y : 0.0;", "y = y < 0.0 ? y : 0.0;"),
    ("epilogue: gelu argument not divided by sqrt 2", "erf(y / sqrt(2.0))", "erf(y)"),
    ("epilogue: gelu without the one half", "y = 0.5 * y * (1.0 +", "y = y * (1.0 +"),
    ("gemm: B read transposed", "transB ? B[j * ldb + k] : B[k * ldb + j]",
     "transB ? B[k * ldb + j] : B[j * ldb + k]"),
    ("gemm: last k dropped", "for (int64_t k = 0; k < K; ++k) {\n    double a = widen(A[i",
     "for (int64_t k = 0; k + 1 < K; ++k) {\n    double a = widen(A[i"),
    ("gemm: magnitude sum without abs", "mag += fabs(a) * fabs(b);", "mag += a * b;"),
    ("gemm: product sign", "acc += a * b;", "acc -= a * b;"),
    ("fp16: exponent bias", "e - 15);", "e - 14);"),
    ("fp16: subnormal scale", "ldexp((double)frac, -24)", "ldexp((double)frac, -25)"),
    ("bf16: shift", "((uint32_t)h) << 16", "((uint32_t)h) << 15"),
    ("rounding: ties away from zero", "(fmod(fl, 2.0) == 0.0) ? fl : fl + 1.0", "fl + 1.0"),
]


def _pins_fail_with(lib_path):
    env = dict(os.environ, MLT_TEST_ORACLE_LIB=lib_path, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider"], env=env, cwd=ROOT,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)
    return r.returncode != 0, r.stdout.decode()[-600:]


def test_every_planted_mistake_is_caught(tmp_path):
    text = open(SRC).read()
    jobs = []
    for n, (name, old, new) in enumerate(MUTATIONS):
        assert text.count(old) == 1, "mutation target not unique/present: %s" % name
        src = tmp_path / ("mut%d.c" % n)
        src.write_text(text.replace(old, new))
        lib = str(tmp_path / ("libmut%d.so" % n))
        oracle.build(force=True, src=str(src), out=lib)
        jobs.append((name, lib))
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda j: _pins_fail_with(j[1]), jobs))
    survivors = [name for (name, _), (failed, _) in zip(jobs, results) if not failed]
    assert not survivors, "pins did not notice: %s" % survivors


def test_unmutated_build_passes_in_child(tmp_path):
    """Control: the same child-process route with a faithful copy passes."""
    lib = str(tmp_path / "libsame.so")
    oracle.build(force=True, src=SRC, out=lib)
    failed, tail = _pins_fail_with(lib)
    assert not failed, tail
