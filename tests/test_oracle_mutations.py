"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's source (a wrong
rounding rule, a dropped term, a wrong sign or index, a transposed operand), builds it, and runs the pin
tests against that build in a child process: the named pin file must fail.  The unmodified copy must pass.
CPU only; nothing here touches the GPU library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import omc_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "omc_oracle.c")

# (name, text in the oracle's source, replacement, pin file that must notice)
MUTATIONS = [
    ("ties away from zero instead of to even",
     "double k = nearbyint(a / ulp);", "double k = round(a / ulp);", "test_oracle_codec.py"),
    ("subnormal step of the wrong binade",
     "mag = ldexp((double)m, 1 - f.bias - M);", "mag = ldexp((double)m, -f.bias - M);", "test_oracle_codec.py"),
    ("no saturation on overflow",
     "if (ex > top - f.bias) {", "if (0) {", "test_oracle_codec.py"),
    ("most significant bit first in the packed stream",
     "out[i / 8] |= (uint8_t)(1u << (i % 8));", "out[i / 8] |= (uint8_t)(0x80u >> (i % 8));", "test_oracle_codec.py"),
    ("a denominator of s that mixes V and Vtilde",
     "double den = dn * STT - ST * ST;", "double den = dn * STT - SV * ST;", "test_oracle_pvt.py"),
    ("the stray factor n in b",
     "b = (SV - s * ST) / dn;", "b = (dn * SV - s * ST) / dn;", "test_oracle_pvt.py"),
    ("exact sum rounded half away instead of half to even",
     "if (round_bit && (sticky || (mant & 1))) mant += 1;", "if (round_bit) mant += 1;", "test_oracle_pvt.py"),
    ("transformation without its offset",
     "out[k] = st + b;", "out[k] = st;", "test_oracle_pvt.py"),
    ("Adam's second moment weighted with 1 - beta1",
     "float g_weighted = fl((double)o->one_minus_beta2 * (double)g);",
     "float g_weighted = fl((double)o->one_minus_beta1 * (double)g);", "test_oracle_pvt.py"),
    ("momentum with the gradient subtracted",
     "*m = fl((double)decayed + (double)g);", "*m = fl((double)decayed - (double)g);", "test_oracle_pvt.py"),
    ("Adam's epsilon inside the square root",
     "float root = fl(sqrt((double)v_unbiased));", "float root = fl(sqrt((double)v_unbiased + (double)o->eps));",
     "test_oracle_pvt.py"),
    ("forward GEMM reading the activations transposed",
     "double a = bf16_value(A[(uint64_t)i * K + k]);", "double a = bf16_value(A[(uint64_t)k * M + i]);",
     "test_oracle_pvt.py"),
    ("mean by multiplication with the reciprocal",
     "out[i] = acc / (float)R;", "out[i] = acc * (1.0f / (float)R);", "test_oracle_aggregate.py"),
]


def _build(text, path):
    c = path + ".c"
    with open(c, "w") as fh:
        fh.write(text)
    subprocess.check_call(["gcc", *orc.GCC_FLAGS, "-w", c, "-o", path, "-lm"])


def _run_pins(lib, pin_file):
    env = dict(os.environ, OMC_ORACLE_LIBRARY=lib)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", pin_file)],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def test_every_planted_mistake_fails_a_pin(tmp_path):
    src = open(SRC).read()
    jobs = []
    for k, (name, old, new, pin_file) in enumerate(MUTATIONS):
        assert src.count(old) == 1, f"mutation '{name}': its anchor text occurs {src.count(old)} times in the oracle"
        lib = str(tmp_path / f"mut{k}.so")
        _build(src.replace(old, new), lib)
        jobs.append((name, lib, pin_file))
    control = str(tmp_path / "control.so")
    _build(src, control)
    with ThreadPoolExecutor(4) as ex:
        results = list(ex.map(lambda j: _run_pins(j[1], j[2]), jobs))
        controls = list(ex.map(lambda f: _run_pins(control, f),
                               ["test_oracle_codec.py", "test_oracle_pvt.py", "test_oracle_aggregate.py"]))
    for r in controls:
        assert r.returncode == 0, "the unmodified oracle fails its own pins:\n" + r.stdout[-2000:]
    survived = [name for (name, _, _), r in zip(jobs, results) if r.returncode == 0]
    assert not survived, f"no pin noticed: {survived}"
    for (name, _, _), r in zip(jobs, results):
        assert "failed" in r.stdout, f"'{name}': the pin run ended without a test failure:\n{r.stdout[-1500:]}"
