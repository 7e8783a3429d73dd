"""The quantize-and-write kernel computes the two divisions of the quantizer (Sec. 3.2 "KV Compression":
lambda = (max - min) / (2^b - 1), then x / lambda) without division instructions.  That both forms give the
correctly rounded quotient is arithmetic, not GPU behaviour, and is checked here on the CPU by
tests/divcheck/quantizer_divisions.c: the division by 255 and 15 on a strided sample of every binary32 range value
(ALISE_EXHAUSTIVE=1 in the environment: all 1.2e9 of them, about a minute), the reciprocal of every fp16 scale from
every starting value within one ulp."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("divcheck") / "quantizer_divisions")
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-o", exe,
                    os.path.join(ROOT, "tests", "divcheck", "quantizer_divisions.c"), "-lm"], check=True)
    return exe


def test_division_by_qmax_without_a_division(checker):
    stride = "1" if os.environ.get("ALISE_EXHAUSTIVE") == "1" else "97"
    run = subprocess.run([checker, "div", stride], capture_output=True, text=True, timeout=900)
    assert run.returncode == 0 and " 0 mismatches" in run.stdout, run.stdout + run.stderr


def test_reciprocal_of_every_scale_from_any_start_within_one_ulp(checker):
    run = subprocess.run([checker, "rcp"], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and " 0 mismatches" in run.stdout, run.stdout + run.stderr
