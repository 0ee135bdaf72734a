"""The quantiser kernel forms Appendix A's q = int(w / s) from one reciprocal per group and two fused
multiply-adds per weight instead of a division per weight.  That this gives the integer the binary32
division gives is a fact about binary16 numerators and binary16 / bfloat16 denominators; it is checked
here on the host, in C (exact fmaf), over every 11th finite scale and every numerator in range
(`tests/encode_identity_check.c`; run the built program without arguments for all scales, ~25 s)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_quotient_from_reciprocal_and_two_fused_corrections(tmp_path):
    exe = str(tmp_path / "encode_identity_check")
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-o", exe, os.path.join(HERE, "encode_identity_check.c"), "-lm"],
                   check=True)
    out = subprocess.run([exe, "11"], capture_output=True, text=True, timeout=300)
    print(out.stdout)
    assert out.returncode == 0, out.stdout + out.stderr
    lines = [l for l in out.stdout.splitlines() if "pairs" in l]
    assert len(lines) == 6
    for line in lines:
        words = line.split()
        pairs, ties, bad = (int(words[words.index(k) - 1]) for k in ("pairs,", "exact", "mismatches"))
        assert pairs > 5_000_000 and ties > 1000 and bad == 0, line
