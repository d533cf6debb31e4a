"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

``oracle/sanitize_check.c`` calls every routine of ``oracle/mx_oracle.c`` on heap buffers of exactly the documented
sizes over ragged shapes, all widths, narrow exponents, subnormals and the top of the fp32 range; an access outside a
buffer, an oversized shift or a signed overflow ends the run with a report and a non-zero status."""
import os
import shutil
import subprocess

import pytest

ORACLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-static-libasan", "-fopenmp", "-ffp-contract=off", "-o", exe, os.path.join(ORACLE, "sanitize_check.c"), "-lm"],
        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "calls clean" in run.stdout
