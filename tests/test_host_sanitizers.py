"""The CPU oracle and the pure host part of the C ABI (argument validators and the per-call
plan) built with the address and undefined-behaviour sanitizers and run on small inputs.  The
sanitizer runtime is linked statically so that the executables run under any preload."""
import os
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
ASAN_OPTIONS = "detect_leaks=1:verify_asan_link_order=0"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan",
       "-static-libubsan", "-g", "-O1"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(map(str, cmd)), r.stdout, r.stderr)
    return r.stdout


@pytest.fixture(scope="module")
def outdir(tmp_path_factory):
    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("no host compiler")
    return tmp_path_factory.mktemp("san")


def test_oracle_under_address_and_ub_sanitizers(outdir):
    exe = outdir / "san_oracle"
    _run(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp", *SAN, str(ROOT / "oracle" / "vt_oracle.c"),
          str(ROOT / "tests" / "san" / "san_oracle_main.c"), "-o", str(exe), "-lm"])
    out = _run([str(exe)], env=dict(os.environ, ASAN_OPTIONS=ASAN_OPTIONS, OMP_NUM_THREADS="2"))
    assert "san_oracle ok" in out


def test_host_validators_and_plan_under_address_and_ub_sanitizers(outdir):
    exe = outdir / "san_plan"
    csrc = ROOT / "paper_2603_05210_amd" / "csrc"
    _run(["g++", "-std=c++17", *SAN, "-I", str(ROOT / "include"), "-I", str(csrc), str(csrc / "vt_plan.cpp"),
          str(ROOT / "tests" / "san" / "san_plan_main.cpp"), "-o", str(exe)])
    out = _run([str(exe)], env=dict(os.environ, ASAN_OPTIONS=ASAN_OPTIONS))
    assert "san_plan ok" in out
