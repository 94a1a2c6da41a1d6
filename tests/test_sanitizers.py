"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only):
the oracle and the input generator on a small workload, and the library's
host-side argument checks in a host-only build (its device code objects are
replaced by empty stand-ins; nothing is launched)."""
import os
import re
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(map(str, cmd))}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    return r


def test_oracle_and_input_generator_under_sanitizers(tmp_path):
    exe = tmp_path / "oracle_driver"
    run(["g++", "-std=c++17", "-ffp-contract=off", "-pthread", "-static-libasan", "-static-libubsan", *SAN, str(ROOT / "tests" / "sanitize" / "oracle_driver.cpp"),
         str(ROOT / "oracle" / "ann_oracle.cpp"), str(ROOT / "inputs" / "gen.cpp"), "-o", str(exe)])
    out = run([str(exe)], env=ENV)
    assert "clean" in out.stdout


def test_library_argument_checks_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not shutil.which(hipcc):
        pytest.skip("hipcc not found")
    csrc = ROOT / "paper_2503_17911_amd" / "csrc"
    host = ["--offload-arch=gfx950", "--cuda-host-only", "-std=c++17", "-ffp-contract=off", "-I", str(ROOT / "include"),
            "-I", str(csrc), *SAN]
    objs = []
    for src in sorted(csrc.glob("*.hip")):
        obj = tmp_path / (src.stem + ".o")
        run([hipcc, *host, "-c", str(src), "-o", str(obj)])
        objs.append(str(obj))
    drv = tmp_path / "abi_driver.o"
    run([hipcc, *host, "-x", "c++", "-c", str(ROOT / "tests" / "sanitize" / "abi_driver.cpp"), "-o", str(drv)])
    # a host-only build refers to the device code objects it would embed: give it empty ones
    syms = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", run(["nm", "-u", *objs]).stdout)))
    stub = tmp_path / "stub.c"
    stub.write_text("".join(f"__attribute__((aligned(4096))) char {s}[4096] = {{0}};\n" for s in syms))
    run(["gcc", "-c", str(stub), "-o", str(tmp_path / "stub.o")])
    exe = tmp_path / "abi_driver"
    run([hipcc, "--offload-arch=gfx950", "--cuda-host-only", "-fsanitize=address,undefined", *objs, str(drv),
         str(tmp_path / "stub.o"), "-o", str(exe)])
    out = run([str(exe)], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))   # the HIP runtime keeps its own allocations
    assert "0 unexpected results" in out.stdout
