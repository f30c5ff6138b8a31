"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code, run on the CPU.

Two small C programs under tests/sanitize/ are compiled here with `-fsanitize=address,undefined`:
  * oracle_driver.c with oracle/dsfq_oracle.c (gcc): every oracle function on exactly sized heap buffers, ragged sizes;
  * abi_driver.c with csrc/api.hip whose HOST code is instrumented (the device code is not: sanitizers for the GPU are
    not used anywhere here): the argument validation and the size arithmetic of every entry point, at the ends of the
    argument ranges, all of which is answered before the first HIP call and so needs no GPU.
A sanitizer report aborts the program, so the tests only look at the exit status and print what the program wrote.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd[:3])} ... failed ({r.returncode}):\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    return r


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-o", exe,
          os.path.join(ROOT, "oracle", "dsfq_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-lm"])
    r = _run([exe], env=ENV)
    assert "0 failed checks" in r.stdout


def test_abi_validation_under_address_and_ub_sanitizers(tmp_path):
    from paper_2509_21302_amd import build as B
    if not shutil.which(B.HIPCC) and not os.path.exists(B.HIPCC):
        pytest.skip("hipcc is not installed")
    others = [os.path.join(B.BUILD, os.path.splitext(s)[0] + ".o") for s in B.SOURCES if s != "api.hip"]
    api_src = os.path.join(B.CSRC, "api.hip")
    newest_source = max(os.path.getmtime(os.path.join(B.CSRC, f)) for f in os.listdir(B.CSRC))
    if not all(os.path.exists(o) and os.path.getmtime(o) >= newest_source for o in others):
        B.build()                               # the other objects carry the kernels api.hip launches; plain builds of them do
    api_obj, drv_obj, exe = (str(tmp_path / n) for n in ("api_san.o", "abi_driver.o", "abi_san"))
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    flags = [f for f in B.FLAGS if f != "-O3"]
    _run([B.HIPCC, *flags, "-O1", "-g", *host_san, "-c", api_src, "-o", api_obj])
    _run([B.HIPCC, "-x", "c", "-std=c11", "-O1", "-g", "-I", B.INCLUDE, "-fsanitize=address,undefined", "-c",
          os.path.join(SAN, "abi_driver.c"), "-o", drv_obj])
    _run([B.HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-o", exe, drv_obj, api_obj, *others])
    # the HIP runtime keeps its own allocations until the process ends: leaks are not what this run looks for
    r = _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
    assert "0 mismatches" in r.stdout
