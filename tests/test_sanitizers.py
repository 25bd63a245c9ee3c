"""Address and undefined-behaviour sanitizer builds of the host code that works on caller-supplied tables and
text: the CPU oracle (encoder, decoder, pre-tokenizer, trainer) and the host-only parts of the library (rule
validation, slot-image placement, vocabulary expansions).  Each driver under tests/sanitize/ runs them on seeded
valid and invalid inputs; a report from a sanitizer ends the driver with a non-zero status.  No GPU is used: the
device code of the two library sources is compiled but never launched.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVERS = os.path.join(ROOT, "tests", "sanitize")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, f"{exe}:\n{r.stdout}\n{r.stderr}"
    return r.stdout


def _instrumented(exe):
    syms = subprocess.run(["nm", exe], capture_output=True, text=True).stdout
    return "__asan_report" in syms and "__ubsan_handle" in syms


def test_oracle_under_sanitizers(tmp_path):
    objs = []
    for src, cc, std in (("oracle/bpe_oracle.c", "gcc", "-std=c11"), ("oracle/bpe_trainer.cpp", "g++", "-std=c++17"),
                         ("tests/sanitize/oracle_driver.c", "gcc", "-std=c11")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.check_call([cc, "-g", "-O1", std, "-Wall", *SAN, "-c", os.path.join(ROOT, src), "-o", obj])
        objs.append(obj)
    exe = str(tmp_path / "oracle_san")
    # the runtimes are linked in: a preloaded library may then come first without upsetting them
    subprocess.check_call(["g++", *SAN, "-static-libasan", "-static-libubsan", *objs, "-lpthread", "-o", exe])
    assert _instrumented(exe)
    assert "ok" in _run(exe)


def test_host_builders_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2603_02597_amd", "csrc")
    exe = str(tmp_path / "host_san")
    host_san = [a for flag in SAN for a in ("-Xarch_host", flag)]      # the device code is built as always
    subprocess.check_call([hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unused-command-line-argument", *host_san,
                           "-I", os.path.join(ROOT, "include"), "-I", csrc,
                           os.path.join(csrc, "bpe_table.hip"), os.path.join(csrc, "bpe_vocab.hip"),
                           os.path.join(DRIVERS, "host_builders_driver.cpp"), "-o", exe],
                          stderr=subprocess.DEVNULL)
    assert _instrumented(exe)
    assert "ok" in _run(exe)
