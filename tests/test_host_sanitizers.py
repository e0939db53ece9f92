"""The library's host-side layout, packing and workspace-size code under AddressSanitizer and
UndefinedBehaviorSanitizer (CPU only: the sources are compiled for the host alone, no device code and no
GPU).  tests/host_sanitize/layout_driver.hip drives the packers over the shape grid of the GPU tests with
output buffers of exactly the reported size, so any index past the end is a sanitizer error."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1911_13252_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = ("api.hip", "hidden.hip", "hidden_fused.hip", "hidden_split.hip", "hidden_tiny.hip", "hidden_diag.hip",
           "hidden_fc.hip", "specrad.hip", "tsqr.hip", "solve.hip", "solve_static.hip", "probe.hip")
FLAGS = ["--offload-host-only", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
         "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_host_layout_code_is_clean_under_asan_and_ubsan(tmp_path):
    objs = []
    jobs = []
    for src in SOURCES + ("layout_driver.hip",):
        path = os.path.join(CSRC, src) if src != "layout_driver.hip" else os.path.join(ROOT, "tests", "host_sanitize", src)
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        jobs.append((src, subprocess.Popen([HIPCC, *FLAGS, "-c", path, "-o", obj], stdout=subprocess.PIPE,
                                           stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in jobs:
        out, _ = p.communicate()
        assert p.returncode == 0, f"{src}:\n{out[-3000:]}"
    # no device code was compiled, so the device binaries the host objects refer to are empty stand-ins
    # (nothing launches a kernel here; the HIP runtime is linked only so that its host calls resolve)
    nm = subprocess.run(["nm", "-u", *objs], stdout=subprocess.PIPE, text=True, check=True).stdout
    fatbins = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", nm)))
    stub = tmp_path / "fatbin_stubs.cpp"
    stub.write_text("".join(f'extern "C" {{ extern const unsigned long long {n}[2]; '
                            f'const unsigned long long {n}[2] = {{0, 0}}; }}\n' for n in fatbins))
    subprocess.run([HIPCC, "-c", str(stub), "-o", str(tmp_path / "fatbin_stubs.o")], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    objs.append(str(tmp_path / "fatbin_stubs.o"))
    exe = str(tmp_path / "layout_driver")
    link = subprocess.run([HIPCC, "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, *objs],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert link.returncode == 0, link.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout[-4000:]
    assert run.stdout.strip().splitlines()[-1].startswith("OK "), run.stdout[-2000:]
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout
    # the instrumentation is live: a packer given a buffer one float short is stopped with a report
    bad = subprocess.run([exe, "--selftest"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                         timeout=120)
    assert bad.returncode != 0 and "AddressSanitizer: heap-buffer-overflow" in bad.stdout, bad.stdout[-2000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
