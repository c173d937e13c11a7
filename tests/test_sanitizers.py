"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU:
  * the oracle (plain C) on small seeded inputs through every entry point;
  * the library's host side -- the argument checks of its entry points and the Huffman builder --
    compiled host-only (no device code, no device touched).
Each program prints "ok"; a sanitizer report ends it with a non-zero status."""
import concurrent.futures
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="2")


def run_ok(exe):
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=ENV)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-2000:] + r.stderr[-4000:]


def test_oracle_under_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("gcc not found")
    exe = str(tmp_path / "oracle_sanitize")
    cmd = [gcc, "-std=c11", "-fopenmp"] + SAN + [os.path.join(ROOT, "oracle", "rnnlm_oracle.c"),
                                                 os.path.join(ROOT, "tests", "host", "oracle_sanitize.c"), "-lm", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    run_ok(exe)


def test_library_host_side_under_sanitizers(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    from paper_2007_11794_amd import build as lib_build
    csrc = os.path.join(ROOT, "paper_2007_11794_amd", "csrc")
    host = [hipcc, "--cuda-host-only", "-x", "hip", "-std=c++17"] + SAN + \
           ["-I" + os.path.join(ROOT, "include"), "-I" + csrc]
    jobs = [(os.path.join(csrc, s), str(tmp_path / (s + ".o"))) for s in lib_build.SOURCES]
    jobs.append((os.path.join(ROOT, "tests", "host", "abi_sanitize.cpp"), str(tmp_path / "driver.o")))

    def compile_one(job):
        return subprocess.run(host + ["-c", job[0], "-o", job[1]], capture_output=True, text=True)

    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as pool:
        for job, r in zip(jobs, pool.map(compile_one, jobs)):
            assert r.returncode == 0, job[0] + "\n" + r.stderr[-3000:]
    objects = [j[1] for j in jobs]
    # A host-only object still refers to the device code that a full build would embed beside it:
    # stand in for each with an empty bundle, which the runtime would find no kernel in (none is asked for).
    undefined = subprocess.run(["nm", "-u"] + objects, capture_output=True, text=True).stdout
    names = sorted(set(re.findall(r"__hip_fatbin_\w+", undefined)))
    stub = tmp_path / "no_device_code.c"
    stub.write_text("#include <stdint.h>\n" + "".join(
        "__attribute__((aligned(4096))) const struct { char magic[24]; uint64_t entries; } %s = "
        "{\"__CLANG_OFFLOAD_BUNDLE__\", 0};\n" % n for n in names))
    r = subprocess.run(["gcc", "-c", str(stub), "-o", str(tmp_path / "no_device_code.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    exe = str(tmp_path / "abi_sanitize")
    r = subprocess.run([hipcc, "-fsanitize=address,undefined"] + objects + [str(tmp_path / "no_device_code.o"), "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    run_ok(exe)
