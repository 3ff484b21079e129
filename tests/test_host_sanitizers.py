"""Sanitizer builds of everything that runs on the host: the library's host half, the cycle-schedule
code the kernels share with the host, and the oracle.  CPU only; every build goes to a scratch folder.

  * tests/host/schedule_check.cpp: build_schedule (csrc/cx_schedule.hpp) run by a group of real threads
    against a serial cycle walk -- under ThreadSanitizer, where a missing group.sync() is a data race,
    and under AddressSanitizer + UBSan at the largest row count;
  * tests/host/host_half_check.cpp: csrc/cx_host.cpp and oracle/cx_oracle.c in one ASan + UBSan program:
    topologies of both compared for every mode, the table checkers, every oracle function on exact-size
    heap buffers;
  * the oracle's own pin tests re-run against an ASan + UBSan build of the oracle;
  * tests/host/hbm_policy_check.cpp: csrc/cx_hbm.cpp (placement of the matrices in physical memory) against a model
    of device memory behind a stand-in runtime header: where the pieces land, what is given back, and every
    runtime call failing once at every position -- paths that must not be provoked on a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2012_15198_amd", "csrc")
HOST = os.path.join(ROOT, "tests", "host")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = {**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
       "TSAN_OPTIONS": "halt_on_error=1"}


def run(cmd, **kw):
    out = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert out.returncode == 0, f"{' '.join(map(str, cmd))}\n{out.stdout[-3000:]}\n{out.stderr[-6000:]}"
    return out.stdout


def test_cycle_schedule_under_thread_sanitizer(tmp_path):
    exe = tmp_path / "schedule_tsan"
    run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-I", CSRC, os.path.join(HOST, "schedule_check.cpp"),
         "-o", str(exe), "-lpthread"])
    assert run([str(exe), "4", "300"], env=ENV).startswith("ok")
    assert run([str(exe), "3", "70"], env=ENV).startswith("ok")          # a thread count that divides nothing


def test_cycle_schedule_under_address_sanitizer_at_the_maximum_row_count(tmp_path):
    exe = tmp_path / "schedule_asan"
    run(["g++", "-std=c++17", *SAN, "-I", CSRC, os.path.join(HOST, "schedule_check.cpp"), "-o", str(exe), "-lpthread"])
    assert run([str(exe), "7", "1024"], env=ENV).startswith("ok")
    assert run([str(exe), "1", "1024"], env=ENV).startswith("ok")


def test_host_half_and_oracle_under_address_and_ub_sanitizers(tmp_path):
    obj = tmp_path / "cx_oracle.o"
    run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fno-fast-math", "-fexcess-precision=standard", "-Wall", "-Wextra",
         "-c", os.path.join(ROOT, "oracle", "cx_oracle.c"), "-o", str(obj)])
    exe = tmp_path / "host_half"
    run(["g++", "-std=c++17", *SAN, "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"),
         os.path.join(HOST, "host_half_check.cpp"), os.path.join(CSRC, "cx_host.cpp"), str(obj), "-o", str(exe), "-lm"])
    assert run([str(exe)], env=ENV).strip().endswith("ok")


def test_placement_policy_and_its_error_paths_against_a_model_of_device_memory(tmp_path):
    exe = tmp_path / "hbm_policy"
    run(["g++", "-std=c++17", *SAN, "-Wall", "-Wextra", "-I", os.path.join(HOST, "fake_hip"), "-I", os.path.join(ROOT, "include"),
         os.path.join(HOST, "hbm_policy_check.cpp"), os.path.join(CSRC, "cx_hbm.cpp"), "-o", str(exe)])
    assert run([str(exe)], env=ENV).strip().endswith("ok")


def test_oracle_pins_pass_against_a_sanitized_oracle(tmp_path):
    lib = tmp_path / "libcx_oracle_san.so"
    run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fno-fast-math", "-fexcess-precision=standard", "-shared", "-fPIC",
         os.path.join(ROOT, "oracle", "cx_oracle.c"), "-o", str(lib), "-lm"])
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan):
        pytest.skip("no libasan.so next to gcc")
    env = {**ENV, "CX_ORACLE_LIB": str(lib), "LD_PRELOAD": asan, "ASAN_OPTIONS": "detect_leaks=0"}   # python leaks by design
    out = run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
               os.path.join(ROOT, "tests", "test_oracle_topology.py"), os.path.join(ROOT, "tests", "test_oracle_mix.py")],
              env=env, cwd=ROOT)
    assert " passed" in out and "failed" not in out
