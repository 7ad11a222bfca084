"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two things run sanitized here:
  * the library's host-side planning (argument validation, digit count, tile geometry, buffer sizes,
    k-step offsets, per-limb constants) -- csrc/pcmm_host.hpp compiled into tests/host/plan_geometry_check.cpp,
    and the PCMv planning (roots of unity, twiddle tables) -- csrc/pcmv_host.hpp in tests/host/pcmv_tables_check.cpp;
  * the C oracles: pcmm_oracle.c and pcmv_oracle.c are built a second time with the sanitizers and their pins run
    on those builds in a child interpreter (the sanitizer runtime has to be loaded before python starts).
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]


def _need(tool):
    if shutil.which(tool) is None:
        pytest.skip("no %s" % tool)


def test_plan_geometry_under_sanitizers(tmp_path):
    _need("g++")
    exe = tmp_path / "plan_geometry_check"
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror"] + SAN +
                   ["-I", os.path.join(ROOT, "paper_2601_18511_amd", "csrc"), "-o", str(exe),
                    os.path.join(ROOT, "tests", "host", "plan_geometry_check.cpp")], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all checks held" in r.stdout


def test_pcmv_tables_under_sanitizers(tmp_path):
    _need("g++")
    exe = tmp_path / "pcmv_tables_check"
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror"] + SAN +
                   ["-I", os.path.join(ROOT, "paper_2601_18511_amd", "csrc"), "-o", str(exe),
                    os.path.join(ROOT, "tests", "host", "pcmv_tables_check.cpp")], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all checks held" in r.stdout


def test_oracle_pins_under_sanitizers(tmp_path):
    _need("gcc")
    lib = tmp_path / "libpcmm_oracle_san.so"
    lib2 = tmp_path / "libpcmv_oracle_san.so"
    for out, src in ((lib, "pcmm_oracle.c"), (lib2, "pcmv_oracle.c")):
        subprocess.run(["gcc", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"] + SAN +
                       ["-o", str(out), os.path.join(ROOT, "oracle", src)], check=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no shared AddressSanitizer runtime")
    env = dict(os.environ)
    env["PCMM_ORACLE_LIB"] = str(lib)
    env["PCMV_ORACLE_LIB"] = str(lib2)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0"                      # the interpreter's own allocations are not ours
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_pcmv_oracle.py")],
                       capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
