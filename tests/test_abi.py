"""The C-ABI library loads without a GPU, exports every symbol the header declares, and turns bad
arguments into status codes (no compute calls here)."""
import ctypes
import os
import re

import pytest

import paper_2601_18511_amd as pkg
from paper_2601_18511_amd import pcmm as binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pcmm.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pcm[mv]_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    lib = pkg.load_library()
    names = _declared_functions()
    assert len(names) >= 7
    for name in names:
        assert getattr(lib, name) is not None, name
        assert hasattr(pkg, name), "python binding lacks " + name
    assert sorted(binding.EXPORTED) == names


def test_status_strings():
    for code in range(5):
        assert pkg.pcmm_status_str(code).startswith("PCMM_")
    assert "unknown" in pkg.pcmm_status_str(99)


def test_argument_validation_needs_no_device():
    lib = pkg.load_library()
    out = ctypes.c_void_p(123)
    q = (ctypes.c_uint64 * 1)(68719403009)
    dummy = ctypes.c_void_p(0x1000)     # never dereferenced: validation fails first
    qp = ctypes.cast(q, ctypes.c_void_p)

    def create(M=4, K=4, N=4, L=1, primes=qp, bits=36, wbits=8, W=dummy, dev=0):
        return lib.pcmm_plan_create(ctypes.byref(out), M, K, N, L, primes, bits, wbits, W, dev, None)

    assert create(M=0) == binding.PCMM_EINVAL and out.value is None
    assert create(K=-1) == binding.PCMM_EINVAL
    assert create(L=0) == binding.PCMM_EINVAL
    assert create(L=65) == binding.PCMM_EINVAL
    assert create(primes=None) == binding.PCMM_EINVAL
    assert create(W=None) == binding.PCMM_EINVAL
    assert create(wbits=12) == binding.PCMM_EINVAL
    assert create(bits=35) == binding.PCMM_EINVAL          # prime not of that size
    assert create(bits=63) == binding.PCMM_EINVAL
    assert create(dev=-1) == binding.PCMM_EINVAL
    even = (ctypes.c_uint64 * 1)(68719403008)
    assert create(primes=ctypes.cast(even, ctypes.c_void_p)) == binding.PCMM_EINVAL
    assert create(K=(1 << 22) - 127) == binding.PCMM_EINVAL   # largest K is 2^22 - 128
    assert create(M=(1 << 24) + 1) == binding.PCMM_EINVAL
    assert create(N=(1 << 22) + 1) == binding.PCMM_EINVAL
    assert lib.pcmm_plan_create(None, 4, 4, 4, 1, qp, 36, 8, dummy, 0, None) == binding.PCMM_EINVAL
    assert lib.pcmm_run(None, dummy, dummy, None) == binding.PCMM_EINVAL
    assert lib.pcmm_run_profiled(None, dummy, dummy, None, None) == binding.PCMM_EINVAL
    assert lib.pcmm_plan_workspace_bytes(None) == 0
    assert lib.pcmm_plan_digits(None) == 0
    lib.pcmm_plan_destroy(None)
    tops, mhz = ctypes.c_double(), ctypes.c_double()
    assert lib.pcmm_mfma_probe(-1, 10, 1, ctypes.byref(tops), ctypes.byref(mhz)) == binding.PCMM_EINVAL
    assert lib.pcmm_mfma_probe(0, 0, 1, ctypes.byref(tops), ctypes.byref(mhz)) == binding.PCMM_EINVAL
    assert lib.pcmm_mfma_probe(0, 10, 1, None, ctypes.byref(mhz)) == binding.PCMM_EINVAL
    for fn in (lib.pcmm_ring_decompose, lib.pcmm_ring_compose):
        assert fn(None, dummy, 1, 64, 8, 0, None) == binding.PCMM_EINVAL
        assert fn(dummy, dummy, 1, 64, 8, 0, None) == binding.PCMM_EINVAL          # aliased
        other = ctypes.c_void_p(0x2000)
        assert fn(dummy, other, 0, 64, 8, 0, None) == binding.PCMM_EINVAL
        assert fn(dummy, other, 1, 96, 8, 0, None) == binding.PCMM_EINVAL          # N not a power of two
        assert fn(dummy, other, 1, 64, 3, 0, None) == binding.PCMM_EINVAL
        assert fn(dummy, other, 1, 64, 128, 0, None) == binding.PCMM_EINVAL        # k > N
        assert fn(dummy, other, 1, 64, 8, -1, None) == binding.PCMM_EINVAL
        assert fn(dummy, other, 1 << 36, 1 << 16, 8, 0, None) == binding.PCMM_EUNSUPPORTED


def test_slot_rearrange_argument_validation_needs_no_device():
    lib = pkg.load_library()
    a, b = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)     # never dereferenced: validation fails first
    f = lib.pcmm_slot_rearrange
    assert f(None, b, 1, 8, 1, 2, 0, 8, 0, None) == binding.PCMM_EINVAL
    assert f(a, a, 1, 8, 1, 2, 0, 8, 0, None) == binding.PCMM_EINVAL          # aliased
    assert f(a, b, 0, 8, 1, 2, 0, 8, 0, None) == binding.PCMM_EINVAL
    assert f(a, b, 1, 0, 1, 2, 0, 8, 0, None) == binding.PCMM_EINVAL
    assert f(a, b, 1, 8, 1, 3, 0, 8, 0, None) == binding.PCMM_EINVAL          # b does not divide d
    assert f(a, b, 1, 8, 1, 2, 0, 9, 0, None) == binding.PCMM_EINVAL          # run of plaintexts past d
    assert f(a, b, 1, 8, 1, 2, -1, 2, 0, None) == binding.PCMM_EINVAL
    assert f(a, b, 1, 8, 1, 2, 0, 8, -1, None) == binding.PCMM_EINVAL
    assert f(a, b, 1, 40000, 1, 2, 0, 8, 0, None) == binding.PCMM_EUNSUPPORTED
    assert f(a, b, 1 << 30, 4096, 1, 2, 0, 8, 0, None) == binding.PCMM_EUNSUPPORTED


def test_pcmv_argument_validation_needs_no_device():
    lib = pkg.load_library()
    out = ctypes.c_void_p(123)
    dummy = ctypes.c_void_p(0x1000)     # never dereferenced: validation fails first
    N = 64
    q = (ctypes.c_uint64 * 1)(68719475713)          # 2^36 - 2^10 + 1... any odd 36-bit number = 1 mod 128 will do for these checks
    q[0] = ((1 << 36) - 1) // 128 * 128 + 1
    qp = ctypes.cast(q, ctypes.c_void_p)

    def create(Mp=2, Kp=1, n=N, L=1, primes=qp, bits=36, pt=dummy, dev=0):
        return lib.pcmv_plan_create(ctypes.byref(out), Mp, Kp, n, L, primes, bits, pt, dev, None)

    assert create(Mp=0) == binding.PCMM_EINVAL and out.value is None
    assert create(Kp=0) == binding.PCMM_EINVAL
    assert create(n=1) == binding.PCMM_EINVAL
    assert create(n=96) == binding.PCMM_EINVAL                 # not a power of two
    assert create(L=0) == binding.PCMM_EINVAL
    assert create(L=65) == binding.PCMM_EINVAL
    assert create(primes=None) == binding.PCMM_EINVAL
    assert create(pt=None) == binding.PCMM_EINVAL
    assert create(bits=35) == binding.PCMM_EINVAL              # prime not of that size
    assert create(dev=-1) == binding.PCMM_EINVAL
    assert create(n=1 << 20) == binding.PCMM_EINVAL            # q is not 1 mod 2N
    assert create(n=8192) in (binding.PCMM_EINVAL, binding.PCMM_EUNSUPPORTED)
    assert create(Kp=5000) == binding.PCMM_EUNSUPPORTED
    big = (ctypes.c_uint64 * 1)(((1 << 56) - 1) // 128 * 128 + 1)
    assert create(primes=ctypes.cast(big, ctypes.c_void_p), bits=56) == binding.PCMM_EUNSUPPORTED
    assert lib.pcmv_plan_create(None, 2, 1, N, 1, qp, 36, dummy, 0, None) == binding.PCMM_EINVAL
    assert lib.pcmv_run(None, dummy, dummy, None) == binding.PCMM_EINVAL
    assert lib.pcmv_plan_workspace_bytes(None) == 0
    lib.pcmv_plan_destroy(None)


def test_header_is_plain_c(tmp_path):
    """include/pcmm.h compiles as C99 and as C++ and declares what the binding expects."""
    import shutil
    import subprocess

    src = tmp_path / "use_pcmm.c"
    src.write_text(
        '#include "pcmm.h"\n'
        "int main(void) {\n"
        "    pcmm_plan *p = 0;\n"
        "    pcmm_status s = pcmm_plan_create(&p, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "    (void)pcmm_ring_decompose(0, 0, 0, 0, 0, 0, 0);\n"
        "    pcmm_plan_destroy(p);\n"
        "    return s == PCMM_EINVAL ? 0 : 1;\n"
        "}\n"
    )
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        if shutil.which(cc) is None:
            pytest.skip("no %s" % cc)
        args = [cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc]
        if cc == "g++":
            args += ["-x", "c++"]
        subprocess.run(args + [str(src)], check=True)
    # and a C program linked against the built library runs the argument checks without a device
    exe = tmp_path / "use_pcmm"
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", os.path.dirname(pkg.build.LIB),
                    "-l:libpcmm.so", "-Wl,-rpath," + os.path.dirname(pkg.build.LIB)], check=True)
    assert subprocess.run([str(exe)]).returncode == 0
