"""Static checks of the generated gfx950 code (no GPU): accumulator discipline and register budget.

The GEMM kernel keeps its MFMA accumulators in accumulation registers that only its own asm
statements name.  Two things would silently break results and are therefore checked on the
compiler's output:
  * compiler-generated code touching an accumulation register (a copy or spill placed right after
    an MFMA would read a stale value: the hardware does not interlock that case);
  * an accumulator read that is not separated from the last MFMA by the drain (s_nop 15 x 2).
The flagship configuration must also stay within 256 registers per lane, which is what lets two
work-groups share a CU.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2601_18511_amd import build as hip_build


@pytest.fixture(scope="module")
def device_asm():
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "pcmm.s")
        flags = [f for f in hip_build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
        cmd = [hip_build.hipcc_path()] + flags + ["--cuda-device-only", "-S", "-o", out, hip_build.SRC]
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert proc.returncode == 0, proc.stdout
        with open(out) as f:
            return f.read()


def _kernels(asm):
    for m in re.finditer(r"^(_ZN\S*gemm_kernel\S+):[^\n]*\n(.*?)^\.Lfunc_end", asm, re.S | re.M):
        yield m.group(1), m.group(2).split("\n")


def test_accumulators_are_touched_only_by_the_kernels_own_asm(device_asm):
    n = 0
    for name, lines in _kernels(device_asm):
        n += 1
        in_asm = False
        seen_last_mfma_at = max(i for i, l in enumerate(lines) if "v_mfma" in l)
        drained = False
        for i, line in enumerate(lines):
            if "#ASMSTART" in line:
                in_asm = True
                continue
            if "#ASMEND" in line:
                in_asm = False
                continue
            code = line.split(";")[0]
            if not in_asm:
                assert not re.search(r"\ba\[?\d", code) and "accvgpr" not in code, (name, line)
                continue
            if i > seen_last_mfma_at:
                if "s_nop 15" in code:
                    drained = True
                if "v_accvgpr_read" in code:
                    assert drained, (name, "accumulator read before the drain", line)
        assert drained, name
    assert n >= 20


def test_register_budget_allows_two_workgroups_per_cu(device_asm):
    found = {}
    for m in re.finditer(r"- \.agpr_count:\s+(\d+).*?\.name:\s+(\S+).*?\.vgpr_count:\s+(\d+)\s+\.vgpr_spill_count:\s+(\d+)",
                         device_asm, re.S):
        agpr, name, total, spill = int(m.group(1)), m.group(2), int(m.group(3)), int(m.group(4))
        if "gemm_kernel" in name:
            assert spill == 0, name
            found[name] = (agpr, total)
    # WM=4, MT=4, NT=2, D=5, S=1, double-precision epilogue: the Llama projection kernel
    flagship = [v for k, v in found.items() if "ILi4ELi4ELi2ELi5ELi1ELi0E" in k]
    assert len(flagship) == 1
    assert flagship[0][0] == 160 and flagship[0][1] <= 256, flagship
    # every 4-wave kernel (the ones large matrices run) fits two work-groups per CU
    big = {k: v for k, v in found.items() if "gemm_kernelILi4E" in k}
    assert len(big) >= 15
    for k, (agpr, total) in big.items():
        assert total <= 256, (k, agpr, total)
