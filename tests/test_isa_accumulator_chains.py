"""Build-time guard for the MFMA chains that start from the inline-constant accumulator.

The first MFMA of such a chain is a volatile asm statement (the compiler folds a constant accumulator into the
instruction only when the constant has a single use).  The compiler's hazard handling does not know that statement is an
MFMA, so nothing but the next MFMA of the chain -- accumulating in place, which may follow back to back -- may touch its
result registers (or, where a chain of a masked block can end with its first MFMA, an explicit run of s_nop stands in
front of the first reader).  The register allocator decides the former; this test compiles the attention kernels to
assembly and checks every chain start in every instantiation, scanning the text linearly."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2409_16997_amd import build as hip_build

REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")


def _regs(text):
    out = set()
    for kind, single, lo, hi in REG.findall(text):
        if single:
            out.add((kind, int(single)))
        else:
            out.update((kind, i) for i in range(int(lo), int(hi) + 1))
    return out


@pytest.mark.timeout(600)
def test_nothing_but_the_next_mfma_of_its_chain_touches_a_chain_start_result():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    flags = [f for f in hip_build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attn.s")
        src = os.path.join(hip_build.CSRC, "intfa_attention.hip")
        subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-I", hip_build.INCLUDE, "-I", hip_build.CSRC, src, "-o", out],
                       check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        lines = open(out).read().splitlines()
    # Only the fused kernel writes its chain starts as assembly; in the other kernels of the file an MFMA with the same
    # inline constant is the compiler's own (it folds a single-use splat) and carries the compiler's hazard handling.
    func, owner = None, []
    for ln in lines:
        m = re.match(r"^(_Z\w+):", ln)
        if m:
            func = m.group(1)
        owner.append(func)
    starts = [i for i, ln in enumerate(lines) if "v_mfma_i32_32x32x32_i8" in ln and ln.rstrip().endswith("0.15915494")
              and owner[i] and "int_flash_attn_fwd_kernel" in owner[i]]
    assert len(starts) >= 8 * 24, f"expected the chain starts of every instantiation, found {len(starts)}"
    for i in starts:
        dst_txt = lines[i].split("v_mfma_i32_32x32x32_i8")[1].split(",")[0]
        dst = _regs(dst_txt)
        assert len(dst) == 16
        nops = 0
        for j in range(i + 1, len(lines)):
            ln = lines[j].split(";")[0].strip()
            if not ln or ln.startswith((".", "#")) or ln.endswith(":"):
                continue                                             # labels, directives: the scan is textual, branches fall through
            if ln.startswith("s_endpgm"):
                raise AssertionError(f"chain of line {i + 1} never continues")
            if ln.startswith("s_nop 15"):
                nops += 1
            if ln.startswith("v_mfma_i32_32x32x32_i8"):
                ops = [o.strip() for o in ln[len("v_mfma_i32_32x32x32_i8"):].split(",")]
                if _regs(ops[0]) == dst:
                    assert _regs(ops[3]) == dst, f"line {j + 1}: overwrites the result of line {i + 1} without accumulating it"
                    assert not (_regs(ops[1]) | _regs(ops[2])) & dst
                    break
            # in a masked block a chain may end with its first MFMA: then four s_nop 15 stand between it and the first reader
            assert nops >= 4 or not _regs(ln) & dst, f"line {j + 1} touches the result of the chain start at line {i + 1}: {ln}"
            if nops >= 4 and _regs(ln) & dst:
                break
