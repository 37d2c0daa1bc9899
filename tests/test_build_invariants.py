"""Static checks on the generated gfx950 code of the bf16 Gram kernels (CPU only: hipcc
cross-compiles).  The hot loop is written in an exact issue order around its 32 MFMAs per
32-token stage; it must not have been duplicated or peeled by the compiler, and no register
spill (scratch access) may sit inside it.  Outside the loop the kernel does spill, so it
must never run with some lanes switched off: spill code that the compiler places inside a
lane-masked region saves only the active lanes (this dropped accumulator lanes in an earlier
form of the epilogue that branched per element); the kernel therefore masks H accesses
through out-of-range buffer offsets and contains no write to EXEC at all."""
import os
import re
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_07004_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_hot_loop_of_the_gram_kernel_is_compact_and_spill_free():
    from paper_2505_07004_amd import build as b
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc] + b.HIPCC_FLAGS + ["-I", b.INCLUDE, "-I", CSRC, "-S", "--cuda-device-only",
                                      os.path.join(CSRC, "fisher_gram_bf16.hip"), "-o", "-"]
    asm = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, check=True).stdout
    kernels = re.findall(r"^(_ZN2gq\S*fisher_gram_bf16_kernel\S*):[^\n]*\n(.*?)s_endpgm", asm, flags=re.S | re.M)
    assert len(kernels) == 6                      # groups per workgroup (4, 2, 1) x one or two terms of the scaled operand
    for name, body in kernels:
        lines = body.splitlines()
        mfma = [i for i, l in enumerate(lines) if "v_mfma_f32_32x32x16_bf16" in l]
        # 2 sub-steps x 16 MFMAs (x 2 terms), exactly once: the loop was neither unrolled further nor peeled
        two_terms = "Lb1E" in name
        assert len(mfma) == (64 if two_terms else 32), (name, len(mfma))
        loop = lines[mfma[0]:mfma[-1] + 1]
        assert not [l for l in loop if "scratch_" in l], f"{name}: register spill inside the hot loop"
        # the direct loads of one stage and the single barrier per stage are in there too
        assert sum("global_load_lds_dword" in l for l in loop) >= 5, name
        assert sum("s_barrier" in l for l in lines[mfma[0] - 80:mfma[-1]]) == 1, name
        writes_exec = [l for l in lines if re.search(r"saveexec|\bs_\w+\s+exec(_lo|_hi)?\s*,", l)]
        assert not writes_exec, (name, writes_exec[:3])
    # the second-pass kernels do mask lanes with branches, so they must not spill at all
    fixups = re.findall(r"^(_ZN2gq\S*fisher_gram_fixup_kernel\S*):[^\n]*\n(.*?)s_endpgm", asm, flags=re.S | re.M)
    assert len(fixups) == 3
    for name, body in fixups:
        assert "scratch_" not in body, name


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_wide_gram_kernel_token_loop_is_the_generated_assembly_and_nothing_else():
    """The wide kernel's token loop is generated inline assembly, one statement per number of live 32-column
    fragments, in two variants (four groups on one row block: ring of 6 stages, 6 direct loads per wave and
    stage; two groups on two row blocks: ring of 5, 8 loads): 2 + 2 x stages sub-steps of 3 x nb matrix
    instructions (one peeled, the unrolled ring stages of two, one tail), with its own register plan.  The
    compiler must have placed the 24 accumulator tiles in both register files without touching the statement,
    the code it generates around it must not write EXEC (spill code inside a lane-masked region saves only
    the active lanes), and the committed include files must be what the generator produces."""
    from paper_2505_07004_amd import build as b
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    incs = [os.path.join(CSRC, f) for f in ("fisher_gram_bf16_wide_loop.inc", "fisher_gram_bf16_wide2_loop.inc")]
    before = [open(inc).read() for inc in incs]
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_gram_wide_loop.py")], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL,
                   env={k: v for k, v in os.environ.items() if not k.startswith("GQW_")})
    assert [open(inc).read() for inc in incs] == before, "an include file is not the generator's output"
    cmd = [hipcc] + b.HIPCC_FLAGS + ["-I", b.INCLUDE, "-I", CSRC, "-S", "--cuda-device-only",
                                      os.path.join(CSRC, "fisher_gram_bf16_wide.hip"), "-o", "-"]
    asm = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, check=True).stdout
    kernels = dict(re.findall(r"^(_ZN2gq\S*fisher_gram_bf16_wide_kernel\S*):[^\n]*\n(.*?)s_endpgm", asm, flags=re.S | re.M))
    assert len(kernels) == 2
    for name, body in kernels.items():
        stages, loads = (6, 6) if "ILi1E" in name else (5, 8)            # template argument: row blocks per item
        assert ("ILi1E" in name) != ("ILi2E" in name), name
        sub_steps = 2 + 2 * stages
        lines = body.splitlines()
        start, end = [i for i, l in enumerate(lines) if "#ASMSTART" in l], [i for i, l in enumerate(lines) if "#ASMEND" in l]
        assert len(start) == 8 and len(end) == 8, name                       # one statement per number of live fragments, 8 .. 1
        inside = set()
        all_dests = None
        blocks = sorted(zip(start, end), key=lambda ab: -sum("v_mfma" in l for l in lines[ab[0]:ab[1] + 1]))   # the compiler orders the cases
        for nb, (a, b2) in zip(range(8, 0, -1), blocks):
            loop = lines[a:b2 + 1]
            inside.update(range(a, b2 + 1))
            mfma = [l for l in loop if "v_mfma_f32_32x32x16_bf16" in l]
            assert len(mfma) == sub_steps * 3 * nb, (name, nb, len(mfma))
            assert not [l for l in loop if "scratch_" in l]
            dests = {l.split()[1].rstrip(",") for l in mfma}
            assert len(dests) == 3 * nb
            if nb == 8:
                all_dests = dests
                assert sum(d.startswith("a[") for d in dests) == 16 and sum(d.startswith("v[") for d in dests) == 8   # both files
                for d in dests:                                              # none of them inside the statement's own registers
                    lo = int(re.match(r"[av]\[(\d+):", d).group(1))
                    assert d.startswith("a[") or lo >= 84, d
            else:
                assert dests <= all_dests                                    # the same tiles in every statement
            assert sum("s_barrier" in l for l in loop) == stages + 1
            assert sum("global_load_lds_dwordx4" in l for l in loop) == (stages - 1) * loads + stages * loads
        assert len([l for l in lines if "v_mfma" in l]) == sub_steps * 3 * 36
        outside = [l for i, l in enumerate(lines) if i not in inside]
        writes_exec = [l for l in outside if re.search(r"saveexec|\bs_\w+\s+exec(_lo|_hi)?\s*,", l)]
        assert not writes_exec, (name, writes_exec[:3])
    (fname, fbody), = re.findall(r"^(_ZN2gq\S*fisher_gram_wide_fixup_kernel\S*):[^\n]*\n(.*?)s_endpgm", asm, flags=re.S | re.M)
    assert "scratch_" not in fbody
