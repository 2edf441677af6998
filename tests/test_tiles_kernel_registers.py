"""The multi-tile matrix-core kernel keeps state in registers the compiler must not touch.

micro_attention_mfma_tiles.hip compiles its own code for vector registers below tiles_asm::kFirstOwnVgpr and leaves
the registers above it, and the whole accumulation file, to hand-written statements (tiles_asm.h) that keep
accumulators, operands and softmax state there from one statement to the next.  Nothing tells the compiler that
those registers are live, so this test compiles the file to assembly and checks that no instruction outside the
hand-written statements names one of them, that nothing was spilled, and that the kernels are given the whole
register file.  The generated header must also be what the generator writes.
"""
import os
import re
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_02669_amd", "csrc")
sys.path.insert(0, ROOT)


def compile_to_asm():
    from paper_2401_02669_amd import build
    out = os.path.join(tempfile.mkdtemp(prefix="tiles_asm_"), "tiles.s")
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["-S", "--cuda-device-only", "-o", out,
                                                                      os.path.join(CSRC, "micro_attention_mfma_tiles.hip")]
    subprocess.run(cmd, check=True, stderr=subprocess.DEVNULL)
    return open(out).read().split("\n")


def test_generated_header_is_current():
    sys.path.insert(0, CSRC)
    import gen_tiles_asm
    assert gen_tiles_asm.emit() == open(os.path.join(CSRC, "tiles_asm.h")).read(), "run python csrc/gen_tiles_asm.py"


def test_compiler_code_stays_out_of_the_hand_allocated_registers():
    sys.path.insert(0, CSRC)
    import gen_tiles_asm
    cap = gen_tiles_asm.CAP
    lines = compile_to_asm()
    in_asm, kernel, bad, kernels = False, None, [], set()
    for n, line in enumerate(lines):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = re.match(r"^(_Z\S*micro_attention_mfma_tiles_kernel\S*):", line)
        if m:
            kernel = m.group(1)
            kernels.add(kernel)
        if in_asm or not t or t.startswith((";", ".")):
            continue
        code = t.split(";")[0]
        if re.search(r"\ba\[?\d+", code) or "accvgpr" in code or code.startswith("scratch_"):
            bad.append((kernel, n, code))
        for mm in re.finditer(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]", code):
            if int(mm.group(1) or mm.group(3)) >= cap:
                bad.append((kernel, n, code))
    assert len(kernels) == 3, kernels  # <2,1>, <4,1>, <4,2>
    assert not bad, bad[:10]
    text = "\n".join(lines)
    # each kernel owns the whole register file (256 + 256) and spills nothing
    assert text.count(".amdhsa_next_free_vgpr 512") == 3 and text.count(".amdhsa_accum_offset 256") == 3
    assert re.findall(r"\.vgpr_spill_count:\s+(\d+)", text) == ["0"] * 3
