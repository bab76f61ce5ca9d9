"""Builds libsage.so (the C-ABI library of hand-written gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsage.so")
SOURCES = ["sage_api.hip", "sage_prepass.hip", "sage_prepass_v.hip", "sage_attn.hip", "sage_attn_pv8.hip",
           "sage_microbench.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                   # quantizer arithmetic: one rounding per operation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
    "-mllvm", "-amdgpu-mfma-vgpr-form",                    # scores must land in VALU-readable registers
    "-Wall", "-Wno-unused-variable",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


HASH_MARKER = b"SAGE_SOURCE_HASH="


def source_files() -> list:
    """Everything the library is compiled from: the kernel sources and headers, and the public header."""
    names = sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    return [os.path.join(CSRC, f) for f in names] + [os.path.join(HERE, "..", "include", "sage.h")]


def source_hash() -> str:
    """SHA-256 over the names and contents of source_files(); compiled into the library, so that a
    built library can be matched against the sources beside it whatever the file times say."""
    import hashlib
    h = hashlib.sha256()
    for path in source_files():
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
        h.update(b"\0")
    return h.hexdigest()


def built_hash(path: str = LIB):
    """The source hash a built library carries (read from the file, nothing is loaded), or None."""
    if not os.path.exists(path):
        return None
    with open(path, "rb") as f:
        blob = f.read()
    at = blob.find(HASH_MARKER)
    if at < 0:
        return None
    digest = blob[at + len(HASH_MARKER): at + len(HASH_MARKER) + 64]
    try:
        return digest.decode("ascii")
    except UnicodeDecodeError:
        return None


def build(verbose: bool = False, extra=()) -> str:
    """Compile every kernel for gfx950 (cross-compiles without a GPU) and return the library path."""
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, f'-DSAGE_SOURCE_HASH="{source_hash()}"', "-o", tmp,
           *[os.path.join(CSRC, s) for s in SOURCES]]
    try:
        res = subprocess.run(cmd, capture_output=True, text=True)
        noise = "packed-fp32-ops"
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + err)
        if verbose and err.strip():
            print(err, file=sys.stderr)
        verify_attention_isa(extra)
        os.replace(tmp, LIB)
    finally:
        if os.path.exists(tmp):         # a failed build or a failed assembly check leaves nothing behind
            os.remove(tmp)
    return LIB


def check_attention_asm(text: str) -> list:
    """Checks the assembly text of the attention kernels for what their hand-placed register use
    relies on (see "Register files" at the top of sage_attn.hip) and returns the list of problems
    found.  The matrix instructions update accumulator registers that they name as inputs, so the
    compiler must keep every accumulator in one place between them:
      - once the first matrix instruction has been issued it never copies an accumulator register
        to another accumulator register (before that, the zero initialisation may),
      - it reads accumulator registers into VGPRs only where the source refreshes them first (the
        rare rescale and the epilogue), i.e. never inside a block that issues matrix instructions
        (AGPRs that no matrix instruction names are the compiler's own parking space and exempt),
      - nothing spills to scratch memory,
      - and it never touches m0, which the hand-written global->LDS loads set.
      - no instruction touches a VGPR within 12 wait states of a matrix instruction writing it
        (except the next matrix instruction of the same accumulation chain), and no matrix
        instruction reads a VGPR that one of the two preceding instructions wrote -- the waits the
        compiler would insert if it knew these were matrix instructions.
    Instructions between ";;#ASMSTART" and ";;#ASMEND" are the source's own assembly."""
    import re
    kernels = re.findall(r"^(_ZN4sage16sage_attn_kernel\w+):.*?^\.Lfunc_end\d+:", text, re.S | re.M)
    bodies = re.findall(r"^_ZN4sage16sage_attn_kernel\w+:.*?^\.Lfunc_end\d+:", text, re.S | re.M)
    problems = []
    # head dimension {64, 128} x workgroup shape {4, 8 wavefronts} x {score dump, causal / full
    # with per-block key scales, causal / full with per-token key scales}, less the two per-token
    # kernels of D = 128 with 4 wavefronts, which are not built; plus the two measurement builds
    # (D = 128, 8 wavefronts, causal / full, with the clock counters)
    if len(bodies) != 20:
        problems.append(f"expected 20 attention kernels in the assembly, found {len(bodies)}")

    def vregs(operand: str) -> set:
        """VGPR numbers named by one operand such as v12 or v[12:15]."""
        m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.fullmatch(r"v(\d+)", operand)
        return {int(m.group(1))} if m else set()

    def aregs(operand: str) -> set:
        """AGPR numbers named by one operand such as a12 or a[12:15]."""
        m = re.fullmatch(r"a\[(\d+):(\d+)\]", operand)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.fullmatch(r"a(\d+)", operand)
        return {int(m.group(1))} if m else set()

    def operands(code: str) -> list:
        parts = code.split(None, 1)
        return [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []

    for name, body in zip(kernels, bodies):
        # AGPRs that matrix instructions name (accumulators, resident operands).  The compiler may
        # park unrelated values in the remaining AGPRs; moving those around is harmless.
        matrix_agprs = set()
        for line in body.split("\n"):
            code = line.split(";")[0].strip()
            if code.startswith("v_mfma"):
                for o in operands(code):
                    matrix_agprs |= aregs(o)
        state = {"mfma": False, "reads": []}
        in_asm = False
        seen_mfma = False
        pending = []          # [registers written by a matrix instruction, wait states since, its text]
        recent = []           # VGPRs written by the last two non-matrix instructions

        def close_block():
            if state["mfma"] and state["reads"]:
                problems.append(f"{name}: accumulator read next to matrix instructions: {state['reads'][0]}")
            state["mfma"], state["reads"] = False, []

        for line in body.split("\n"):
            code = line.split(";")[0].strip()
            if "#ASMSTART" in line:
                in_asm = True
                continue
            if "#ASMEND" in line:
                in_asm = False
                continue
            if re.match(r"^\.LBB\d+_\d+:", line) or code.startswith("s_cbranch") or code.startswith("s_branch"):
                close_block()
                if code.startswith("s_branch"):
                    pending, recent = [], []          # nothing falls through an unconditional branch
                elif code:
                    for p_ in pending:
                        p_[1] += 1
                continue
            if not code or code.startswith("."):
                continue
            ops = operands(code)
            touched = set().union(*[vregs(o) for o in ops]) if ops else set()
            is_mfma = code.startswith("v_mfma")
            # --- hazard windows
            for p_ in pending:
                same_chain = is_mfma and ops and vregs(ops[0]) == p_[0] and vregs(ops[-1]) == p_[0]
                if touched & p_[0] and not same_chain:
                    problems.append(f"{name}: '{code}' touches the result of '{p_[2]}' after {p_[1]} wait states")
            if is_mfma:
                for o in ops[1:]:
                    for w in recent:
                        if vregs(o) & w:
                            problems.append(f"{name}: '{code}' reads a register written less than 2 wait states before")
            m = re.match(r"s_nop\s+(\d+)", code)
            step = int(m.group(1)) + 1 if m else 1
            for p_ in pending:
                p_[1] += step
            pending = [p_ for p_ in pending if p_[1] < 12]
            if is_mfma:
                dst = vregs(ops[0]) if ops else set()
                if dst:
                    pending.append([dst, 0, code])
                recent = []
            else:
                wrote = vregs(ops[0]) if ops and code.startswith("v_") else set()      # VALU results only: loads are covered by s_waitcnt
                recent = ([wrote] + recent)[:2] if step == 1 else []
            # --- register-file rules
            if in_asm:
                if is_mfma:
                    state["mfma"] = True
                    seen_mfma = True
                continue
            named = set().union(*[aregs(o) for o in ops]) if ops else set()
            if code.startswith("v_accvgpr_mov") and seen_mfma and named & matrix_agprs:
                problems.append(f"{name}: accumulator-to-accumulator copy: {code}")
            if code.startswith("v_accvgpr_read") and named & matrix_agprs:
                state["reads"].append(code)
            if code.startswith("scratch_"):
                problems.append(f"{name}: scratch access: {code}")
            if re.search(r"\bm0\b", code):
                problems.append(f"{name}: compiler-generated use of m0: {code}")
        close_block()
    return problems


def check_pv8_asm(text: str) -> list:
    """Checks the assembly text of the INT8-P~V attention kernels (sage_attn_pv8.hip).  Their matrix
    instructions are compiler builtins, so the compiler places the waits itself; what the source
    relies on is only that nothing spills to scratch memory and that the compiler never touches m0,
    which the hand-written global->LDS loads set."""
    import re
    bodies = re.findall(r"^(_ZN4sage20sage_attn_pv8_kernel\w+):(.*?)^\.Lfunc_end\d+:", text, re.S | re.M)
    problems = []
    if len(bodies) != 16:     # head dimension {64, 128} x {causal, full} x {per-block, per-token key scales} x {whole, key chunks}
        problems.append(f"expected 16 INT8-P~V attention kernels in the assembly, found {len(bodies)}")
    for name, body in bodies:
        in_asm = False
        for line in body.split("\n"):
            if "#ASMSTART" in line:
                in_asm = True
                continue
            if "#ASMEND" in line:
                in_asm = False
                continue
            code = line.split(";")[0].strip()
            if in_asm or not code:
                continue
            if code.startswith("scratch_"):
                problems.append(f"{name}: scratch access: {code}")
            if re.search(r"\bm0\b", code):
                problems.append(f"{name}: compiler-generated use of m0: {code}")
    return problems


def check_no_spills(text: str) -> list:
    """The pre-pass kernels hold a quantization block in registers; a register spill would turn the
    one pass over memory they are built around into several.  Returns the kernels that touch scratch."""
    import re
    problems = []
    for m in re.finditer(r"^(_ZN4sage\w+):.*?^\.Lfunc_end\d+:", text, re.S | re.M):
        if "scratch_" in m.group(0):
            problems.append(f"{m.group(1)}: scratch access (register spill)")
    return problems


def verify_attention_isa(extra=()) -> None:
    """Compiles the kernel sources to assembly and raises RuntimeError if check_attention_asm(),
    check_pv8_asm() or check_no_spills() objects."""
    import tempfile
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    problems = []
    with tempfile.TemporaryDirectory() as tmp:
        for src, check in (("sage_attn.hip", check_attention_asm), ("sage_attn_pv8.hip", check_pv8_asm),
                           ("sage_prepass.hip", check_no_spills), ("sage_prepass_v.hip", check_no_spills)):
            out = os.path.join(tmp, src + ".s")
            cmd = [hipcc(), *flags, *extra, "-S", "--cuda-device-only", "-o", out, os.path.join(CSRC, src)]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc -S failed:\n" + res.stderr)
            problems += check(open(out).read())
    if problems:
        raise RuntimeError("attention kernel ISA check failed:\n  " + "\n  ".join(problems[:20]))


def is_stale() -> bool:
    """True when there is no built library or it was not built from the sources as they are now."""
    return built_hash() != source_hash()


def have_compiler() -> bool:
    import shutil
    cc = hipcc()
    return os.path.exists(cc) if os.path.isabs(cc) else shutil.which(cc) is not None


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
