"""Builds libinfinipot.so (gfx950) in-tree with hipcc.  `python -m paper_2410_01518_amd.build`."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libinfinipot.so")
SOURCES = ["infinipot_api.hip", "ccd_score_valu.hip", "ccd_score_mfma.hip", "ccd_score_unit.hip", "ccd_select.hip", "ccd_compact.hip",
           "ccd_nuc.hip"]
# ccd_score_unit.hip keeps its query fragments at fixed places in the accumulation registers (named in its inline
# assembly): the compiler must put nothing of its own there, so matrix-instruction results go to vector registers and
# the generated code is checked for accumulation registers outside the assembly statements.
SOURCE_FLAGS = {"ccd_score_unit.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}
ACC_REGISTERS_RESERVED = {"ccd_score_unit.hip"}
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


_ACC_REG = re.compile(r"(?<![A-Za-z0-9_.$])a(\[\d+(:\d+)?\]|\d+)(?![A-Za-z0-9_])")


def check_acc_registers_untouched(asm_path: str) -> None:
    """Fails if compiler-generated code (outside inline assembly) names an accumulation register, or spills."""
    in_asm = False
    bad = []
    with open(asm_path) as f:
        for n, line in enumerate(f, 1):
            if ";;#ASMSTART" in line:
                in_asm = True
            elif ";;#ASMEND" in line:
                in_asm = False
            elif not in_asm:
                code = line.split(";")[0]
                if code.lstrip().startswith("."):
                    continue
                if _ACC_REG.search(code):
                    bad.append(f"{n}: {line.rstrip()}")
    if bad:
        raise RuntimeError(f"{asm_path}: the compiler uses accumulation registers that the kernel reserves:\n" + "\n".join(bad[:10]))


_VGPR_RANGE = re.compile(r"v\[(\d+):(\d+)\]")
_VGPR_ONE = re.compile(r"v(\d+)")


def _vgprs(token: str) -> set:
    token = token.strip()
    m = _VGPR_RANGE.fullmatch(token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = _VGPR_ONE.fullmatch(token)
    return {int(m.group(1))} if m else set()


def check_matrix_operand_distance(asm_path: str) -> None:
    """A matrix instruction must not read, as its first or second operand, a vector register that an ALU instruction
    wrote in the two issue slots before it.  The compiler keeps that distance for matrix instructions it generates; the
    ones in ccd_score_unit.hip are inline assembly, which it schedules around without knowing what they are.  Checked on
    straight-line code (history is dropped at every label)."""
    bad, hist = [], []
    with open(asm_path) as f:
        for n, line in enumerate(f, 1):
            text = line.split(";")[0].strip()
            if not text or text.startswith("."):
                continue
            if text.endswith(":"):
                hist = []
                continue
            parts = text.split(None, 1)
            op = parts[0]
            args = [a.strip() for a in parts[1].split(",")] if len(parts) > 1 else []
            if op.startswith("v_mfma"):
                src = set()
                for a in args[1:3]:
                    src |= _vgprs(a)
                for ln, tx, wr in hist[-2:]:
                    if wr & src:
                        bad.append(f"{n}: {text}   <- {ln}: {tx}")
                hist.append((n, text, set()))
            elif op == "s_nop":
                hist.extend([(n, text, set())] * (int(args[0], 0) + 1))
            else:
                wr = _vgprs(args[0]) if (op.startswith("v_") and not op.startswith("v_cmp") and args) else set()
                hist.append((n, text, wr))
            hist = hist[-4:]
    if bad:
        raise RuntimeError(f"{asm_path}: an ALU write directly before the matrix instruction that reads it:\n" + "\n".join(bad[:10]))


def build_library(verbose: bool = True, extra_flags=()) -> str:
    """Compiles every kernel source and links the shared library; returns its path."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        flags = [*FLAGS, *SOURCE_FLAGS.get(src, []), *extra_flags]
        if src in ACC_REGISTERS_RESERVED:
            asm = os.path.join(objdir, src.replace(".hip", ".s"))
            r = subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", asm],
                               capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
            check_acc_registers_untouched(asm)
            check_matrix_operand_distance(asm)
        cmd = [hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
            if lines:
                print("\n".join(lines), file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + ".tmp"
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}")
    build_c_client(verbose)
    return LIB


C_CLIENT_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_client", "ccd_client.c")
C_CLIENT = os.path.join(HERE, "ccd_client")


def build_c_client(verbose: bool = True) -> str:
    """The plain C client of the ABI (gcc, C99): the header and the library must be usable without C++ or Python."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(os.path.dirname(HERE), "include"),
           "-I", os.path.join(rocm, "include"), C_CLIENT_SRC, "-o", C_CLIENT, "-L", HERE, "-linfinipot",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath,$ORIGIN", f"-Wl,-rpath,{os.path.join(rocm, 'lib')}"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gcc failed on the C client:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {C_CLIENT}")
    return C_CLIENT


if __name__ == "__main__":
    build_library()
