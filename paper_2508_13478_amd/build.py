"""Builds libdhq.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdhq.so")
SOURCES = ["dhq_api.hip", "dhq_layerwise.hip", "dhq_fused.hip", "dhq_fused_wide.hip"]
HEADERS = ["dhq_internal.h", "dhq_device.h", "dhq_fused_common.h"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "dhq.h")]
    return any(os.path.getmtime(d) > t for d in deps)


# flags that shape the generated device code
CODEGEN_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17",
                 # packed fp32 instructions are kept out of the generated code
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                 # MFMA accumulators in ordinary vector registers even in kernels that also park values
                 # in accumulation registers: the epilogue then reads them without a register move
                 "-mllvm", "-amdgpu-mfma-vgpr-form",
                 "-I", os.path.join(ROOT, "include"), "-I", CSRC]

# dhq_fused_wide.hip addresses the accumulation registers from this one up by number
WIDE_FIRST_FIXED_AGPR = 160


def _agprs_named(line: str):
    """Accumulation-register indices an assembly line names (a12, a[12], a[12:15])."""
    import re
    out = []
    for m in re.finditer(r"(?<![\w.])a(\d+)\b", line):
        out.append(int(m.group(1)))
    for m in re.finditer(r"(?<![\w.])a\[(\w+)(?::(\w+))?\]", line):
        out.append(int(m.group(2) or m.group(1), 0))
    return out


def check_wide_register_map(asm_text: str) -> None:
    """The width-512 kernel keeps its codes and its copy staging in accumulation registers
    a160..a255 that only its inline assembly names.  That is sound only if the compiler's own
    code never touches them and if they lie inside the kernel's register allocation; both are
    checked here on the compiler's assembly output, and a violation fails the build."""
    in_asm = False
    kernel = False
    accum_offset = next_free = None
    for ln in asm_text.splitlines():
        t = ln.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        head = t.split(";")[0].strip()
        if "dhq_fused_wide_kernel" in head and head.endswith(":") and not head.startswith("."):
            kernel = True
        if t.startswith(".amdhsa_accum_offset"):
            accum_offset = int(t.split()[1])
        if t.startswith(".amdhsa_next_free_vgpr"):
            next_free = int(t.split()[1])
        if not kernel or in_asm or not t or t[0] in ";.":
            continue
        code = t.split(";")[0]
        bad = [r for r in _agprs_named(code) if r >= WIDE_FIRST_FIXED_AGPR]
        if bad:
            raise RuntimeError(f"compiler-generated code touches a fixed accumulation register: {t}")
    if not kernel or accum_offset is None or next_free is None:
        raise RuntimeError("dhq_fused_wide_kernel not found in the assembly output")
    if next_free - accum_offset < 256:
        raise RuntimeError(f"the kernel is allocated {next_free - accum_offset} accumulation registers, 256 are needed")


def wide_asm_cmd(out_path: str):
    return [_hipcc()] + CODEGEN_FLAGS + ["-S", "--cuda-device-only", "-o", out_path,
                                         os.path.join(CSRC, "dhq_fused_wide.hip")]


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    import tempfile
    cmd = [_hipcc()] + CODEGEN_FLAGS + ["-fPIC", "-shared", "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    with tempfile.TemporaryDirectory() as td:
        asm_path = os.path.join(td, "dhq_fused_wide.s")
        chk = subprocess.Popen(wide_asm_cmd(asm_path), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        chk_out, _ = chk.communicate()
        if r.returncode == 0:
            if chk.returncode != 0:
                os.remove(LIB)
                raise RuntimeError("hipcc -S failed:\n" + chk_out)
            try:
                with open(asm_path) as f:
                    check_wide_register_map(f.read())
            except RuntimeError:
                os.remove(LIB)
                raise
    msgs = [ln for ln in (r.stdout + r.stderr).splitlines() if "not a recognized feature" not in ln]
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(msgs))
    if verbose and msgs:
        print("\n".join(msgs))
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
