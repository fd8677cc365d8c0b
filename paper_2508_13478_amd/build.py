"""Builds libdhq.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdhq.so")
SOURCES = ["dhq_api.hip", "dhq_layerwise.hip", "dhq_fused.hip", "dhq_fused_wide.hip", "dhq_float.hip",
           "dhq_fused_two_sided.hip", "dhq_fused_pair.hip"]
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
                 # the hand-scheduled GEMM loops must unroll completely (their schedule tables fold to
                 # constants only then); the default size limit for "#pragma unroll" is too small for them
                 "-mllvm", "-pragma-unroll-threshold=131072",
                 "-I", os.path.join(ROOT, "include"), "-I", CSRC]

# Kernels that address accumulation registers by number from inline assembly: source file, a
# substring of the kernel's (mangled) name, first register the compiler must leave alone.
FIXED_AGPR_KERNELS = [("dhq_fused_wide.hip", "dhq_fused_wide_kernel", 0),
                      ("dhq_float.hip", "dhq_float_kernel", 128)]
WIDE_FIRST_FIXED_AGPR = 0


def _agprs_named(line: str):
    """Accumulation-register indices an assembly line names (a12, a[12], a[12:15])."""
    import re
    out = []
    for m in re.finditer(r"(?<![\w.])a(\d+)\b", line):
        out.append(int(m.group(1)))
    for m in re.finditer(r"(?<![\w.])a\[(\w+)(?::(\w+))?\]", line):
        out.append(int(m.group(2) or m.group(1), 0))
    return out


def check_fixed_agprs(asm_text: str, kernel_substr: str, first_fixed: int) -> int:
    """Some kernels keep operands in accumulation registers a<first_fixed>..a255 that only their
    inline assembly names.  That is sound only if the compiler's own code never touches those
    registers and if they lie inside the kernel's register allocation; both are checked here on
    the compiler's assembly output for every kernel whose name contains kernel_substr, and a
    violation fails the build.  Returns the number of kernels checked."""
    in_asm = False
    current = None          # function whose body is being read
    descriptor = None       # kernel whose .amdhsa_ block is being read
    alloc = {}              # kernel -> [accum_offset, next_free_vgpr]
    seen = set()
    for ln in asm_text.splitlines():
        t = ln.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        head = t.split(";")[0].strip()
        if head.endswith(":") and not head.startswith(".") and not head.startswith("$"):
            current = head[:-1]
            if kernel_substr in current:
                seen.add(current)
            continue
        if t.startswith(".amdhsa_kernel"):
            descriptor = t.split()[1]
            alloc[descriptor] = [None, None]
        elif t.startswith(".end_amdhsa_kernel"):
            descriptor = None
        elif descriptor and t.startswith(".amdhsa_accum_offset"):
            alloc[descriptor][0] = int(t.split()[1])
        elif descriptor and t.startswith(".amdhsa_next_free_vgpr"):
            alloc[descriptor][1] = int(t.split()[1])
        if current is None or kernel_substr not in current or in_asm or not t or t[0] in ";.":
            continue
        bad = [r for r in _agprs_named(head) if r >= first_fixed]
        if bad:
            raise RuntimeError(f"{current}: compiler-generated code touches a fixed accumulation register: {t}")
    if not seen:
        raise RuntimeError(f"no kernel named *{kernel_substr}* in the assembly output")
    for k in seen:
        off, nxt = alloc.get(k, [None, None])
        if off is None or nxt is None:
            raise RuntimeError(f"{k}: register allocation not found in the assembly output")
        if nxt - off < 256:
            raise RuntimeError(f"{k} is allocated {nxt - off} accumulation registers, 256 are needed")
    return len(seen)


def check_wide_register_map(asm_text: str) -> None:
    check_fixed_agprs(asm_text, "dhq_fused_wide_kernel", WIDE_FIRST_FIXED_AGPR)


def asm_cmd(source: str, out_path: str):
    return [_hipcc()] + CODEGEN_FLAGS + ["-S", "--cuda-device-only", "-o", out_path, os.path.join(CSRC, source)]


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    import tempfile
    cmd = [_hipcc()] + CODEGEN_FLAGS + ["-fPIC", "-shared", "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if os.path.exists(LIB):
        os.remove(LIB)  # a failed build must not leave an older library behind to be loaded in its place
    if verbose:
        print(" ".join(cmd), flush=True)
    with tempfile.TemporaryDirectory() as td:
        # the same sources once more to assembly, in parallel with the real build, for the register check
        checks = []
        for src, name, first in FIXED_AGPR_KERNELS:
            asm_path = os.path.join(td, src + ".s")
            checks.append((subprocess.Popen(asm_cmd(src, asm_path), stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True), asm_path, name, first))
        r = subprocess.run(cmd, capture_output=True, text=True)
        for proc, asm_path, name, first in checks:
            out_text, _ = proc.communicate()
            if r.returncode != 0:
                continue
            try:
                if proc.returncode != 0:
                    raise RuntimeError("hipcc -S failed:\n" + out_text)
                with open(asm_path) as f:
                    check_fixed_agprs(f.read(), name, first)
            except RuntimeError:
                if os.path.exists(LIB):
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
