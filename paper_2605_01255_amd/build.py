"""Compile csrc/ into libacc.so for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libacc.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def build(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, *sources(), "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


def _scalar_regs(token: str) -> set:
    """Scalar registers an assembly operand names: s7, s[4:7], vcc_lo, vcc, m0."""
    import re
    token = token.strip(",")
    m = re.fullmatch(r"s\[(\d+):(\d+)\]", token)
    if m:
        return {f"s{k}" for k in range(int(m.group(1)), int(m.group(2)) + 1)}
    if token == "vcc":
        return {"vcc_lo", "vcc_hi"}
    return {token} if re.fullmatch(r"s\d+|vcc_lo|vcc_hi|m0", token) else set()


def scan_assembly(lines, names) -> dict:
    """{kernel: {"mfma_regions": ..., "stale_transfer_operands": ...}} for the kernels in `names`, from the lines of
    the compiler's assembly output (see kernel_resources)."""
    import re
    found = {}
    name, count, regions, recent, stale = None, 0, {}, [], 0
    for line in lines:
        m = re.match(r"(\w+):\s", line)
        if m and m.group(1) in names:
            name, count, regions, recent, stale = m.group(1), 0, {}, [], 0
            continue
        if name is None:
            continue
        text = line.strip()
        if "; sched_barrier" in text:
            regions[count] = regions.get(count, 0) + 1
            count = 0
        if not text or text[0] in ";." or text.endswith(":"):
            continue
        if "v_mfma" in text:
            count += 1
        if text.startswith("buffer_load") and text.endswith(" lds"):
            used = set().union(*(_scalar_regs(t) for t in text.split()[1:]))
            stale += sum(1 for w in recent[-5:] if w & used)
        w = re.match(r"v_read(?:first)?lane_b32 (\S+),", text)
        recent.append(_scalar_regs(w.group(1)) if w else set())
        if "s_endpgm" in text:
            found[name] = {"mfma_regions": regions, "stale_transfer_operands": stale}
            name = None
    return found


def kernel_resources() -> dict:
    """Compile the device code only and return, per mangled kernel name, {"scratch": bytes per lane, "vgpr_spill": n}
    from the compiler's resource remarks and {"mfma_regions": {k: number of scheduling regions that hold k matrix
    instructions}} from the assembly (a region = the instructions between two scheduling fences; kernels without
    fences have none) and {"stale_transfer_operands": n}.  The slot-program kernels keep whole arrays in registers and
    place one matrix instruction per slot: a build that puts the arrays into scratch memory, or that moves the matrix
    instructions out of their slots, computes the same results much more slowly, so both are worth checking.
    stale_transfer_operands counts global -> LDS transfers (written as inline assembly, so the compiler does not
    know them as memory instructions and inserts no wait states for them) that read a scalar register which one of
    the five instructions before wrote from a vector register (v_readlane / v_readfirstlane: how the compiler
    restores scalar registers it had parked in vector lanes): the hardware needs five wait states there, and without
    them the transfer uses the register's old value."""
    import re
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    out = {}
    with tempfile.TemporaryDirectory() as tmp:
        asm_path = os.path.join(tmp, "dev.s")
        cmd = [hipcc, *flags, "--cuda-device-only", "-S", "-Rpass-analysis=kernel-resource-usage", *sources(),
               "-o", asm_path]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stderr)
        name = None
        for line in res.stderr.splitlines():
            m = re.search(r"remark: Function Name: (\S+)", line)
            if m:
                name = m.group(1)
                out[name] = {}
                continue
            m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", line)
            if m and name:
                out[name]["scratch"] = int(m.group(1))
            m = re.search(r"remark:\s+VGPRs Spill: (\d+)", line)
            if m and name:
                out[name]["vgpr_spill"] = int(m.group(1))
        with open(asm_path) as f:
            for name, found in scan_assembly(f, set(out)).items():
                out[name].update(found)
    return out


def build_c_client(verbose: bool = True) -> str:
    """The plain-C client of the ABI under tests/c_client (host code only: gcc-style compile through hipcc,
    linked against the HIP runtime and libacc.so, found at run time next to this package)."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "c_client", "acc_client.c")
    exe = os.path.join(root, "tests", "c_client", "acc_client")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-x", "c", "-O2", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", src, "-o", exe,
           "-L" + HERE, "-lacc", "-L/opt/rocm/lib", "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2605_01255_amd", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("C client build failed:\n" + res.stdout + res.stderr)
    return exe


if __name__ == "__main__":
    build()
    print("built", LIB)
    build_c_client()
    sys.exit(0)
