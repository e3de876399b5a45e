"""Compile the HIP sources of the library for gfx950 into paper_2505_16162_amd/libknnssd.so."""
import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libknnssd.so")
SOURCES = ["knnssd.hip"]
NO_SPILL_KERNELS = ["gemv_kernel", "gemm_mfma_kernel"]     # mangled-name fragments of the kernels that must not spill


def build_library(verbose: bool = False) -> str:
    """Always compiles (hipcc cross-compiles without a GPU present)."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(HERE, "..", "include"),
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    # The draft GEMV and the verification GEMM issue streaming loads the compiler does not track (hand-placed waits); a register of such a
    # load must never be spilled or copied while the load is in flight. The resource remarks of the same compile
    # tell whether any kernel spills vector registers: the build fails if one of the kernels named below does.
    cmd += ["-Rpass-analysis=kernel-resource-usage"]
    if verbose:
        print(" ".join(cmd))
    proc = subprocess.run(cmd, check=False, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    remarks = [ln for ln in proc.stderr.splitlines() if "remark:" in ln]
    other = [ln for ln in proc.stderr.splitlines() if "remark:" not in ln and "kernel-resource-usage" not in ln]
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stderr[-4000:])
    if verbose and other:
        print("\n".join(other))
    current = None
    for ln in remarks:
        m = re.search(r"Function Name: (\S+)", ln)
        if m:
            current = m.group(1)
        m = re.search(r"VGPRs Spill: (\d+)", ln)
        if m and current and any(k in current for k in NO_SPILL_KERNELS) and int(m.group(1)) > 0:
            os.remove(LIB)
            raise RuntimeError(f"{current} spills {m.group(1)} vector registers; its hand-placed loads forbid that")
    check_hand_placed_loads(verbose)
    return LIB


def check_hand_placed_loads(verbose: bool = False) -> None:
    """Second compile to assembly text, then the static checks of isa_check.py: the library is deleted and the
    build fails if the GEMV has any instruction that can touch a register with a hand-placed load in flight, or
    if a variant of the verification GEMM copies or spills a register of its weight stream."""
    import tempfile
    from . import isa_check
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "knnssd.s")
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
               "-I", os.path.join(HERE, "..", "include"), "-o", asm] + [os.path.join(CSRC, s) for s in SOURCES]
        proc = subprocess.run(cmd, check=False, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
        if proc.returncode != 0:
            os.remove(LIB)
            raise RuntimeError("hipcc -S failed:\n" + proc.stderr[-4000:])
        text = open(asm).read()
    problems = []
    gemv = isa_check.kernel_bodies(text, "gemv_kernel")
    gemm = isa_check.kernel_bodies(text, "gemm_mfma_kernel")
    if not gemv or not gemm:
        problems.append("kernels not found in the assembly text")
    for name, body in gemv:
        for n, t, r, why in isa_check.inflight_flags(body)[:5]:
            problems.append(f"{name}: line {n}: {t}: v{r}: {why}")
    for name, body in gemv + gemm:
        for n, t in isa_check.weight_register_copies(body)[:5]:
            problems.append(f"{name}: line {n}: {t}: reads a register of the weight stream")
    if verbose:
        print(f"isa_check: {len(gemv)} GEMV and {len(gemm)} GEMM kernel bodies, {len(problems)} problems")
    if problems:
        os.remove(LIB)
        raise RuntimeError("hand-placed loads: the compiled code is not safe:\n" + "\n".join(problems))


if __name__ == "__main__":
    print(build_library(verbose=True))
