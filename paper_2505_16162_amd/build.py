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
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
