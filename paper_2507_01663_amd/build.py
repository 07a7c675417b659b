"""Compile the HIP sources into paper_2507_01663_amd/librollout_attn.so for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librollout_attn.so")
SOURCES = ["ra_kernels.hip", "ra_prefill.hip", "ra_api.cpp", "ra_balance.cpp"]
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-inline-asm", "-Wno-int-to-pointer-cast", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]
# The decode kernels keep their few MFMA accumulators in ordinary vector registers; the prefill kernel has more
# accumulators than those hold and leaves them in the accumulation registers, where the matrix cores reach them directly.
EXTRA = {"ra_kernels.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"], "ra_prefill.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def flags_for(source: str):
    """Compile flags of one source file (no output, no link)."""
    return COMMON + EXTRA.get(source, [])


FLAGS = flags_for("ra_kernels.hip")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        cmd = [hipcc] + flags_for(src) + ["-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, obj, subprocess.Popen(cmd)))
    for cmd, obj, p in procs:
        if p.wait() != 0:
            raise subprocess.CalledProcessError(p.returncode, cmd)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [obj for _, obj, _ in procs]
    if verbose:
        print(" ".join(link))
    subprocess.run(link, check=True)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "rollout_attn.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build(verbose=True))
