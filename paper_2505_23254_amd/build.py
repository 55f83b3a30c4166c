"""Compile the HIP sources in csrc/ for gfx950 into paper_2505_23254_amd/libma_step.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libma_step.so")
SOURCES = ["ma_api.hip", "ma_norm.hip", "ma_adamw.hip", "ma_accum.hip", "ma_probe.hip", "ma_arena.hip", "ma_pool.cpp"]
HEADERS = ["ma_device.h", "ma_internal.h", os.path.join("..", "..", "include", "ma.h")]

# -ffp-contract=off: the update kernel states every fused multiply-add itself.
# The packed-fp32 target feature is switched off for all device code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def up_to_date() -> bool:
    if not os.path.exists(OUT):
        return False
    t = os.path.getmtime(OUT)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, extra_flags=(), out: str = OUT) -> str:
    if not force and out == OUT and up_to_date():
        return out
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *FLAGS, *extra_flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


EXAMPLE_SRC = os.path.join(HERE, "..", "examples", "step_from_c.c")
EXAMPLE_OUT = os.path.join(HERE, "step_from_c")


def build_example(out: str = EXAMPLE_OUT) -> str:
    """The plain-C99 example program (examples/step_from_c.c), linked against the library."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(HERE, "..", "include"), "-I", os.path.join(rocm, "include"), EXAMPLE_SRC,
           "-L", HERE, "-lma_step", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", out]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
    print(build_example())
