"""Compile the HIP sources into paper_2401_16677_amd/libt3.so for gfx950 (in-tree)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libt3.so")
SOURCES = ["t3_api.hip"]          # t3_kernels.hip is included by t3_api.hip
DEPS = ["t3_api.hip", "t3_kernels.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-pragma-unroll-threshold=1000000",
    "-Wall", "-Wno-unused-command-line-argument",
]


def up_to_date():
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, d) for d in DEPS] + [os.path.join(ROOT, "include", "t3.h")]
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force=True, extra_flags=()):
    if not force and up_to_date():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    subprocess.run(cmd, check=True)
    return LIB


C_CLIENT_SRC = os.path.join(ROOT, "tests", "c_abi_client.c")
C_CLIENT = os.path.join(ROOT, "tests", "c_abi_client")


def build_c_client(force=True):
    """Compile tests/c_abi_client.c, a plain C11 user of include/t3.h, with gcc against the
    built library and the HIP runtime (it is run by the GPU tests)."""
    if not force and os.path.exists(C_CLIENT) and \
            os.path.getmtime(C_CLIENT) >= max(os.path.getmtime(C_CLIENT_SRC), os.path.getmtime(LIB)):
        return C_CLIENT
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
           C_CLIENT_SRC, "-o", C_CLIENT, "-L", HERE, "-l:libt3.so",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2401_16677_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.run(cmd, check=True)
    return C_CLIENT


if __name__ == "__main__":
    print(build())
    print(build_c_client())
