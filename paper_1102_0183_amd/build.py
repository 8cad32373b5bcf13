"""Compile the gfx950 kernels and the C ABI into paper_1102_0183_amd/libcnn355.so with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcnn355.so")
SOURCES = ["cnn355_kernels.hip", "cnn355_flow.hip", "cnn355_batch.hip", "cnn355_deform.hip", "cnn355_api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-FP32 instructions are switched off on purpose: some of their forms have given wrong
# results on this hardware, without any error
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-Wno-pass-failed"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "cnn355_dev.h"), os.path.join(CSRC, "cnn355_flowspec.h"),
                        os.path.join(HERE, "..", "include", "cnn355.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    extra = ["-DCNN355_STAMPS"] if os.environ.get("CNN355_STAMPS") else []
    cmd = [HIPCC] + FLAGS + extra + ["-o", tmp] + sources()
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
