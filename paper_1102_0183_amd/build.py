"""Compile the gfx950 kernels and the C ABI into paper_1102_0183_amd/libcnn355.so with hipcc.

Every source is compiled to an object of its own (side by side, in _build/ next to this file), then the
objects are linked.  build(force=True) compiles everything; build(force=False) only what is older than
its source or one of the headers."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcnn355.so")
SOURCES = ["cnn355_kernels.hip", "cnn355_flow.hip", "cnn355_batch.hip", "cnn355_deform.hip", "cnn355_api.hip"]
HEADERS = [os.path.join(CSRC, "cnn355_dev.h"), os.path.join(CSRC, "cnn355_flowspec.h"),
           os.path.join(HERE, "..", "include", "cnn355.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-FP32 instructions are switched off on purpose: some of their forms have given wrong
# results on this hardware, without any error
# (the resident kernel takes its plan as a by-value kernel argument; the optimiser turns the copy of it that the
# language semantics ask for back into scalar loads of the argument only if it can look at every use, and gives
# up beyond 300 of them: the plan has more, and would otherwise be copied to scratch memory and read from there)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-mllvm", "-instcombine-max-copied-from-constant-users=100000",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-Wno-pass-failed"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def _obj(src):
    return os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")


def _older(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def stale() -> bool:
    return _older(LIB, sources() + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    extra = ["-DCNN355_STAMPS"] if os.environ.get("CNN355_STAMPS") else []
    jobs = []
    for src in sources():
        if force or _older(_obj(src), [src] + HEADERS):
            cmd = [HIPCC] + FLAGS + extra + ["-c", "-o", _obj(src), src]
            if verbose:
                print(" ".join(cmd))
            jobs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = []
    for src, p in jobs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip():
            print(out)
        if p.returncode != 0:
            failed.append(src)
    if failed:
        raise RuntimeError("hipcc failed on " + ", ".join(failed))
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", tmp] + [_obj(s) for s in sources()]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-g"]


def build_host_sanitizer_driver(driver_cpp: str, force: bool = False) -> str:
    """An executable of `driver_cpp` plus the library's sources with AddressSanitizer and
    UndefinedBehaviorSanitizer on the HOST pass (the device pass is compiled as usual and never runs here):
    for checking parser, planners and workspace sizing without a GPU.  Objects live in _build/san/."""
    out_dir = os.path.join(OBJ, "san")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "plan_san")
    srcs = sources() + [driver_cpp]
    objs = [os.path.join(out_dir, os.path.basename(x).rsplit(".", 1)[0] + ".o") for x in srcs]
    jobs = []
    for src, obj in zip(srcs, objs):
        if force or _older(obj, [src] + HEADERS):
            cmd = [HIPCC] + [f for f in FLAGS if f != "-O3"] + ["-O1", "-x", "hip"] + SAN_FLAGS + ["-c", "-o", obj, src]
            jobs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in jobs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("hipcc (host sanitizers) failed on %s:\n%s" % (src, out))
    if jobs or not os.path.exists(exe):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-rdc", "-fsanitize=address", "-fsanitize=undefined",
                        "-o", exe] + objs, check=True)
    return exe


if __name__ == "__main__":
    import sys
    print(build(force="--all" in sys.argv, verbose=True))
