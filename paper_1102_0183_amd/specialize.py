"""Compile the resident kernel for one network and load it into a handle.

The resident mode runs the benchmark networks in kernels compiled for them (every size a literal) and any
other network in a kernel that reads its plan at run time, which costs about 1.5 x the time per image.
specialize(net) closes that gap for any network: it asks the handle for a description of its network
(cnn_resident_spec_source), compiles csrc/cnn355_flow.hip against it with hipcc (device code only, the
library's own flags, some 10 - 40 s), keeps the code object under _spec/ next to this file under a name made of
a hash of the description and of the sources, and loads it (cnn_load_resident_code), which checks the plan
inside against the handle's own.  Compiling needs no GPU: code_object_for(text) can run ahead of time, e.g. in a
build step, and the files travel with the package.

    net = binding.Cnn(arch); ...; net.set_mode(binding.MODE_RESIDENT)
    specialize.specialize(net)          # from here on train_many runs the kernel compiled for this network
"""
import hashlib
import os
import subprocess

from . import build as _build

HERE = os.path.dirname(os.path.abspath(__file__))
SPEC_DIR = os.path.join(HERE, "_spec")
SOURCE = os.path.join(_build.CSRC, "cnn355_flow.hip")
# the library's flags, without the host-side ones
FLAGS = [f for f in _build.FLAGS if f not in ("-fPIC", "-Wall", "-Wno-unused-function", "-Wno-pass-failed")]


def _digest(text):
    h = hashlib.sha256(text.encode())
    for path in [SOURCE] + _build.HEADERS[:2]:
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()[:20]


def code_object_for(text, force=False, verbose=False):
    """Path of the code object for the network described by `text` (cnn_resident_spec_source), compiled now
    unless it is already there."""
    os.makedirs(SPEC_DIR, exist_ok=True)
    tag = _digest(text)
    header = os.path.join(SPEC_DIR, "spec_%s.h" % tag)
    out = os.path.join(SPEC_DIR, "spec_%s.hsaco" % tag)
    if os.path.exists(out) and not force:
        return out
    with open(header, "w") as f:
        f.write(text)
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [_build.HIPCC] + FLAGS + ["--cuda-device-only", '-DCNN355_SPECIAL_HEADER="%s"' % header, "-o", tmp, SOURCE]
    if verbose:
        print(" ".join(cmd))
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    msg = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed on the resident kernel for this network:\n" + msg)
    os.replace(tmp, out)
    return out


# Networks the build step compiles code objects for, so that they are there where no compiler should run (the
# GPU tests load them): (architecture, fan_in), fan_in > 0 meaning that output map j of every convolutional layer
# above the first reads the input maps j .. j + fan_in - 1 (mod M_i), 0 fully connected tables, -d: M_i / d of them.
EXAMPLES = {
    "narrow": ("1x29x29-24C4-MP2-48C5-MP3-150N-10N", 0),       # the benchmark net's shape with other map counts
    "benchmark": ("1x29x29-20C4-MP2-40C5-MP3-150N-10N", 0),    # the library also holds a compiled-in kernel for it
    "sparse": ("1x29x29-20C4-MP2-40C5-MP3-150N-10N", 8),
    "streamed": ("3x32x32-80C5-MP2-110C5-MP2-80N-10N", 0),     # does not fit with every layer's inputs in LDS
    # Sec. 4.3's CIFAR10 architectures with 100 and 200 maps a layer (their second hidden layer is held by columns)
    "cifar100": ("3x32x32-100C3-MP3-100C3-MP2-100C3-MP2-300N-100N-10N", 0),
    "cifar200": ("3x32x32-200C3-MP3-200C3-MP2-200C3-MP2-300N-100N-10N", 0),
    # Sec. 4.1's deepest net (Table 1: 20 to 120 maps in six convolutional layers, 150 hidden neurons), kernel sizes
    # that end at 1 x 1 maps (the paper does not give them), half of the connections above the first layer
    "mnist-deep": ("1x29x29-20C4-MP2-40C2-60C3-80C3-MP2-100C2-120C3-150N-10N", -2),
}


def prune():
    """Delete the code objects of sources that have changed since (their names no longer match what they hold)."""
    if not os.path.isdir(SPEC_DIR):
        return
    for name in sorted(os.listdir(SPEC_DIR)):
        if name.startswith("spec_") and name.endswith(".h"):
            tag = name[5:-2]
            with open(os.path.join(SPEC_DIR, name)) as f:
                stale = _digest(f.read()) != tag
            if stale:
                for ext in (".h", ".hsaco"):
                    try:
                        os.remove(os.path.join(SPEC_DIR, "spec_" + tag + ext))
                    except FileNotFoundError:
                        pass


def build_examples(force=True):
    """Compile the code objects of EXAMPLES side by side.  Returns their paths by name."""
    from concurrent.futures import ThreadPoolExecutor

    from . import binding
    prune()
    texts = {k: binding.resident_spec_source_for(a, f) for k, (a, f) in EXAMPLES.items()}
    with ThreadPoolExecutor(max_workers=4) as ex:
        paths = list(ex.map(lambda k: code_object_for(texts[k], force=force), sorted(texts)))
    return dict(zip(sorted(texts), paths))


def built_code_object(net):
    """Path of the code object for the network of `net` if an earlier call or the build step compiled it, else None."""
    out = os.path.join(SPEC_DIR, "spec_%s.hsaco" % _digest(net.resident_spec_source()))
    return out if os.path.exists(out) else None


def specialize(net, force=False, verbose=False):
    """Compile (or find) the resident kernel for the network of `net` as it stands and load it.  Returns the
    code object's path."""
    path = code_object_for(net.resident_spec_source(), force=force, verbose=verbose)
    net.load_resident_code(path)
    return path
