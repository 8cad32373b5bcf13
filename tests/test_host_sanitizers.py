"""AddressSanitizer + UndefinedBehaviorSanitizer runs of everything that executes on the host (no GPU): the CPU
oracle, and the library's parser, Eq. 1 shapes, workspace sizing, stage planner and resident-mode planner.  Each is
compiled into a small driver of its own (tests/sanitize/) with -fsanitize=address,undefined on the host pass and
run as a separate program, so that neither this interpreter nor its preloaded libraries are involved; a report of
either sanitizer ends the driver with a non-zero status."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
OUT = os.path.join(ROOT, "paper_1102_0183_amd", "_build", "san")


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    src = os.path.join(HERE, "sanitize", "oracle_driver.cpp")
    exe = os.path.join(OUT, "oracle_san")
    dep = os.path.join(ROOT, "oracle", "cnn_oracle.cpp")
    if not os.path.exists(exe) or os.path.getmtime(exe) < max(os.path.getmtime(src), os.path.getmtime(dep)):
        subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe, src], check=True)
    assert "oracle sanitizer run: clean" in _run(exe)


def test_host_planner_is_clean_under_address_and_undefined_behaviour_sanitizers():
    from paper_1102_0183_amd import build
    exe = build.build_host_sanitizer_driver(os.path.join(HERE, "sanitize", "plan_driver.cpp"))
    assert "host planner sanitizer run: clean" in _run(exe)
