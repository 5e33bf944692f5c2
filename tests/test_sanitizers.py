"""The oracle and the host side of libgg under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

* oracle/gg_oracle.c is built with gcc's sanitizers and the oracle's pins (four test files) run against that build:
  an out-of-bounds access, a signed overflow, a shift past the width or a misaligned access in the checker itself
  would end the run.
* libgg's HOST code (argument validation, geometry, workspace layout, host helpers) is built with the sanitizers in
  the host pass only -- the device code is compiled as always and never runs here -- and the boundary tests of
  test_abi.py (every host-side rejection path, the host helpers) run against that build.

Each run is a process of its own with the sanitizer runtime preloaded (the interpreter is not instrumented)."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

RUN = """
import sys
sys.path[:0] = [{root!r}, {tests!r}]
{redirect}
import pytest
sys.exit(pytest.main({files!r} + ["-q", "-x", "-p", "no:cacheprovider"]))
"""


def _run_with_runtime(runtime, redirect, files):
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # leaks of the interpreter are not the subject; everything else ends the process with a report
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:exitcode=97:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    script = RUN.format(root=ROOT, tests=HERE, redirect=redirect, files=[os.path.join(HERE, f) for f in files])
    return subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, timeout=900, env=env)


def _runtime_of(compiler_cmd, name):
    path = subprocess.run(compiler_cmd + ["-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_hold_under_asan_and_ubsan(tmp_path):
    runtime = _runtime_of(["gcc"], "libasan.so")
    if runtime is None:
        pytest.skip("gcc's sanitizer runtime is not installed")
    so = str(tmp_path / "libgg_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", so,
                    os.path.join(ROOT, "oracle", "gg_oracle.c"), "-lm"], check=True)
    redirect = "import oracle\noracle._lib = oracle.load(%r)" % so
    done = _run_with_runtime(runtime, redirect, ["test_oracle_stats.py", "test_oracle_rate.py",
                                                 "test_oracle_penalty_sampler.py", "test_oracle_next.py"])
    assert done.returncode == 0, (done.returncode, done.stdout[-3000:], done.stderr[-3000:])
    assert " passed" in done.stdout and "failed" not in done.stdout


def test_libgg_host_code_under_asan_and_ubsan(tmp_path):
    clang_rt = None
    for line in subprocess.run([HIPCC, "--version"], capture_output=True, text=True).stdout.splitlines():
        if line.startswith("InstalledDir:"):
            clang = os.path.join(line.split(":", 1)[1].strip(), "clang++")
            clang_rt = _runtime_of([clang], "libclang_rt.asan-x86_64.so")
    if clang_rt is None:
        pytest.skip("the HIP compiler's sanitizer runtime is not installed")
    sys.path.insert(0, os.path.join(ROOT, "paper_2506_00486_amd", "csrc"))
    try:
        import gen_solve_curve
    finally:
        sys.path.pop(0)
    gen_solve_curve.generate()
    so = str(tmp_path / "libgg_host_san.so")
    csrc = os.path.join(ROOT, "paper_2506_00486_amd", "csrc")
    # sanitizers in the host pass only; the device pass is not optimised (its code is never run here)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-Xarch_device", "-O0", "-Xarch_host", "-O1", "-g", "-std=c++17", "-fPIC",
                    "-shared", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan",
                    "-I", os.path.join(ROOT, "include"), "-o", so,
                    os.path.join(csrc, "gg_kernels.hip"), os.path.join(csrc, "gg_train.hip")],
                   check=True, capture_output=True)
    redirect = "import paper_2506_00486_amd.binding as b\nb.lib_path = lambda: %r" % so
    done = _run_with_runtime(clang_rt, redirect, ["test_abi.py"])
    assert done.returncode == 0, (done.returncode, done.stdout[-3000:], done.stderr[-3000:])
    assert " passed" in done.stdout and "failed" not in done.stdout
