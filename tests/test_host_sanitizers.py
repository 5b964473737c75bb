"""The library's host side under sanitizers: router bookkeeping, CPU scan, worker pool,
dispatcher threads, partitioning model.  tests/sanitize/host_driver.cpp drives them
through the C ABI on device-less indexes; it is built twice with the library's sources
(hipcc, host code instrumented, device code as always) - AddressSanitizer +
UndefinedBehaviorSanitizer, and ThreadSanitizer - and each build must run clean.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_2504_08930_amd.build import CSRC, FLAGS, HIPCC, SOURCES  # noqa: E402

DRIVER = os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp")


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    assert p.returncode == 0, f"build failed: {' '.join(cmd)}\n{out[-4000:]}"


@pytest.fixture(scope="module")
def kernel_objects(tmp_path_factory):
    """The kernel files, whose host side is launch code that a device-less run never
    reaches: compiled once, uninstrumented, and linked into both sanitizer builds."""
    tmp = str(tmp_path_factory.mktemp("kernels"))
    objs, procs = [], []
    for src in SOURCES:
        if src.endswith(".hip"):
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            cmd = [HIPCC, *[f for f in FLAGS if f != "-O3"], "-O1", "-x", "hip", "-c",
                   os.path.join(CSRC, src), "-o", obj]
            procs.append(subprocess.Popen(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL))
            objs.append(obj)
    for p in procs:
        assert p.wait() == 0, "kernel compile failed"
    return objs


def _build(tmp, tag, sanitizers, kernel_objs):
    """Host sources and the driver on hipcc lines where every -fsanitize= goes to the
    host pass only."""
    san = []
    for s in sanitizers:
        san += ["-Xarch_host", f"-fsanitize={s}"]
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fno-omit-frame-pointer"]
    exe = os.path.join(tmp, f"host_driver_{tag}")
    host = [os.path.join(CSRC, s) for s in SOURCES if s.endswith(".cpp")]
    _run([HIPCC, *flags, *san, "-x", "hip", DRIVER, *host, "-x", "none", *kernel_objs,
          "-o", exe, "-lpthread"])
    return exe


@pytest.mark.parametrize("tag,sanitizers,env", [
    ("asan_ubsan", ("address", "undefined"),
     {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
      "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"}),
    ("tsan", ("thread",), {"TSAN_OPTIONS": "halt_on_error=1:second_deadlock_stack=1"}),
])
def test_host_side_runs_clean_under(tmp_path, kernel_objects, tag, sanitizers, env):
    exe = _build(str(tmp_path), tag, sanitizers, kernel_objects)
    for threads in ("1", "4"):
        run_env = dict(os.environ, IVF_CPU_THREADS=threads, **env)
        p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                           env=run_env, timeout=600)
        assert p.returncode == 0 and "host driver ok" in p.stdout, \
            f"{tag} with {threads} worker threads:\n{p.stdout[-6000:]}"
        for word in ("ERROR: AddressSanitizer", "WARNING: ThreadSanitizer", "runtime error:",
                     "ERROR: LeakSanitizer"):
            assert word not in p.stdout, f"{tag}:\n{p.stdout[-6000:]}"
