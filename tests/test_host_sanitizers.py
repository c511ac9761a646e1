"""The host part of the library (sampler, spectral test, mask object, clustering and pairing of the tile
rows, packed layouts, transposes) under AddressSanitizer and UndefinedBehaviorSanitizer: the library is
built once more with its host code instrumented (device code as usual) and the host tests of
tests/test_abi_host.py run against that build in a child process, with the sanitizer runtime preloaded.
Any report of either sanitizer ends the child with an error."""
import glob
import os
import subprocess
import sys

from paper_2006_13486_amd import build as lib_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sanitized_library():
    lib = os.path.join(os.path.dirname(lib_build.LIB), "librbgp_asan.so")
    sources = glob.glob(os.path.join(lib_build.CSRC, "*.hip")) + glob.glob(os.path.join(lib_build.CSRC, "*.cpp")) + \
        glob.glob(os.path.join(lib_build.CSRC, "*.h")) + [os.path.join(ROOT, "include", "rbgp.h")]
    if not os.path.exists(lib) or os.path.getmtime(lib) < max(os.path.getmtime(f) for f in sources):
        lib_build.build_sanitized()
    return lib


def test_host_tests_pass_under_address_and_undefined_behaviour_sanitizers():
    env = dict(os.environ)
    runtime = lib_build.sanitizer_runtime()
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["RBGP_LIB"] = _sanitized_library()
    env["RBGP_NO_TORCH"] = "1"              # (torch is not needed by the host tests and is not instrumented)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_host.py"), "-x", "-q", "-s",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=900)
    tail = run.stdout[-3000:]
    assert "runtime error:" not in run.stdout and "ERROR: AddressSanitizer" not in run.stdout, tail
    assert run.returncode == 0, tail
    assert " passed" in run.stdout, tail
