"""The host side of the library (split planner, argument validation, offset helpers, the left-inverse solve, the path
model) under the address and undefined-behaviour sanitizers: the CPU tests of tests/test_host_abi.py are run once more,
in a child interpreter, against a build of the library whose host code is instrumented (GPU code objects as usual; no
GPU call is made by these tests)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_abi_cases_under_address_and_ub_sanitizers():
    sys.path.insert(0, ROOT)
    from paper_2605_15250_amd import build as Bld
    lib, runtime = Bld.build_hostcheck()
    env = dict(os.environ)
    env["GQLA_LIB_PATH"] = lib
    # the interpreter itself is not instrumented: the sanitizer runtime has to be loaded ahead of the library.  Whatever
    # is already preloaded stays in the list, behind it.
    env["LD_PRELOAD"] = runtime + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    # leaks: the interpreter's own allocations would drown the report; link order: other preloaded libraries may come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=23"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=24"
    # the child really maps the instrumented build and the sanitizer runtime
    probe = subprocess.run([sys.executable, "-c",
                            "from paper_2605_15250_amd import binding as B; B.lib(); print(open('/proc/self/maps').read())"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert probe.returncode == 0, probe.stderr[-2000:]
    assert "libgqla_hostcheck.so" in probe.stdout and "libclang_rt.asan" in probe.stdout
    assert "/libgqla.so" not in probe.stdout
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_host_abi.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in r.stdout and "libgqla_hostcheck" in lib
