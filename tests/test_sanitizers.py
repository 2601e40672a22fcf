"""Host-side sanitizer leg (CPU only): the fp64 oracle and the host code of the C-ABI library (argument
checks, workspace arithmetic, launch geometry) are rebuilt with AddressSanitizer and
UndefinedBehaviourSanitizer, and the oracle's pins / the ABI's host-side rejections are run against those
builds in a child interpreter.  Device code is not instrumented (no GPU sanitizer here); a sanitizer
report aborts the child and fails the test."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import ctypes, sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {root!r} + "/tests")
{setup}
import pytest
sys.exit(pytest.main(["-q", "-x", "-p", "no:cacheprovider"] + {args!r}))
"""


def _run_child(setup, args, runtime):
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:protect_shadow_gap=0"            # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["LD_PRELOAD"] = " ".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    p = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, setup=setup, args=args)], env=env,
                       capture_output=True, text=True, timeout=900)
    assert p.returncode == 0, (p.stdout[-3000:], p.stderr[-3000:])
    assert "passed" in p.stdout and "ERROR: AddressSanitizer" not in p.stderr and "runtime error" not in p.stderr


def test_oracle_pins_under_address_and_ub_sanitizers(tmp_path):
    lib = tmp_path / "liboracle_san.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fno-fast-math",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", str(lib),
                           os.path.join(ROOT, "oracle", "svip_oracle.c"), "-lm"])
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    setup = f"import oracle\noracle._lib = oracle._bind(ctypes.CDLL({str(lib)!r}))"
    # every pin except the three 10^6-trial ones (minutes under the sanitizers; they add no new code paths)
    _run_child(setup, [os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-k",
                       "not brute_force and not through_the_entry_points and not frequencies"], runtime)


def test_abi_host_checks_under_address_and_ub_sanitizers(tmp_path):
    from paper_2411_18462_amd import build as hip_build
    lib = tmp_path / "libsvip_san.so"
    flags = [f for f in hip_build.HIPCC_FLAGS if f != "-O3"]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), *flags, "-O1", "-g",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", *hip_build.SOURCES, "-o", str(lib)]
    p = subprocess.run(cmd, capture_output=True, text=True)
    assert p.returncode == 0, p.stderr[-3000:]
    rts = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    assert rts, "the ROCm clang AddressSanitizer runtime is not where it is expected"
    setup = f"import paper_2411_18462_amd.binding as b\nb.LIB_PATH = {str(lib)!r}"
    _run_child(setup, [os.path.join(ROOT, "tests", "test_abi.py"), "-k", "not header_is_plain"], rts[0])
