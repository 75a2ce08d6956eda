"""CPU sanitizer tier: the oracle under AddressSanitizer + UndefinedBehaviorSanitizer, the library's host half
(argument checks, planner, scratch bookkeeping) under UndefinedBehaviorSanitizer.  No GPU is involved: the oracle is
plain C, and the host tests never get as far as a HIP call.

Each part builds its sanitized library and runs the existing test files against it in a child process (the sanitizer's
runtime has to be in the process before Python starts; the children find the libraries through CHELA_ORACLE_LIB and
CHELA_LIB)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest(files, env_extra):
    env = dict(os.environ)
    env.update(env_extra)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = "\n".join(r.stdout.splitlines()[-25:])
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout.splitlines()[-1], tail
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, tail
    return r.stdout


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    from oracle.build import asan_runtime, build
    lib = build(force=True, sanitize=True)
    pre = os.environ.get("LD_PRELOAD", "")
    out = _run_pytest(
        ["tests/test_oracle_pins.py", "tests/test_oracle_layer_pins.py", "tests/test_oracle_conv_pins.py"],
        {"CHELA_ORACLE_LIB": lib,
         "LD_PRELOAD": asan_runtime() + (":" + pre if pre else ""),        # the runtime has to come first
         # Python itself leaks by design; a report there would bury the oracle's
         "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1",
         "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"})
    print(out.splitlines()[-1])


def test_host_half_of_the_library_under_undefined_behaviour_sanitizer():
    from paper_2406_08128_amd.build import build_host_ubsan
    lib = build_host_ubsan()
    # every host test, the 3000-shape planner sweep and the eight-thread scratch test among them; a trap ends the child
    out = _run_pytest(["tests/test_abi_host.py"], {"CHELA_LIB": lib})
    print(out.splitlines()[-1])
