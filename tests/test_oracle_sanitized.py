"""The oracle and the host side of the ABI under AddressSanitizer + UndefinedBehaviorSanitizer.

CPU only: the oracle's C source is rebuilt with -fsanitize=address,undefined and the pin suite and
the host ABI checks run against that build in a child process whose LD_PRELOAD starts with the
sanitizer runtime (whatever the environment already preloads stays in the list). An out-of-bounds
access, a misaligned load or a signed overflow anywhere in the oracle aborts the child."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_and_host_abi_pass_under_address_and_ub_sanitizers():
    sys.path.insert(0, ROOT)
    from oracle import build as obuild
    lib = obuild.build_sanitized()
    rt = obuild.sanitizer_runtime()
    assert os.path.exists(rt), rt
    env = dict(os.environ)
    env["RTL_ORACLE_LIB"] = lib
    env["LD_PRELOAD"] = " ".join(x for x in (rt, env.get("LD_PRELOAD", "")) if x)
    # python itself leaks by design at exit; the oracle allocates nothing that outlives a call
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:allocator_may_return_null=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = env.get("OMP_NUM_THREADS", "8")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_abi_host.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
