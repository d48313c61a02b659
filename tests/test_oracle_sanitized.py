"""The oracle's pins once more against a build of the same source with AddressSanitizer and
UndefinedBehaviorSanitizer (every finding fatal): an out-of-bounds index, a use of uninitialised stack or
heap bookkeeping, a signed overflow or a bad shift in the checker would otherwise go unnoticed, or be
mistaken for a property of the method.  Host code only; runs in a child process because the sanitizer
runtime has to be loaded before Python's own allocations."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    path = subprocess.check_output(["gcc", "-print-file-name=" + name], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("gcc's sanitizer runtimes are not installed")
    from oracle import hx_oracle as o
    lib = o.build_sanitized(str(tmp_path / "libhx_oracle_san.so"))
    env = dict(os.environ)
    env["HXO_LIB"] = lib
    env["LD_PRELOAD"] = ":".join(x for x in (asan, ubsan, env.get("LD_PRELOAD", "")) if x)
    # Python itself leaks by design; the link order check would object to whatever else is preloaded
    log = str(tmp_path / "sanitizer")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=86:log_path=" + log
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:log_path=" + log
    env["OMP_NUM_THREADS"] = "2"
    pins = sorted(f for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle_") and f.endswith(".py")
                  and f != os.path.basename(__file__))
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *[os.path.join(ROOT, "tests", f) for f in pins]]
    run = subprocess.run(cmd, env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = "\n".join(run.stdout.splitlines()[-40:])
    for f in sorted(os.listdir(tmp_path)):             # what the sanitizers wrote before ending the child
        if f.startswith("sanitizer"):
            tail += "\n" + open(tmp_path / f).read()[:4000]
    assert run.returncode == 0, tail
    assert "passed" in tail and "ERROR: AddressSanitizer" not in run.stdout and "runtime error" not in run.stdout, tail
    # and the child really ran on the sanitized build
    probe = subprocess.run([sys.executable, "-c", "from oracle import hx_oracle as o; o.lib(); "
                            "print(any('libhx_oracle_san' in l for l in open('/proc/self/maps')))"],
                           env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert probe.stdout.strip().endswith("True"), probe.stdout
