"""The host side of the C-ABI library (argument checks, error texts, struct handling) built with
AddressSanitizer and UndefinedBehaviorSanitizer, and the ABI tests run against that build in a child
process.  Device code is compiled as usual; nothing here launches a kernel."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _clang_runtime(name):
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/" + name))
    return hits[-1] if hits else None


def test_abi_checks_pass_with_host_sanitizers(tmp_path):
    asan = _clang_runtime("libclang_rt.asan-x86_64.so")
    if not asan:
        pytest.skip("the compiler's sanitizer runtimes are not installed")
    from paper_2605_16637_amd import build
    lib = build.build(out=str(tmp_path / "libhx_san.so"), extra_flags=build.HOST_SANITIZE)
    env = dict(os.environ)
    # the address sanitizer's runtime carries the undefined-behaviour handlers too (preloading the stand-alone
    # runtime beside it makes every process spin at start-up)
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    log = str(tmp_path / "sanitizer")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:exitcode=86:protect_shadow_gap=0:log_path=" + log
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:log_path=" + log
    # the child hands the binding the sanitized build, loaded directly (nothing here touches a GPU, so the order in
    # which PyTorch's and the library's HIP runtimes come up does not matter)
    code = ("import ctypes, sys, pytest\n"
            "from paper_2605_16637_amd import binding\n"
            "binding.LIB_PATH = %r\n"
            "lib = ctypes.CDLL(binding.LIB_PATH)\n"
            "for name in binding.EXPORTS: getattr(lib, name).restype = ctypes.c_int\n"
            "lib.hx_last_error.restype = ctypes.c_char_p\n"
            "binding._lib = lib\n"
            "rc = pytest.main(['-x', '-q', '-p', 'no:cacheprovider', %r])\n"
            "assert any('libhx_san' in l for l in open('/proc/self/maps')), 'the sanitized build was not the one loaded'\n"
            "sys.exit(int(rc))\n") % (lib, os.path.join(ROOT, "tests", "test_abi.py"))
    run = subprocess.run([sys.executable, "-c", code], env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=120)
    tail = "\n".join(run.stdout.splitlines()[-40:])
    for f in sorted(os.listdir(tmp_path)):
        if f.startswith("sanitizer"):
            tail += "\n" + open(tmp_path / f).read()[:4000]
    assert run.returncode == 0, tail
    assert "passed" in tail and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
