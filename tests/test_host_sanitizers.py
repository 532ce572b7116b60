"""The library's host side (argument checks, context bookkeeping, plans, the layout functions, the stack
driver's glue) under AddressSanitizer and UndefinedBehaviorSanitizer: ptenc_api.hip and stack_api.hip are
rebuilt with both on their host code, and the host-only ABI tests run against that build in a child
process (the sanitizer runtime has to be loaded before the interpreter's own allocator is used).  No
kernel runs, so this needs no GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_glue_is_clean_under_address_and_undefined_behaviour_sanitizers():
    from paper_2602_16839_amd import build as B
    if not os.path.exists(os.path.join(B.OBJ_DIR, "decode_mfma.o")):
        pytest.skip("the ordinary build's objects are not there (run python -m paper_2602_16839_amd.build)")
    lib = B.build_host_sanitized()
    env = dict(os.environ)
    env.update(LD_PRELOAD=B.sanitizer_runtime(), PTENC_LIB=lib,
               # the interpreter and its extension modules are not built for leak checking
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_host.py"), "-q", "-x",
                          "-p", "no:cacheprovider"],
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    out = res.stdout
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert res.returncode == 0 and " passed" in out, out[-4000:]
    # and the child really ran on the sanitized build
    probe = subprocess.run([sys.executable, "-c",
                            "from paper_2602_16839_amd import ptenc; ptenc.lib(); "
                            "print(any('libptenc_hostsan' in l for l in open('/proc/self/maps')))"],
                           cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert probe.stdout.strip().endswith("True"), probe.stdout[-2000:]
