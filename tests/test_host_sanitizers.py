"""Sanitizer tier for the host-side logic of the library: argument validation, workspace sizing, the pseudo-sequence
builder and the draft maker are rebuilt with AddressSanitizer + UndefinedBehaviorSanitizer in their HOST code (device
code is never sanitized) and the host test files are run against that build in a child process.  No GPU involved."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    from paper_2407_12021_amd import build
    try:
        rt = build.asan_runtime()
    except RuntimeError as e:
        pytest.skip(str(e))
    lib = build.build_host_sanitizer_library()
    env = dict(os.environ)
    env.update({
        "LD_PRELOAD": (rt + ":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else rt,
        # the interpreter and the vendor runtime are not built for leak checking; every other report is fatal
        "ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
        "DED_VERIFY_LIB": lib,
        "PYTHONPATH": ROOT,
    })
    # test_host_api_from_plain_c links an unsanitized C program against the library: not part of this tier
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", "not plain_c",
           os.path.join(ROOT, "tests", "test_abi_host.py"), os.path.join(ROOT, "tests", "test_drafter_host.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in out
