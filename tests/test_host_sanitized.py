"""The host-side sources of the library (index maps, hybrid token scheduler, graph pruning) compiled for the CPU
under AddressSanitizer + UndefinedBehaviorSanitizer, with the host test files run against that build in a child
process (the sanitizer runtime has to be the first library of the process).  Any finding aborts the child."""
import importlib.util
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build_module():
    spec = importlib.util.spec_from_file_location("flexco_build", os.path.join(ROOT, "paper_2402_18789_amd", "build.py"))
    b = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(b)
    return b


def test_host_sources_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = str(tmp_path / "libflexco_host_san.so")
    _build_module().build_host_sanitized(lib)
    asan = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no shared AddressSanitizer runtime beside g++")
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["FLEXCO_LIB_PATH"], env["FLEXCO_HOST_ONLY"] = lib, "1"
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"        # the interpreter's own allocations are not ours
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           "tests/test_abi_host.py", "tests/test_sched_host.py", "tests/test_prune_host.py"]
    # (the few tests there that call device entry points skip themselves on a host-only build)
    r = subprocess.run(cmd, capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    out = r.stdout + r.stderr
    if "ASan runtime does not come first" in out:
        pytest.skip("another preloaded library precedes the sanitizer runtime in this environment")
    assert r.returncode == 0, out[-4000:]
    assert "passed" in r.stdout and "failed" not in r.stdout, out[-2000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
