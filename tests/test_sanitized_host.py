"""Host-side sanitizer runs (CPU only): the oracle built with AddressSanitizer + UBSan runs its pins, and the
HIP library built with the sanitizers on its host code (argument checking, workspace planning, launch glue)
runs the ABI tests.  Each run is a child pytest process with the matching sanitizer runtime preloaded."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUILD = os.path.join(ROOT, "_build")


def run_child(tests, env_extra, runtime):
    env = dict(os.environ)
    env.update(env_extra)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + pre if pre else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + tests,
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return tail


def test_oracle_pins_under_asan_and_ubsan():
    from oracle import build as ob
    os.makedirs(BUILD, exist_ok=True)
    lib = ob.build(sanitize=True, out=os.path.join(BUILD, "libsfo_san.so"))
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime):
        pytest.skip("gcc has no shared AddressSanitizer runtime here")
    tail = run_child(["tests/test_oracle_accept.py", "tests/test_oracle_attention.py", "tests/test_oracle_ops.py",
                      "tests/test_oracle_model.py"], {"SFO_LIB": lib}, runtime)
    assert " passed" in tail


def test_abi_host_glue_under_asan_and_ubsan():
    from paper_2511_20340_amd import build as hb
    os.makedirs(BUILD, exist_ok=True)
    lib = hb.build_host_sanitized(os.path.join(BUILD, "libspecformer_san.so"))
    clang = os.path.join(os.path.dirname(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), "..", "lib", "llvm", "bin", "clang++")
    runtime = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True,
                             text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("clang has no shared AddressSanitizer runtime here")
    tail = run_child(["tests/test_abi.py", "tests/test_linear_config.py"], {"SF_LIB": lib}, runtime)
    assert " passed" in tail
