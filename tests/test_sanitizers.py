"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The library's host side (lane assignment, allocator, scheduler, C ABI argument
checks) and the dense oracle are rebuilt with the sanitizers and the existing
CPU tests are run against those builds in a child process; any report makes the
child fail.  Device code is not instrumented (host flags only)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG_ASAN = "/opt/rocm/lib/llvm/lib/clang/22/lib/linux/libclang_rt.asan-x86_64.so"


def run_under(preload, env_extra, args):
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # Python itself leaks by design and is not linked against the runtime
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(env_extra)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *args],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, r.stdout[-4000:]
    return r.stdout


def test_host_core_and_c_abi_under_asan_ubsan(tmp_path):
    if not os.path.exists(CLANG_ASAN):
        pytest.skip("clang sanitizer runtime not found")
    sys.path.insert(0, ROOT)
    from paper_1902_04610_amd import build as b
    so = str(tmp_path / "libsalus_san.so")
    b.build(extra_flags=("-g", "-shared-libsan",
                         "-Xarch_host", "-fsanitize=address",
                         "-Xarch_host", "-fsanitize=undefined",
                         "-Xarch_host", "-fno-sanitize-recover=undefined"), out=so)
    out = run_under(CLANG_ASAN, {"SALUS_LIBRARY": so},
                    ["tests/test_host_logic.py", "tests/test_replay.py", "-m", "not gpu"])
    assert " passed" in out


def test_dense_oracle_under_asan_ubsan(tmp_path):
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(asan):
        pytest.skip("gcc sanitizer runtime not found")
    so = str(tmp_path / "liboracle_dense_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fPIC", "-shared", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-o", so, os.path.join(ROOT, "oracle", "dense.c"), "-lm"])
    out = run_under(asan, {"ORACLE_DENSE_SO": so},
                    ["tests/test_oracle_dense.py", "tests/test_oracle_train.py", "-m", "not gpu"])
    assert " passed" in out
