"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code, on the CPU:
  * the oracle (gcc -fsanitize=address,undefined) under its whole pin suite;
  * the library's host side -- argument validation and dispatch -- (hipcc with the sanitizers on
    the host pass only; device code is built as usual) under the host ABI tests.
Each runs in a child interpreter with the matching sanitizer runtime loaded first (the two
compilers' runtimes cannot share a process).  An existing LD_PRELOAD is kept, after the runtime."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _env(runtime, **extra):
    env = dict(os.environ)
    prior = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + prior if prior else "")
    # the interpreter itself is not instrumented: its exit-time leaks are not ours to report, and the
    # runtime arrives by preload rather than as the executable's first dependency
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def _run_pytest(files, env, timeout):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + files
    r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=timeout)
    text = r.stdout.decode(errors="replace")
    assert r.returncode == 0, text[-4000:]
    assert "runtime error" not in text and "AddressSanitizer" not in text, text[-4000:]
    return text


def test_oracle_pins_under_asan_ubsan(tmp_path):
    import oracle
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"]).decode().strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    so = str(tmp_path / "libbwta_oracle_san.so")
    oracle.build(out=so, extra_flags=["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"])
    text = _run_pytest(["tests/test_oracle_pins.py"], _env(runtime, BWTA_ORACLE_LIB=so), 900)
    assert " passed" in text


def test_host_abi_under_asan_ubsan(tmp_path):
    import glob
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    rts = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not os.path.exists(hipcc) or not rts:
        pytest.skip("hipcc or its AddressSanitizer runtime is not installed")
    from paper_2604_03957_amd import build as hip_build
    so = str(tmp_path / "libbwta_san.so")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    # only the host-side translation unit with the C ABI needs the instrumented build to be meaningful,
    # but the launchers it calls live in the other files: build all of them the same way, at -O1
    cmd = [hipcc] + [f for f in hip_build.HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g", "-shared"] + san + \
          ["-shared-libsan", "-o", so] + hip_build.sources()
    subprocess.check_call(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = _run_pytest(["tests/test_abi_host.py"], _env(rts[0], BWTA_LIB=so), 900)
    assert " passed" in text
