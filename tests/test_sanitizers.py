"""CPU sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer) of the two pieces of native code that run on the
host: the C oracle, and the argument-validation layer of libssmv (csrc/api.hip, everything above the first launch).

* The oracle is rebuilt with gcc's sanitizers and its pins and invariants are run on that build, in a child interpreter
  that has the sanitizer runtime preloaded.
* api.hip is compiled for the host with clang's sanitizers (device code is not instrumented) and linked against stand-in
  launchers (tests/host_stubs) into a library of its own; the ABI tests, whose calls all end on the host, are run on it.
Any report of either sanitizer aborts the child (-fno-sanitize-recover / halt_on_error), which fails the test.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2408_15237_amd", "csrc")


def _run(env_extra, args, timeout=600):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1"     # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + args, cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=timeout)
    assert r.returncode == 0, "sanitizer run failed:\n%s\n%s" % (r.stdout[-4000:], r.stderr[-4000:])
    assert "passed" in r.stdout
    return r.stdout


def _preload(env, lib):
    return {"LD_PRELOAD": lib + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")}


def test_oracle_pins_under_address_and_ub_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    env = _preload(os.environ, os.path.realpath(asan))
    env["SSM_ORACLE_SANITIZE"] = "1"
    out = _run(env, ["tests/test_oracle_pins.py", "tests/test_oracle_invariants.py"])
    assert os.path.exists(os.path.join(ROOT, "oracle", "libssm_oracle_san.so")), out


def test_argument_validation_layer_under_address_and_ub_sanitizers(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc"
    rt = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        import glob
        cand = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        if not cand:
            pytest.skip("clang's AddressSanitizer runtime is not installed")
        rt = cand[0]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    common = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC"] + inc
    objs = []
    for src in (os.path.join(CSRC, "api.hip"), os.path.join(ROOT, "tests", "host_stubs", "launch_stubs.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        cmd = common + host_san + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    lib = str(tmp_path / "libssmv_hostsan.so")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
                        "-shared-libsan"] + objs + ["-o", lib], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = _preload(os.environ, os.path.realpath(rt))
    env["SSMV_LIBRARY"] = lib
    _run(env, ["tests/test_abi.py"])
