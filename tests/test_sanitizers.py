"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

1. The oracle (oracle/modet_oracle.cpp) is rebuilt with g++ -fsanitize=address,undefined and the oracle's own
   pin tests run against that build in a child process.
2. The host side of the C ABI (csrc/modet_api.hip: argument validation, which returns before any HIP call) is
   rebuilt with the sanitizers on the host pass only and tests/test_host_abi.py runs against that library.
The sanitizer runtimes are preloaded into the child interpreters; a report makes the child exit non-zero."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _rt(compiler, name):
    try:
        p = subprocess.run([compiler, f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    except OSError:
        return None
    return p if os.path.isabs(p) and os.path.exists(p) else None


def _child_env(preload, **extra):
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload
    # python itself leaks at exit and installs its own handlers; everything else stays fatal
    env["ASAN_OPTIONS"] = "detect_leaks=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"      # (the code under test is built with -fno-sanitize-recover)
    env["PYTHONPATH"] = ROOT + os.pathsep + os.path.join(ROOT, "tests")
    env.update(extra)
    return env


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    asan, ubsan = _rt("gcc", "libasan.so"), _rt("gcc", "libubsan.so")
    if not asan or not ubsan:
        pytest.skip("gcc's sanitizer runtimes are not installed")
    lib = str(tmp_path / "libmodet_oracle_san.so")
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-o", lib, os.path.join(ROOT, "oracle", "modet_oracle.cpp")], check=True)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_warp_adjoint.py"),
                        os.path.join(ROOT, "tests", "test_oracle_fields.py")],
                       env=_child_env(asan + ":" + ubsan, MODET_ORACLE_LIBRARY=lib), capture_output=True, text=True,
                       cwd=ROOT)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout


def test_host_abi_under_asan_and_ubsan(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not hipcc or not os.path.exists(clang):
        pytest.skip("hipcc is not installed")
    asan = _rt(clang, "libclang_rt.asan-x86_64.so")
    objdir = os.path.join(ROOT, "paper_2403_16526_amd", "_build")
    from paper_2403_16526_amd import build as b
    others = [os.path.join(objdir, s.replace(".hip", ".o")) for s in b.SOURCES if s != "modet_api.hip"]
    if not asan or not all(os.path.exists(o) for o in others):
        pytest.skip("needs clang's asan runtime and the objects of a previous build of libmodet")
    obj, lib = str(tmp_path / "modet_api_san.o"), str(tmp_path / "libmodet_san.so")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    subprocess.run([hipcc, *b.FLAGS, *san, "-g", "-c", os.path.join(b.CSRC, "modet_api.hip"), "-o", obj], check=True,
                   stderr=subprocess.DEVNULL)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan", "-fsanitize=address",
                    "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", lib, obj, *others], check=True,
                   stderr=subprocess.DEVNULL)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "-k", "not binding",      # (that test imports torch, which is not what is under test here)
                        os.path.join(ROOT, "tests", "test_host_abi.py")],
                       env=_child_env(asan, MODET_LIBRARY=lib), capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout
