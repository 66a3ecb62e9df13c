"""CPU-side hardening: the oracle and the host layer of the C ABI run under the address and
undefined-behaviour sanitizers (no GPU, no GPU code instrumented).

* tests/c_abi/oracle_sanitized.c + oracle/ems_oracle.c, built with gcc -fsanitize=address,undefined,
  drive every oracle function over ragged inputs in exactly-sized buffers;
* the oracle's pin tests run against a copy of the oracle built with -fsanitize=undefined
  (no recovery: any undefined operation aborts the child process);
* tests/c_abi/api_host_sanitized.c + csrc/ems_api.hip with its host side instrumented + launch stubs,
  built with the ROCm clang's sanitizers, walk every entry point's refusals and accepted paths.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = os.path.join(ROOT, "oracle", "ems_oracle.c")
C_ABI = os.path.join(ROOT, "tests", "c_abi")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    return res.returncode, res.stdout, err


def test_oracle_functions_are_memory_safe_on_exactly_sized_buffers(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    rc, out, err = run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp"] + SAN +
                       ["-o", exe, os.path.join(C_ABI, "oracle_sanitized.c"), ORACLE_SRC, "-lm"])
    assert rc == 0, err
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    rc, out, err = run([exe], env=env)
    assert rc == 0 and out.strip() == "ok", (rc, out, err[-3000:])
    assert "AddressSanitizer" not in err and "runtime error" not in err, err[-3000:]


def test_oracle_pins_pass_without_undefined_behaviour(tmp_path):
    lib = str(tmp_path / "libems_oracle_ubsan.so")
    rc, out, err = run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fsanitize=undefined",
                        "-fno-sanitize-recover=all", "-o", lib, ORACLE_SRC, "-lm"])
    assert rc == 0, err
    env = dict(os.environ, EMS_ORACLE_LIBRARY=lib, OMP_NUM_THREADS="4")
    pins = ["tests/test_oracle_attention.py", "tests/test_oracle_accept_append.py", "tests/test_oracle_tree.py",
            "tests/test_oracle_padded.py"]
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + pins,
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert res.returncode == 0, (res.stdout[-2000:], res.stderr[-2000:])
    assert "runtime error" not in res.stderr, res.stderr[-3000:]


def test_api_host_layer_is_memory_safe_down_to_every_launch(tmp_path):
    hipcc = os.path.join(ROCM, "bin", "hipcc")
    clang = os.path.join(ROCM, "lib", "llvm", "bin", "clang")
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("needs the ROCm compilers")
    host_san = []
    for flag in SAN:
        host_san += ["-Xarch_host", flag]
    api_o, stubs_o, drv_o, exe = (str(tmp_path / n) for n in ("api_host.o", "stubs.o", "driver.o", "api_host_sanitized"))
    api_src = os.path.join(ROOT, "paper_2405_07542_amd", "csrc", "ems_api.hip")
    for cmd in (
        # (host code instrumented, device image left as it is: the API's translation unit carries the
        # static device buffer of ems_verify_attention_noalloc, which its host side registers)
        [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950"] + host_san + ["-c", api_src, "-o", api_o],
        [hipcc, "-O1", "-g", "-std=c++17", "-x", "hip", "--cuda-host-only"] + host_san +
        ["-c", os.path.join(C_ABI, "launch_stubs.cpp"), "-o", stubs_o],
        [clang, "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-Werror"] + SAN +
        ["-I", os.path.join(ROOT, "include"), "-c", os.path.join(C_ABI, "api_host_sanitized.c"), "-o", drv_o],
        [hipcc] + host_san + ["-o", exe, drv_o, stubs_o, api_o, "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
                                "-Wl,-rpath," + os.path.join(ROCM, "lib")],
    ):
        rc, out, err = run(cmd)
        assert rc == 0, (" ".join(cmd), err[-3000:])
    # (leak checking off: the HIP runtime's own start-up allocations are not this library's)
    rc, out, err = run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert rc == 0 and out.startswith("ok "), (rc, out, err[-3000:])
    assert "AddressSanitizer" not in err and "runtime error" not in err, err[-3000:]
