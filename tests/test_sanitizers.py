"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two jobs, each in a process of its own because the two compilers bring their own sanitizer runtimes:
  * the oracle (oracle/conv_oracle.c, gcc) rebuilt with -fsanitize=address,undefined and run through its pin tests;
  * the host dispatcher of the HIP library (csrc/api.hip: descriptor validation, variant registry and selection, cache
    files, every entry point's argument checks) rebuilt with the host pass instrumented, linked against the
    uninstrumented kernel objects, and run through the host-API tests.
A sanitizer report makes the child process exit non-zero.  The jobs are skipped when a tool they need is missing.
"""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run_pytest(files, env_extra, preload):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = ":".join([preload] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    env["OMP_NUM_THREADS"] = "4"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + files
    return subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip() if gcc else ""
    if not gcc or not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc or its libasan.so is not available")
    lib = str(tmp_path / "liboracle_conv_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", lib,
                           os.path.join(ROOT, "oracle", "conv_oracle.c")])
    p = _run_pytest(["tests/test_oracle_pins.py"], {"ORACLE_CONV_LIB": lib}, asan)
    assert p.returncode == 0, p.stdout[-4000:]
    assert "passed" in p.stdout and "ERROR: AddressSanitizer" not in p.stdout and "runtime error:" not in p.stdout, p.stdout[-4000:]


def test_host_dispatcher_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    rt = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    objs = [o for o in glob.glob(os.path.join(ROOT, "_build", "*.o")) if os.path.basename(o) != "api.o"]
    if not os.path.exists(HIPCC) or not rt:
        pytest.skip("hipcc or the clang AddressSanitizer runtime is not available")
    if len(objs) < 10:
        pytest.skip("the kernel objects of a library build (_build/*.o) are not there to link against")
    api_o = str(tmp_path / "api_san.o")
    flags = ["-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-value", "-Wno-unknown-warning-option", "-fno-omit-frame-pointer",
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined"]
    subprocess.run([HIPCC] + flags + ["-c", os.path.join(ROOT, "paper_1611_06945_amd", "csrc", "api.hip"), "-o", api_o],
                   check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    lib = str(tmp_path / "libconvfwd_san.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-shared-libsan", "-o", lib, api_o] + objs, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    p = _run_pytest(["tests/test_host_api.py"], {"CONVFWD_LIB": lib}, rt[0])
    assert p.returncode == 0, p.stdout[-4000:]
    assert "passed" in p.stdout and "ERROR: AddressSanitizer" not in p.stdout and "runtime error:" not in p.stdout, p.stdout[-4000:]
