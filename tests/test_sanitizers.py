"""Host-side sanitizer runs (no GPU): the C oracle and the ABI's host logic (argument checks,
launch planning, workspace carving) are rebuilt with AddressSanitizer and
UndefinedBehaviorSanitizer and their CPU tests are run again against those builds, each in a
process of its own that has the sanitizer runtime loaded first.  Device code is not
instrumented: GPU sanitizers are not available here."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest_with(preload, patch, test_file, tmp_path):
    """Runs `test_file` in a child interpreter after `patch` (python source that points the
    package at the sanitized library), with `preload` ahead of whatever is preloaded already."""
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (preload, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    code = (f"import sys; sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})\n"
            f"{patch}\n"
            f"import pytest; sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', {test_file!r}]))\n")
    r = subprocess.run([sys.executable, "-c", code], env=env, cwd=str(tmp_path), capture_output=True, text=True)
    tail = (r.stdout + r.stderr)[-3000:]
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert r.returncode == 0, tail
    return r.stdout


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libcaote_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", "-o", lib, os.path.join(ROOT, "oracle", "caote_oracle.c"), "-lm"])
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.exists(asan)
    out = _run_pytest_with(asan, f"import oracle; oracle._LIB = {lib!r}",
                           os.path.join(ROOT, "tests", "test_oracle_pins.py"), tmp_path)
    assert " passed" in out and "failed" not in out


def test_abi_host_logic_under_asan_and_ubsan(tmp_path):
    """caote_abi.hip (every host-side check, plan() and the workspace arithmetic) compiled with the
    host sanitizers and linked with the kernels' ordinary objects; the host ABI tests run against it."""
    from paper_2504_14051_amd import build as hip_build
    if not glob.glob(os.path.join(hip_build.OBJ, "*.o")):
        hip_build.build()
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rt:
        pytest.skip("clang's shared AddressSanitizer runtime is not installed")
    obj = str(tmp_path / "caote_abi.san.o")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f for f in hip_build.FLAGS if f != "-O3"]
    subprocess.run([hip_build.HIPCC, *flags, "-O1", "-g", *san, "-c",
                    os.path.join(hip_build.CSRC, "caote_abi.hip"), "-o", obj],
                   check=True, capture_output=True)
    others = [o for o in glob.glob(os.path.join(hip_build.OBJ, "*.o")) if not o.endswith("caote_abi.hip.o")]
    lib = str(tmp_path / "libcaote_hip_san.so")
    subprocess.run([hip_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan",
                    "-fsanitize=address", "-fsanitize=undefined", "-o", lib, obj, *others],
                   check=True, capture_output=True)
    out = _run_pytest_with(rt[0], f"from paper_2504_14051_amd import binding; binding.LIB_PATH = {lib!r}",
                           os.path.join(ROOT, "tests", "test_abi_host.py"), tmp_path)
    assert " passed" in out and "failed" not in out
