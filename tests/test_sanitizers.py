"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

  * the oracle (oracle/cask_ref.c) is rebuilt with -fsanitize=address,undefined and its whole pin
    suite (tests/test_oracle_pins.py, tests/test_parity_rules.py) runs against that build in a
    child process;
  * the HIP library's host layer (argument checks, budget split, workspace layout) is rebuilt
    with the sanitizers on the host pass only (device code cannot be sanitized here) and
    tests/test_abi_host.py runs against it.
A report from either sanitizer aborts the child (halt_on_error / -fno-sanitize-recover), so a
zero exit status means none was raised.  Leak checking is off: the interpreter itself never
frees everything."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(compiler, name):
    out = subprocess.run([compiler, f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def _child_env(preload, **extra):
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join([preload] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["PYTHONPATH"] = ROOT
    env.update(extra)
    return env


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    asan = _runtime("gcc", "libasan.so")
    if asan is None:
        pytest.skip("gcc has no libasan here")
    lib = str(tmp_path / "libcask_ref_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-fno-omit-frame-pointer", "-o", lib, os.path.join(ROOT, "oracle", "cask_ref.c"), "-lm"],
                   check=True)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_parity_rules.py")],
                       cwd=ROOT, env=_child_env(asan, CASK_REF_LIB=lib, OMP_NUM_THREADS="4"),
                       capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail


def test_library_host_layer_passes_under_asan_and_ubsan(tmp_path):
    """libcask.so with its host pass sanitized; no kernel is launched by tests/test_abi_host.py."""
    from paper_2604_10900_amd import build as B
    hipcc = B.hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    clang = os.path.join(os.path.dirname(hipcc), "..", "llvm", "bin", "clang")
    asan = _runtime(clang, "libclang_rt.asan-x86_64.so") if os.path.exists(clang) else None
    if asan is None:
        pytest.skip("no shared ASan runtime for the HIP host compiler")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-shared-libsan", "-g"]
    lib = str(tmp_path / "libcask_san.so")
    objs = []
    for src in B.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        flags = [f for f in B.compile_flags() if f != "-O3"] + ["-O1"]
        subprocess.run([hipcc] + flags + san + ["-c", os.path.join(B.CSRC, src), "-o", obj],
                       check=True, capture_output=True)
        objs.append(obj)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address",
                    "-fsanitize=undefined", "-shared-libsan", "-o", lib] + objs, check=True, capture_output=True)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi_host.py")],
                       cwd=ROOT, env=_child_env(asan, CASK_LIB=lib), capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
