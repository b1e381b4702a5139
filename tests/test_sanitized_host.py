"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the oracle's C file
and the host side of the library (argument checks, the fusion pass) are rebuilt with
-fsanitize=address,undefined and the CPU suites that drive them run again in a child process
against those builds.  Device code is not instrumented; nothing here launches a kernel."""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1904_08368_amd", "csrc")
OBJ = os.path.join(ROOT, "paper_1904_08368_amd", "_build")
LLVM = "/opt/rocm/lib/llvm"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SUITES = ["tests/test_abi_cpu.py", "tests/test_fusion.py", "tests/test_oracle_pins.py"]

RUNNER = r"""
import sys
sys.path.insert(0, {root!r})
import oracle
oracle._SO = {oracle_so!r}
oracle.build = lambda force=False: oracle._SO          # the sanitized build is the one to load
from paper_1904_08368_amd import binding
binding.LIB_PATH = {relay_so!r}
import pytest
sys.exit(pytest.main(["-q", "-x", "-p", "no:cacheprovider", "-k", "not sanitized"] + {suites!r}))
"""


def _asan_runtime():
    hits = glob.glob(os.path.join(LLVM, "lib", "clang", "*", "lib", "linux", "libclang_rt.asan-x86_64.so"))
    return hits[0] if hits else None


@pytest.mark.timeout(600)
def test_host_suites_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    rt = _asan_runtime()
    clang = os.path.join(LLVM, "bin", "clang")
    if rt is None or not os.path.exists(clang) or not os.path.exists(HIPCC):
        pytest.skip("no clang sanitizer runtime in this image")
    from paper_1904_08368_amd.build import SOURCES
    others = [os.path.join(OBJ, src + ".o") for src in SOURCES if src not in ("api.cpp", "fusion.cpp")]
    if not all(os.path.exists(o) for o in others):
        pytest.skip("the library's objects are not built (run build() first)")
    san = ["-fsanitize=address", "-fsanitize=undefined"]
    oracle_so = str(tmp_path / "liboracle_san.so")
    subprocess.run([clang, "-O1", "-g", *san, "-fno-sanitize-recover=undefined", "-shared-libsan", "-ffp-contract=off",
                    "-fPIC", "-shared", "-std=c11", "-Wall", "-o", oracle_so, os.path.join(ROOT, "oracle", "oracle.c")],
                   check=True)
    # host passes instrumented, device passes untouched (each -fsanitize= directly behind -Xarch_host)
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-x", "hip", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument", *host_san]
    objs = []
    for src in ("api.cpp", "fusion.cpp"):
        obj = str(tmp_path / (src + ".o"))
        r = subprocess.run([HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    relay_so = str(tmp_path / "librelayfused_san.so")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                        "-shared-libsan", "-fno-gpu-sanitize", "-o", relay_so, *objs, *others], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ)
    # the runtime has to be in the process before the interpreter's own allocations; whatever is
    # preloaded already stays in place
    env["LD_PRELOAD"] = ":".join(x for x in (rt, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "1"
    code = RUNNER.format(root=ROOT, oracle_so=oracle_so, relay_so=relay_so, suites=SUITES)
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=540)
    tail = (r.stdout + r.stderr)[-4000:]
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert r.returncode == 0, tail
    assert " passed" in r.stdout, tail
