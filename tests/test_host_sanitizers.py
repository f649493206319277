"""The host layer of the library (argument checks, range planning, rank selection: csrc/skv_host.cpp) built
with AddressSanitizer and UndefinedBehaviorSanitizer and put through the C-ABI tests of test_abi_host.py.
Kernel launchers are replaced by stubs that launch nothing, so no GPU is needed; the sanitised build holds the
host layer only."""
import os
import re
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_21686_amd", "csrc")
OUT_DIR = os.path.join(ROOT, "_build", "sanitized")


def _launcher_stubs() -> str:
    """A definition that launches nothing for every launcher skv_internal.h declares."""
    hdr = open(os.path.join(CSRC, "skv_internal.h")).read()
    hdr = re.sub(r"//.*", "", hdr)
    lines = ['#include "skv_internal.h"', "namespace skv {"]
    for m in re.finditer(r"hipError_t\s+(launch_[a-z0-9_]+)\s*\(([^;{]*?)\)\s*;", hdr, flags=re.S):
        lines.append(f"hipError_t {m.group(1)}({m.group(2)}) {{ return hipSuccess; }}")
    lines.append("}")
    return "\n".join(lines) + "\n"


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_host_layer_under_address_and_undefined_behaviour_sanitizers():
    os.makedirs(OUT_DIR, exist_ok=True)
    stubs = os.path.join(OUT_DIR, "launcher_stubs.cpp")
    with open(stubs, "w") as f:
        f.write(_launcher_stubs())
    lib = os.path.join(OUT_DIR, "libskv_host_sanitized.so")
    rocm_inc = "/opt/rocm/include"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-I" + rocm_inc,
           os.path.join(CSRC, "skv_host.cpp"), stubs, "-o", lib]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr[-4000:]
    asan_rt = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.exists(asan_rt), asan_rt
    env = dict(os.environ)
    env["SKV_LIBRARY"] = lib
    env["LD_PRELOAD"] = asan_rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"      # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_host.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    tail = (run.stdout + run.stderr)[-6000:]
    assert run.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert re.search(r"\d+ passed", run.stdout), tail
