"""Compiles the HIP sources into paper_2601_21686_amd/libskv.so for gfx950.

Run as `python -m paper_2601_21686_amd.build` (or through
__graft_entry__.build()).  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libskv.so")
PROBE_OUT = os.path.join(PKG, "libskv_probe.so")     # the benchmark's plain streaming kernels: a library of their own
BUILD_DIR = os.path.join(ROOT, "_build")

KEY_RANKS = (16, 32, 48, 64, 80, 96, 112, 128)
Q8_KEY_RANKS = (32, 64, 96, 128)          # the 8-bit quantised cache takes multiples of 32
Q4_KEY_RANKS = (64, 128)                  # the 4-bit one multiples of 64 (a lane owns whole 32-bit words of a row)

# Packed-FP32 instruction selection is switched off for all device code.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# The chunk attention keeps its matrix-core accumulators in ordinary vector registers (they are
# read by the softmax right after each product), which saves the copies out of the accumulation file.
PREFILL_FLAGS = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
# The matrix-core range kernel feeds its score accumulators to the softmax and rescales its mix
# accumulators in place: the same form saves it about 80 register copies per 32-row tile.
DECODE_FLAGS = PREFILL_FLAGS
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
          "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _jobs():
    jobs = [("skv_host.o", [os.path.join(CSRC, "skv_host.cpp")], []),
            ("skv_decode_combine.o", ["-x", "hip", os.path.join(CSRC, "skv_decode_combine.hip")], DEVICE_FLAGS),
            ("skv_project.o", ["-x", "hip", os.path.join(CSRC, "skv_project.hip")], DEVICE_FLAGS),
            ("skv_folded.o", ["-x", "hip", os.path.join(CSRC, "skv_folded.hip")], DEVICE_FLAGS),
            ("skv_append.o", ["-x", "hip", os.path.join(CSRC, "skv_append.hip")], DEVICE_FLAGS),
            ("skv_basis.o", ["-x", "hip", os.path.join(CSRC, "skv_basis.hip")], DEVICE_FLAGS),
            ("skv_static.o", ["-x", "hip", os.path.join(CSRC, "skv_static.hip")], DEVICE_FLAGS),
            ("skv_probe.o", ["-x", "hip", os.path.join(CSRC, "skv_probe.hip")], DEVICE_FLAGS)]
    for rk in KEY_RANKS:
        jobs.append((f"skv_decode_partial_rk{rk}.o",
                     ["-x", "hip", os.path.join(CSRC, "skv_decode_partial.hip"), f"-DSKV_RK={rk}"],
                     DEVICE_FLAGS + DECODE_FLAGS))
    for rk in KEY_RANKS:
        jobs.append((f"skv_prefill_rk{rk}.o",
                     ["-x", "hip", os.path.join(CSRC, "skv_prefill.hip"), f"-DSKV_RK={rk}"],
                     DEVICE_FLAGS + PREFILL_FLAGS))
    for rk in KEY_RANKS:                  # the chunk kernel over a paged cache
        jobs.append((f"skv_prefill_paged_rk{rk}.o",
                     ["-x", "hip", os.path.join(CSRC, "skv_prefill.hip"), f"-DSKV_RK={rk}", "-DSKV_PAGED=1"],
                     DEVICE_FLAGS + PREFILL_FLAGS))
    for rk in KEY_RANKS:                  # the same range kernel addressing its rows through a page table
        jobs.append((f"skv_decode_partial_paged_rk{rk}.o",
                     ["-x", "hip", os.path.join(CSRC, "skv_decode_partial.hip"), f"-DSKV_RK={rk}", "-DSKV_PAGED=1"],
                     DEVICE_FLAGS + DECODE_FLAGS))
    for rk in Q8_KEY_RANKS:
        jobs.append((f"skv_decode_partial_q8_rk{rk}.o",
                     ["-x", "hip", os.path.join(CSRC, "skv_decode_partial.hip"), f"-DSKV_RK={rk}", "-DSKV_QBITS=8"],
                     DEVICE_FLAGS + DECODE_FLAGS))
    for bits, ranks in ((8, Q8_KEY_RANKS), (4, Q4_KEY_RANKS)):   # quantised rows in pages (matrix-core kernel only)
        for rk in ranks:
            jobs.append((f"skv_decode_partial_paged_q{bits}_rk{rk}.o",
                         ["-x", "hip", os.path.join(CSRC, "skv_decode_partial.hip"), f"-DSKV_RK={rk}",
                          f"-DSKV_QBITS={bits}", "-DSKV_PAGED=1"], DEVICE_FLAGS + DECODE_FLAGS))
    for rk in Q4_KEY_RANKS:
        jobs.append((f"skv_decode_partial_q4_rk{rk}.o",
                     ["-x", "hip", os.path.join(CSRC, "skv_decode_partial.hip"), f"-DSKV_RK={rk}", "-DSKV_QBITS=4"],
                     DEVICE_FLAGS + DECODE_FLAGS))
    return jobs


def _up_to_date(out: str, cmd_line: str) -> bool:
    """True if the object exists, was made by the same command and is newer than every file it was made from
    (as listed by the compiler's dependency output)."""
    dep, tag = out + ".d", out + ".cmd"
    if not (os.path.exists(out) and os.path.exists(dep) and os.path.exists(tag)):
        return False
    with open(tag) as f:
        if f.read() != cmd_line:
            return False
    with open(dep) as f:
        words = f.read().replace("\\\n", " ").split()
    t = os.path.getmtime(out)
    for w in words:
        if w.endswith(":"):
            continue
        if not os.path.exists(w) or os.path.getmtime(w) > t:
            return False
    return True


def build(verbose: bool = True, workers: int | None = None, incremental: bool = False) -> str:
    """Compiles every source and links the libraries.  incremental: objects whose sources, headers and
    command line have not changed since they were made are kept (a developer's shortcut; the default
    compiles everything)."""
    hipcc = _hipcc()
    os.makedirs(BUILD_DIR, exist_ok=True)
    workers = workers or min(8, os.cpu_count() or 1)

    def compile_one(job):
        obj, src_args, extra = job
        out = os.path.join(BUILD_DIR, obj)
        cmd = [hipcc, "-c", *COMMON, *extra, *src_args, "-MD", "-MF", out + ".d", "-o", out]
        if incremental and _up_to_date(out, " ".join(cmd)):
            if verbose:
                print(f"[build] {obj} (up to date)", flush=True)
            return out
        if os.path.exists(out + ".cmd"):
            os.remove(out + ".cmd")
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
        with open(out + ".cmd", "w") as f:
            f.write(" ".join(cmd))
        if verbose:
            err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
            print(f"[build] {obj}" + (f"\n{err}" if err else ""), flush=True)
        return out

    with ThreadPoolExecutor(max_workers=workers) as ex:
        objs = list(ex.map(compile_one, _jobs()))
    probe_objs = [o for o in objs if os.path.basename(o) == "skv_probe.o"]
    objs = [o for o in objs if o not in probe_objs]
    for out, members in ((OUT, objs), (PROBE_OUT, probe_objs)):
        cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out, *members]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"link failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
        if verbose:
            print(f"[build] linked {out}", flush=True)
    return OUT


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    sys.exit(0)
