"""Builds the native library in-tree with hipcc for gfx950.

    python -m paper_2507_20424_amd.build
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
# one translation unit per family of kernels, so that they compile side by side
UNITS = ["dppf_api", "dppf_launch_reduce", "dppf_launch_step_reduce", "dppf_launch_update", "dppf_launch_seq",
         "dppf_launch_adamw", "dppf_launch_misc", "dppf_launch_any", "dppf_launch_lds"]
OBJ_DIR = os.path.join(CSRC, "_build")
LIB = os.path.join(CSRC, "libdppf.so")
CLI_SRC = os.path.join(PKG_DIR, "csrc", "dppf_cli.c")
CLI = os.path.join(PKG_DIR, "csrc", "dppf_cli")
INCLUDE = os.path.join(ROOT, "include")
LAST_KERNEL_RESOURCES = []     # filled by build_library: one dict per kernel

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unused-function",
    # one remark block per kernel with its register, LDS and scratch use (parsed below)
    "-Rpass-analysis=kernel-resource-usage",
]


def hipcc_path() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the DPPF library needs the ROCm toolchain")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + res.stdout)
    return res.stdout


_REMARK = re.compile(r"remark: .*?(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"LDS Size \[bytes/block\]): (\S+)")


def kernel_resources(compiler_output: str):
    """[{name, vgprs, agprs, scratch, occupancy, lds}] from the compiler's kernel-resource-usage remarks."""
    kernels, cur = [], None
    for line in compiler_output.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = {"name": val}
            kernels.append(cur)
        elif cur is not None:
            cur[{"VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch",
                 "Occupancy [waves/SIMD]": "occupancy", "LDS Size [bytes/block]": "lds"}[key]] = int(val)
    return kernels


def _without_remarks(compiler_output: str) -> str:
    keep, skip = [], 0
    for line in compiler_output.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in line:
            skip = 2                     # the remark is followed by the source line and a caret line
            while keep and keep[-1].startswith("In file included from"):
                keep.pop()               # and preceded by its include chain
            continue
        if skip and re.match(r"^\s*(\d+\s*)?\|", line):
            skip -= 1
            continue
        skip = 0
        if "packed-fp32-ops" not in line and not re.match(r"^\d+ (warning|remark)s? generated", line):
            keep.append(line)
    return "\n".join(keep)


def compile_unit(name: str, extra_flags=(), verbose: bool = True) -> str:
    """hipcc -c one translation unit of csrc/ into csrc/_build/; returns the compiler's output."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-I", CSRC, "-c", "-o",
           os.path.join(OBJ_DIR, name + ".o"), os.path.join(CSRC, name + ".hip")]
    return _run(cmd, verbose)


def build_library(verbose: bool = True, jobs: int = 8) -> str:
    """Compile every unit of csrc/ (always recompiles) and link them into csrc/libdppf.so.
    Fails if any kernel spills registers to scratch memory: every kernel is meant to run out of
    registers and LDS alone."""
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(UNITS)))) as pool:
        outs = list(pool.map(lambda u: compile_unit(u, verbose=verbose), UNITS))
    kernels = []
    for unit, out in zip(UNITS, outs):
        rest = _without_remarks(out)
        if verbose and rest.strip():
            print(rest)
        found = kernel_resources(out)
        for k in found:
            k["unit"] = unit
        kernels += found
    if not kernels:
        raise RuntimeError("the compiler reported no kernels: is -Rpass-analysis=kernel-resource-usage still understood?")
    spilled = [k for k in kernels if k.get("scratch", 0) > 0]
    if spilled:
        raise RuntimeError("kernels with scratch spills:\n" + "\n".join(
            f"  {k['unit']}: {k['name']}: {k['scratch']} bytes/lane" for k in spilled))
    if verbose:
        print(f"{len(kernels)} kernels, none spills to scratch; most registers: "
              f"{max(k.get('vgprs', 0) + k.get('agprs', 0) for k in kernels)}")
    global LAST_KERNEL_RESOURCES
    LAST_KERNEL_RESOURCES = kernels
    objs = [os.path.join(OBJ_DIR, u + ".o") for u in UNITS]
    out = _run([hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument",
                "-o", LIB + ".tmp", *objs], verbose)
    if verbose and out.strip():
        print(out)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_cli(verbose: bool = True) -> str:
    """Compile csrc/dppf_cli.c -- plain C against the C ABI and the HIP runtime API -- with gcc."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    gcc = shutil.which("gcc") or "gcc"
    cmd = [gcc, "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", INCLUDE, "-o", CLI + ".tmp", CLI_SRC, "-L", os.path.dirname(LIB), "-ldppf",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout)
    if verbose and res.stdout.strip():
        print(res.stdout)
    os.replace(CLI + ".tmp", CLI)
    return CLI


def build_all(verbose: bool = True) -> None:
    build_library(verbose)
    build_cli(verbose)


if __name__ == "__main__":
    build_all()
    sys.exit(0)
