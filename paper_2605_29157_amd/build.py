"""Build the gfx950 HIP library (C ABI in include/parallax.h) in-tree with hipcc."""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_PATH = os.path.join(PKG, "libparallax_hip.so")
BUILD_DIR = os.path.join(ROOT, "_build")

SOURCES = ["parallax_api.hip", "decode_bf16.hip", "decode_mla_bf16.hip", "decode_mla_wide_bf16.hip", "prefill_bf16.hip", "prefill_bwd_bf16.hip",
           "generic_f32.hip", "norm_rope.hip", "util_kernels.hip"]

# packed-fp32 instructions are disabled for all device code (hipcc's host pass prints a
# harmless "not a recognized feature" note for the flag)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build the Parallax HIP library")
    return exe


def _device_asm_path(src: str) -> str:
    """Device assembly that hipcc leaves next to the object when asked to keep its temporaries."""
    return os.path.join(BUILD_DIR, os.path.splitext(src)[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s")


def _compile(src: str, extra: list[str]) -> str:
    """Compile one source to an object. The intermediate files are kept, so that the assembly
    checks below read the device code of THIS compile, the one that is linked."""
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "--save-temps=obj", "-c",
           os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, log))
    if log.strip():
        print(log)
    return obj


def _check_pipelined_assembly(src: str, full: bool) -> None:
    """Verify the hand-placed assembly of a kernel file on the device code that was linked."""
    from . import asm_check
    asm = _device_asm_path(src)
    if full:  # prefill forward: also its unguarded score MFMAs
        asm_check.check_file(asm)
        return
    with open(asm) as f:
        text = f.read()
    bad = (asm_check.find_early_reads_of_asm_mfma_results(text)
           + asm_check.find_m0_uses_outside_inline_asm(text)
           + asm_check.find_foreign_uses_of_asm_loaded_registers(text))
    if bad:
        raise RuntimeError("hazard in %s:\n  %s" % (asm, "\n  ".join(bad[:20])))


def _check_decode_assembly() -> None:
    """The bf16 decode kernel sits at the 256-register limit of two workgroups per compute
    unit; one spilled register costs it 10 %. Fail the build if any decode kernel spills."""
    import re
    with open(_device_asm_path("decode_bf16.hip")) as f:
        text = f.read()
    spills = {}
    for block in text.split("  - .agpr_count")[1:]:
        name = re.search(r"\.name:\s+(\S+)", block).group(1)
        if "decode_bf16_kernel" in name:
            spills[name] = int(re.search(r"\.vgpr_spill_count:\s+(\d+)", block).group(1))
    # (the instantiations that normalise and rotate q, rho first -- last template flag set -- may
    # park a few registers around that prologue: the paged one does, 9 of them, which costs it
    # 6 us of a 38 us step; with 50 and more spilled, as a first form of that prologue had, the
    # reloads queue up behind the tile loads and the step takes half as long again)
    prep = "Lb1EEEvNS_12DecodeParamsE"
    bad = {n: c for n, c in spills.items() if c > (16 if n.endswith(prep) else 0)}
    if not spills or bad:
        raise RuntimeError("decode_bf16.hip: register spills in a decode kernel (%s)" % bad)


def build_library(extra_flags: list[str] | None = None, verbose: bool = True) -> str:
    """Compile every kernel file for gfx950 and link libparallax_hip.so next to this file."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    extra = list(extra_flags or [])
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objs = list(pool.map(lambda src: _compile(src, extra), SOURCES))
    _check_pipelined_assembly("prefill_bf16.hip", True)
    _check_pipelined_assembly("prefill_bwd_bf16.hip", False)
    _check_pipelined_assembly("decode_mla_bf16.hip", False)
    _check_pipelined_assembly("decode_mla_wide_bf16.hip", False)
    _check_decode_assembly()
    tmp = LIB_PATH + ".tmp%d" % os.getpid()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout)
    os.replace(tmp, LIB_PATH)
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
