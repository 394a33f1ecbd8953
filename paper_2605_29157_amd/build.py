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

SOURCES = ["parallax_api.hip", "decode_bf16.hip", "decode_mla_bf16.hip", "prefill_bf16.hip", "prefill_bwd_bf16.hip",
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


def _compile(src: str, extra: list[str]) -> str:
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-c",
           os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, log))
    if log.strip():
        print(log)
    return obj


def _check_prefill_assembly(extra: list[str], src: str = "prefill_bf16.hip", m0: bool = True) -> None:  # m0: full check
    """Emit the device assembly of a prefill kernel file and verify its hand-placed MFMAs."""
    from . import asm_check
    asm = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".gfx950.s")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-S",
           "--cuda-device-only", os.path.join(CSRC, src), "-o", asm]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc -S failed on %s:\n%s" % (src, res.stdout))
    if m0:
        asm_check.check_file(asm)
    else:  # the backward kernels use guarded assembly MFMAs only (nothing "unguarded" to find)
        with open(asm) as f:
            text = f.read()
        bad = (asm_check.find_early_reads_of_asm_mfma_results(text)
               + asm_check.find_m0_uses_outside_inline_asm(text)
               + asm_check.find_foreign_uses_of_asm_loaded_registers(text))
        if bad:
            raise RuntimeError("hazard in %s:\n  %s" % (asm, "\n  ".join(bad[:20])))


def _check_decode_assembly(extra: list[str]) -> None:
    """The bf16 decode kernel sits at the 256-register limit of two workgroups per compute
    unit; one spilled register costs it 10 %. Fail the build if any decode kernel spills."""
    import re
    asm = os.path.join(BUILD_DIR, "decode_bf16.gfx950.s")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-S",
           "--cuda-device-only", os.path.join(CSRC, "decode_bf16.hip"), "-o", asm]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc -S failed on decode_bf16.hip:\n" + res.stdout)
    with open(asm) as f:
        text = f.read()
    spills = re.findall(r"\.vgpr_spill_count:\s+(\d+)", text)
    if not spills or any(int(n) for n in spills):
        raise RuntimeError("decode_bf16.hip: register spills in a decode kernel (%s)" % spills)


def build_library(extra_flags: list[str] | None = None, verbose: bool = True) -> str:
    """Compile every kernel file for gfx950 and link libparallax_hip.so next to this file."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    extra = list(extra_flags or [])
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES) + 3) as pool:
        checks = [pool.submit(_check_prefill_assembly, extra),
                  pool.submit(_check_prefill_assembly, extra, "prefill_bwd_bf16.hip", False),
                  pool.submit(_check_prefill_assembly, extra, "decode_mla_bf16.hip", False),
                  pool.submit(_check_decode_assembly, extra)]
        objs = list(pool.map(lambda s: _compile(s, extra), SOURCES))
        for c in checks:
            c.result()
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
