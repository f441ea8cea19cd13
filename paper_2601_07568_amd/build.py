"""Builds the HIP library (libdllm.so) for gfx950 in-tree with hipcc, and the symbol list check."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdllm.so")
HEADER = os.path.join(os.path.dirname(HERE), "include", "dllm.h")
SOURCES = ["api.hip", "kernels_generic.hip", "kernels_skinny.hip", "kernels_attention.hip", "kernels_gemm.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-sanitize",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for p in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.exists(p) or p == "hipcc":
            return p
    return "hipcc"


# Kernels that wait on their own count of outstanding memory instructions (s_waitcnt vmcnt(n) against copies
# straight into LDS).  A spill to scratch between such a kernel's first and last copy would add instructions the
# count does not know (and stores may complete out of order with the loads), so the build looks at the generated code
# and refuses it.  Scratch traffic before the first copy or after the loop's final wait is harmless.
COUNTED = {"kernels_gemm.hip": ("k_gemm_t256", "k_gemm_ts"), "kernels_attention.hip": ("k_attn_dl",)}


def _check_counted_loops(src: str, asm: str) -> None:
    name, body = None, []
    def check():
        if name is None or not any(k in name for k in COUNTED[src]):
            return
        copies = [i for i, l in enumerate(body) if "global_load_lds" in l]
        if not copies:
            return
        for l in body[copies[0]:copies[-1] + 1]:
            if "scratch_" in l:
                raise RuntimeError(f"{src}: kernel {name} spills to scratch between its copies into LDS "
                                   f"({l.strip()}); its explicit memory-instruction counts do not allow that")
    for line in asm.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            check()
            name, body = m.group(1), []
        elif name is not None:
            body.append(line)
    check()


def build(verbose: bool = False) -> str:
    """Compiles every source (always, also when a built library exists) and links libdllm.so."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            errs = [l for l in err.splitlines() if "error" in l]
            raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(errs[:20] or err.splitlines()[-20:]))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    def check_one(src):
        asm = os.path.join(objdir, src.replace(".hip", ".s"))
        cmd = [_hipcc(), *FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", asm]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src}:\n" + r.stderr[-2000:])
        with open(asm) as f:
            _check_counted_loops(src, f.read())
        os.remove(asm)

    with ThreadPoolExecutor(max_workers=4) as ex:
        checks = [ex.submit(check_one, s) for s in srcs if s in COUNTED]
        objs = list(ex.map(compile_one, srcs))
        for c in checks:
            c.result()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


def build_host_check() -> str:
    """Sanitizer build of the host side of the library: every source compiled with AddressSanitizer and
    UndefinedBehaviorSanitizer on the HOST code only (device code as usual), linked with csrc/host_check_main.cpp into
    _build/host_check, an executable that drives every entry point's validation without a GPU."""
    objdir = os.path.join(HERE, "_build", "san")
    os.makedirs(objdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-g"]
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1"] + san

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o").replace(".cpp", ".o"))
        extra = ["-x", "hip"] if src.endswith(".cpp") else []
        r = subprocess.run([_hipcc(), *flags, "-c", *extra, os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src} (sanitizer build):\n" + r.stderr[-3000:])
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES + ["host_check_main.cpp"]))
    exe = os.path.join(HERE, "_build", "host_check")
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-fno-gpu-sanitize", "-Xarch_host", "-fsanitize=address",
                        "-Xarch_host", "-fsanitize=undefined", "-o", exe, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed (sanitizer build):\n" + r.stderr[-3000:])
    return exe


def declared_symbols() -> list[str]:
    """Names of the functions include/dllm.h declares."""
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dllm_[a-z_0-9]+)\s*\(", text)))


if __name__ == "__main__":
    print(build(verbose=True))
