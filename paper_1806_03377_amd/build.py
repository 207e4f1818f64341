"""Builds the HIP/C++ sources under csrc/ into libpd.so next to this file (gfx950 only)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpd.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions (v_pk_*_f32)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def build(verbose: bool = True) -> str:
    objs = []
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in sources():
        obj = os.path.join(build_dir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [HIPCC, "-x", "hip", "-c", src, "-o", obj] + [f for f in FLAGS if f != "-shared"]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] FAILED {src}\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"[build] {os.path.basename(src)}:\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    if verbose:
        sys.stderr.write(f"[build] wrote {LIB}\n")
    return LIB


def build_host_sanitized(verbose: bool = False) -> str:
    """The host side of the runtime (pd_runtime.cpp, pd_partition.cpp) compiled with AddressSanitizer and
    UndefinedBehaviorSanitizer on the host pass only, linked with the ordinary kernel objects and the host-only driver
    tests/host/sanitize_main.cpp into _build/host_sanitize.  The driver calls nothing that touches a GPU."""
    build_dir = os.path.join(HERE, "_build")
    if not all(os.path.exists(os.path.join(build_dir, os.path.basename(s) + ".o")) for s in sources()):
        build(verbose)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    flags = [f for f in FLAGS if f not in ("-shared", "-O3")] + ["-O1"] + san
    main_src = os.path.join(os.path.dirname(HERE), "tests", "host", "sanitize_main.cpp")
    objs, procs = [], []
    for src in sources():
        base = os.path.basename(src)
        if src.endswith(".cpp"):
            obj = os.path.join(build_dir, base + ".san.o")
            procs.append((src, subprocess.Popen([HIPCC, "-x", "hip", "-c", src, "-o", obj] + flags,
                                                stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        else:
            obj = os.path.join(build_dir, base + ".o")
        objs.append(obj)
    main_obj = os.path.join(build_dir, "sanitize_main.san.o")
    procs.append((main_src, subprocess.Popen([HIPCC, "-x", "hip", "-c", main_src, "-o", main_obj] + flags,
                                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    exe = os.path.join(build_dir, "host_sanitize")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, main_obj] + objs,
                   check=True)
    return exe


if __name__ == "__main__":
    build()
