"""Builds libyoco.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libyoco.so")
STAMP = os.path.join(PKG, "libyoco.stamp")      # hash of the sources the library was built from
SOURCES = ["yoco_api.hip", "attn_generic.hip", "swa_mfma.hip", "decode_bf16.hip", "gret_generic.hip", "gret_chunk.hip", "cache_i8.hip", "ceilings.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
         "-fno-honor-nans",        # fmax without NaN canonicalisation; -inf (the mask value) is still honoured
         "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def source_hash():
    """SHA-256 over every file the library is compiled from (sources, headers, the public header) and the flags."""
    import hashlib
    h = hashlib.sha256(" ".join(f for f in FLAGS if not f.startswith("-I")).encode())
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    for path in files + [os.path.join(ROOT, "include", "yoco.h")]:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_current():
    """True if libyoco.so exists and was built from the sources as they are now."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return False
    with open(STAMP) as f:
        return f.read().strip() == source_hash()


def build_lib(verbose=False):
    """Compile every translation unit and link the shared library in-tree."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    cmd = ["hipcc", "-shared", "-o", LIB] + objs + ["--offload-arch=gfx950"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stdout)
    with open(STAMP, "w") as f:
        f.write(source_hash() + "\n")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
