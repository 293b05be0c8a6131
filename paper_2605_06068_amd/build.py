"""Builds libpa_decode.so from csrc/ with hipcc for gfx950 (cross-compiles without a GPU).

Two passes per source file: the device pass compiles the kernels with packed-fp32 VALU
instructions switched off (a target feature only the gfx950 back end knows), the host pass
compiles the launch code and embeds the device pass's code-object bundle.  One pass with the
switch on the command line builds the same library but has the host back end print a warning
about a feature it does not know.
"""
from __future__ import annotations

import hashlib
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_PKG, "libpa_decode.so")

ARCH = "--offload-arch=gfx950"
COMMON_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wextra", "-Wno-unused-parameter"]
# keep the compiler from forming v_pk_add_f32 / v_pk_mul_f32 / v_pk_fma_f32
DEVICE_ONLY_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]


def source_digest() -> str:
    """SHA-256 over the kernel sources and the public header (names and contents): identifies the
    code a built library, or a measurement, belongs to."""
    h = hashlib.sha256()
    for d, names in ((CSRC, sorted(os.listdir(CSRC))), (INCLUDE, ["pa_decode.h"])):
        for f in names:
            if f.endswith((".hip", ".hpp", ".h")):
                h.update(f.encode())
                with open(os.path.join(d, f), "rb") as fh:
                    h.update(fh.read())
    return h.hexdigest()


def hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def device_asm(extra_flags=()) -> str:
    """The gfx950 assembly of every kernel, as the device pass of build() generates it (for checks
    of what the compiler emitted; nothing is linked)."""
    out = []
    for src in sources():
        out.append(subprocess.check_output(
            [hipcc(), ARCH, *COMMON_FLAGS, *DEVICE_ONLY_FLAGS, *extra_flags, "--cuda-device-only", "-S",
             f"-DPA_SOURCE_DIGEST=\"{source_digest()}\"", f"-I{INCLUDE}", f"-I{CSRC}", "-o", "-", src],
            stderr=subprocess.DEVNULL).decode())
    return "\n".join(out)


def build(force: bool = True, verbose: bool = False, extra_flags=()) -> str:
    """Compile the library in-tree.  ``force=False`` rebuilds only when the built library does not
    carry the digest of the present sources."""
    if not force and built_digest() == source_digest():
        return LIB_PATH
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    objs = []
    defs = [f"-DPA_SOURCE_DIGEST=\"{source_digest()}\"", f"-I{INCLUDE}", f"-I{CSRC}"]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    try:
        for i, src in enumerate(sources()):
            bundle, obj = f"{tmp}.{i}.hipfb", f"{tmp}.{i}.o"
            objs += [bundle, obj]
            run([hipcc(), ARCH, *COMMON_FLAGS, *DEVICE_ONLY_FLAGS, *extra_flags, *defs, "--cuda-device-only",
                 "-o", bundle, src])
            run([hipcc(), ARCH, *COMMON_FLAGS, *extra_flags, *defs, "--cuda-host-only", "-Xclang",
                 "-fcuda-include-gpubinary", "-Xclang", bundle, "-c", "-o", obj, src])
        run([hipcc(), "-shared", "-fPIC", "-o", tmp, *[o for o in objs if o.endswith(".o")]])
        os.replace(tmp, LIB_PATH)
    finally:
        for f in objs + [tmp]:
            if os.path.exists(f):
                os.remove(f)
    return LIB_PATH


def built_digest():
    """The source digest the built library was compiled from (its pa_source_digest()), or None
    when there is no library or it predates that export."""
    if not os.path.exists(LIB_PATH):
        return None
    import ctypes

    try:
        fn = ctypes.CDLL(LIB_PATH).pa_source_digest
    except (OSError, AttributeError):
        return None
    fn.restype = ctypes.c_char_p
    return fn().decode()


if __name__ == "__main__":
    print(build(verbose=True))
