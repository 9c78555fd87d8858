"""Builds libsdkde.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "sdkde.hip")]      # one translation unit; the kernels live in the headers
HEADERS = [os.path.join(ROOT, "include", "sdkde.h")] + [
    os.path.join(HERE, "csrc", name)
    for name in ("common.h", "prep.h", "pair_mfma.h", "pair_lds.h", "pair_sym.h", "pair_thin.h", "epilogue.h")]
LIBRARY = os.path.join(HERE, "libsdkde.so")
PEAKS_SOURCE = os.path.join(HERE, "csrc", "peaks.hip")
PEAKS_BINARY = os.path.join(HERE, "sdkde_peaks")     # micro-benchmark of the instruction rates that bound the kernels

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept off
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-mfma-vgpr-form",     # MFMA accumulators in VGPRs: no AGPR copies around VALU work
    "-Wno-unused-command-line-argument",
]


RECORD = LIBRARY + ".sources"       # digest of the sources and flags the library was built from


def source_digest() -> str:
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for path in SOURCES + HEADERS:
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when the library is missing or was built from other sources than the tree holds now (by content, so
    that a copy of the tree with fresh time stamps does not count as changed)."""
    if not os.path.exists(LIBRARY):
        return True
    if not os.path.exists(RECORD):
        return False        # a library without its record (copied on its own): nothing says it is out of date
    with open(RECORD) as f:
        return f.read().strip() != source_digest()


def kernels_using_scratch(remarks: str):
    """Names of kernels whose resource-usage remarks report a non-zero scratch size."""
    import re
    out, name = [], None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and int(m.group(1)) > 0 and name:
            out.append(name)
    return out


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; with force=False only when a source is newer than the binary."""
    if not force and not is_stale():
        return LIBRARY
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-I", os.path.join(ROOT, "include"),
           "-o", LIBRARY, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        lines = [ln for ln in proc.stdout.splitlines() if "remark:" not in ln]
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    spilled = kernels_using_scratch(proc.stdout)
    if spilled:
        os.remove(LIBRARY)
        raise RuntimeError("kernels spill registers to scratch memory (not allowed in this library): " + ", ".join(spilled))
    with open(RECORD, "w") as f:
        f.write(source_digest() + "\n")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    proc = subprocess.run([hipcc, *flags, "-o", PEAKS_BINARY, PEAKS_SOURCE], stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed (peaks):\n" + proc.stdout)
    return LIBRARY


if __name__ == "__main__":
    print(build(force=True, verbose=True))
