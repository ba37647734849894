"""Build libxyattn.so (host planner + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
import sys

try:
    from . import hazard_lint
except ImportError:          # run as a script
    import hazard_lint

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libxyattn.so")
SOURCES = ["plan.cpp", "serving.cpp", "attn_kernels.hip", "probe_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
STAMP = LIB + ".sources"        # digest of what the library was built from, written next to it


def sources_digest():
    """sha256 over everything the library is built from: the sources, every header they include, this script."""
    import glob
    import hashlib
    files = [os.path.join(CSRC, s) for s in SOURCES] + sorted(glob.glob(os.path.join(CSRC, "*.h"))) \
        + sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))) \
        + [os.path.abspath(__file__), os.path.join(PKG, "hazard_lint.py")]
    h = hashlib.sha256()
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def is_current():
    """Whether the library that is there was built from the sources that are there."""
    try:
        with open(STAMP) as f:
            return os.path.exists(LIB) and f.read().strip() == sources_digest()
    except OSError:
        return False


def _scratch_report(remarks):
    """{kernel name: scratch bytes per lane} from the compiler's kernel-resource-usage remarks."""
    out, name = {}, None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name is not None:
            out[name] = int(m.group(1))
    return out


def build(verbose=False):
    if os.path.exists(STAMP):
        os.remove(STAMP)        # written again only behind a library that passed every check
    cmd = [HIPCC, "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB + ".tmp"
    cmd += ["-o", tmp, "-Rpass-analysis=kernel-resource-usage"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        if os.path.exists(LIB):
            os.remove(LIB)      # never leave a stale library behind a failed build
        raise RuntimeError("hipcc failed:\n" + err)
    # The attention kernel requests LDS fragments and issues MFMAs by hand; the compiler does not know
    # when their results arrive, so a register spilled right behind such an instruction would be saved
    # before it holds its value.  No kernel of this library may use scratch memory.
    spills = _scratch_report(err)
    if any(size for size in spills.values()):
        if os.path.exists(LIB):
            os.remove(LIB)
        os.remove(tmp)
        raise RuntimeError(f"a kernel uses scratch memory (bytes per lane: {spills}); refusing to install the library")
    # the device sources once more as assembly text, for the check of the hand-issued instructions
    for source in (s for s in SOURCES if s.endswith(".hip")):
        asm_cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
                   "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
                   "-o", "-", os.path.join(CSRC, source)]
        asm = subprocess.run(asm_cmd, capture_output=True, text=True)
        if asm.returncode != 0:
            os.remove(tmp)
            raise RuntimeError("hipcc -S failed:\n" + asm.stderr)
        problems = hazard_lint.lint(asm.stdout)
        if problems:
            if os.path.exists(LIB):
                os.remove(LIB)
            os.remove(tmp)
            raise RuntimeError(f"hazards around hand-issued instructions in {source}:\n" +
                               "\n".join(f"  line {n}: {m}" for n, m in problems))
    os.replace(tmp, LIB)
    with open(STAMP, "w") as f:
        f.write(sources_digest() + "\n")
    if verbose:
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
