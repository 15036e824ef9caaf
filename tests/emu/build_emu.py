"""TEST INFRASTRUCTURE ONLY: compiles the library's kernel sources against the CPU stand-in for the HIP
runtime (tests/emu/hip/hip_runtime.h) with AddressSanitizer and UBSan, into tests/emu/_build/<tag>/emu_driver.

Three builds: "default" (the library's own size thresholds: small tensors take the tile search),
"streaming" (thresholds lowered so that tiny tensors take the streaming search, for bf16 the value
table, and from 2048 elements on the large-tensor forms of quantize+pack and unpack+dequantize) and "streaming_c2f" (as "streaming", plus the coarse-to-fine sweeps on the streaming kernel, which the
library itself never launches).  Returns None when no host clang++ with C++20 is available."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2211_04515_amd", "csrc")
VARIANTS = {
    "default": [],
    "streaming": ["-DQP_TILE_SEARCH_MAX_N=0", "-DQP_VALUE_TABLE_MIN_N=4096", "-DQP_SEARCH_FILL_BLOCKS=8",
                  "-DQP_LARGE_FORMS_MIN_N=2048"],
    # as "streaming", and a coarse-to-fine search runs its two sweeps on the streaming kernel: the sequence that
    # the library refuses because its only GPU run faulted (the macro exists for this build alone)
    "streaming_c2f": ["-DQP_TILE_SEARCH_MAX_N=0", "-DQP_VALUE_TABLE_MIN_N=4096", "-DQP_SEARCH_FILL_BLOCKS=8",
                      "-DQP_LARGE_FORMS_MIN_N=2048", "-DQP_EMULATE_STREAMING_C2F=1"],
}


def find_cxx():
    for c in ("/opt/rocm/llvm/bin/clang++", shutil.which("clang++")):
        if c and os.path.exists(c):
            return c
    return None


def build(tag: str):
    cxx = find_cxx()
    if cxx is None:
        return None
    out = os.path.join(HERE, "_build", tag)
    os.makedirs(out, exist_ok=True)
    flags = ["-std=c++20", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer", "-ffp-contract=off", "-pthread", "-Wno-unused-value",
             "-I", HERE, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *VARIANTS[tag]]
    units = [(s, ["-x", "c++"]) for s in sorted(glob.glob(os.path.join(CSRC, "*.hip")))]
    units += [(os.path.join(HERE, "emu_rt.cpp"), []), (os.path.join(HERE, "emu_driver.cpp"), [])]

    def cc(unit):
        src, lang = unit
        obj = os.path.join(out, os.path.basename(src) + ".o")
        subprocess.run([cxx, *flags, *lang, "-c", src, "-o", obj], check=True, capture_output=True)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(cc, units))
    exe = os.path.join(out, "emu_driver")
    subprocess.run([cxx, *flags, *objs, "-o", exe], check=True, capture_output=True)
    return exe


def build_all():
    """Both builds at once: {tag: path or None}."""
    with ThreadPoolExecutor(max_workers=len(VARIANTS)) as ex:
        return dict(zip(VARIANTS, ex.map(build, VARIANTS)))


if __name__ == "__main__":
    print(build_all())
