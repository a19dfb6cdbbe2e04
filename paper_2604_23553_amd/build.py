"""Builds the C-ABI HIP library in-tree for gfx950, twice from the same sources:

    libcfpp.so          the product (include/cfpp.h)
    libcfpp_profile.so  the profiling build (-DCFPP_PROFILE: kernel timeline tracer,
                        skip bits, test taps, calibration kernels; include/cfpp_profile.h)

    python -m paper_2604_23553_amd.build [--force] [--keep-temps]
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcfpp.so")
LIB_PROFILE = os.path.join(PKG, "libcfpp_profile.so")
SOURCES = ["api.hip", "decode_kernels.hip", "fused_kernel.hip", "lm_kernels.hip", "batched_kernels.hip",
           "prep_kernels.hip", "prefill_kernels.hip"]
HEADERS = ["layout.h", "device_utils.h", "decode_params.h", "attention_common.h", "decode_blocks.h",
           "attention_blocks.h", "lm_params.h", "batched_params.h", "prefill_params.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _stale() -> bool:
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS if os.path.exists(os.path.join(CSRC, s))]
    deps += [os.path.join(ROOT, "include", "cfpp.h"), os.path.join(ROOT, "include", "cfpp_profile.h"),
             os.path.abspath(__file__)]
    for lib in (LIB, LIB_PROFILE):
        if not os.path.exists(lib):
            return True
        t = os.path.getmtime(lib)
        if any(os.path.getmtime(d) > t for d in deps):
            return True
    return False


def build(force: bool = False, extra_flags=()) -> str:
    if not force and not _stale():
        return LIB
    variants = [(LIB, "", []), (LIB_PROFILE, "_profile", ["-DCFPP_PROFILE"])]
    procs, objs = [], {LIB: [], LIB_PROFILE: []}
    for lib, suffix, defs in variants:
        for s in SOURCES:
            obj = os.path.join(CSRC, s.replace(".hip", suffix + ".o"))
            cmd = ["hipcc", *HIPCC_FLAGS, *defs, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                   "-c", os.path.join(CSRC, s), "-o", obj]
            procs.append((cmd, subprocess.Popen(cmd, cwd=CSRC)))
            objs[lib].append(obj)
    for cmd, p in procs:
        if p.wait() != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
    for lib, _, _ in variants:
        # -Bsymbolic: each library calls its own functions even when both are loaded in one process
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-Bsymbolic", *objs[lib],
                               "-o", lib])
    return LIB


if __name__ == "__main__":
    extra = ["-save-temps"] if "--keep-temps" in sys.argv else []
    print(build(force="--force" in sys.argv or bool(extra), extra_flags=extra))
