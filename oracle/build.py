"""Compile the C oracle into two shared objects next to its source:
liboracle_f64.so (arithmetic in double, the parity reference) and
liboracle_f32.so (same source with float arithmetic).

Test infrastructure only; nothing in the HIP library depends on it."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "neox_block_oracle.c")
VARIANTS = {"f64": "double", "f32": "float"}


def lib_path(variant: str) -> str:
    return os.path.join(HERE, f"liboracle_{variant}.so")


def build(force: bool = False) -> None:
    for variant, ctype in VARIANTS.items():
        out = lib_path(variant)
        if (not force and os.path.exists(out)
                and os.path.getmtime(out) >= os.path.getmtime(SRC)):
            continue
        # -ffp-contract=off / no fast-math: keep the arithmetic exactly as written
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", f"-DORACLE_REAL={ctype}", SRC, "-o", out, "-lm"]
        subprocess.check_call(cmd)


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    print("built", [lib_path(v) for v in VARIANTS])
