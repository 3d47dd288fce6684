"""Compile the C oracle with gcc into oracle/libhyp_oracle_{f32,f64}.so."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "hyp_oracle.c"


def lib_path(real: str) -> pathlib.Path:
    return HERE / f"libhyp_oracle_{real}.so"


def build(force: bool = False) -> None:
    for real, ctype in (("f32", "float"), ("f64", "double")):
        out = lib_path(real)
        if not force and out.exists() and out.stat().st_mtime >= SRC.stat().st_mtime:
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               f"-DORACLE_REAL={ctype}", str(SRC), "-o", str(out), "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path("f32"), lib_path("f64"))
