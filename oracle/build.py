"""Build the CPU oracle (test infrastructure) with gcc: an fp32 library and its fp64 twin."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fg_oracle.c")
LIBS = {"f32": ("liboracle_f32.so", "float"), "f64": ("liboracle_f64.so", "double")}


def lib_path(kind):
    return os.path.join(HERE, LIBS[kind][0])


def build(force=True):
    for kind, (name, ctype) in LIBS.items():
        out = os.path.join(HERE, name)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-fno-fast-math", "-shared",
               "-fPIC", "-std=c11", "-Wall", f"-DORC_REAL={ctype}", SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build()
    print("built", [lib_path(k) for k in LIBS])
