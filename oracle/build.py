"""Compile the CPU oracle (test infrastructure) into two shared libraries:
liboracle_f32.so (the arithmetic the GPU path is compared with) and
liboracle_f64.so (same source in double, for gradient checks and noise floors)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sgns_oracle.c")


def lib_path(real: str) -> str:
    return os.path.join(HERE, f"liboracle_{'f32' if real == 'float' else 'f64'}.so")


def build(force: bool = False) -> None:
    for real in ("float", "double"):
        out = lib_path(real)
        if (not force and os.path.exists(out)
                and os.path.getmtime(out) >= os.path.getmtime(SRC)):
            continue
        # linked under another name and moved into place: a process that has the old library mapped keeps it
        tmp = f"{out}.{os.getpid()}.tmp"
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall",
               "-shared", "-fPIC", f"-DREAL={real}", SRC, "-o", tmp, "-lm"]
        subprocess.check_call(cmd)
        os.replace(tmp, out)


if __name__ == "__main__":
    build(force=True)
    print("oracle built")
