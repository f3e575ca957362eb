"""Compile the CPU oracle (plain C, OpenMP) into oracle/liblsp_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lsp_oracle.c")
LIB = os.path.join(HERE, "liblsp_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized(out_dir: str) -> tuple[str, str]:
    """The oracle's own driver (oracle/sanitize_driver.c, which includes lsp_oracle.c)
    as two executables in out_dir: one plain, one under -fsanitize=address,undefined.
    Returns (plain, sanitized)."""
    drv = os.path.join(HERE, "sanitize_driver.c")
    plain, san = os.path.join(out_dir, "oracle_driver"), os.path.join(out_dir, "oracle_driver_asan")
    base = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-Wall", "-Wextra", "-I", HERE, drv, "-lm"]
    subprocess.run(base + ["-o", plain], check=True)
    subprocess.run(base + ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", san],
                   check=True)
    return plain, san


if __name__ == "__main__":
    print(build())
