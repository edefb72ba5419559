"""Compile the C oracle into oracle/libxnor_oracle.so with gcc (test infrastructure only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "xnor_oracle.c")
LIB = os.path.join(HERE, "libxnor_oracle.so")
LIB_UBSAN = os.path.join(HERE, "libxnor_oracle_ubsan.so")
CHECK_SRC = os.path.join(HERE, "sanitize_check.c")


def build(force: bool = True, sanitize: bool = False) -> str:
    """The oracle library; sanitize=True builds the variant instrumented with UndefinedBehaviorSanitizer
    (aborting on the first finding), which loads into an ordinary Python process."""
    lib = LIB_UBSAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    opt = ["-O1", "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"] if sanitize else ["-O3"]
    cmd = ["gcc"] + opt + ["-fopenmp", "-ffp-contract=off", "-std=c11", "-Wall", "-Wextra",
                           "-shared", "-fPIC", SRC, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


def build_sanitize_check(exe: str) -> str:
    """oracle/sanitize_check.c + the oracle under AddressSanitizer and UndefinedBehaviorSanitizer, as one
    executable (AddressSanitizer cannot be loaded into an uninstrumented Python)."""
    cmd = ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp",
           "-ffp-contract=off", "-std=c11", "-Wall", CHECK_SRC, SRC, "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build())
