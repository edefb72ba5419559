"""Builds paper_1603_05279_amd/libxnor.so from csrc/*.hip for gfx950 with hipcc.

Every source is compiled to an object of its own (in parallel), then linked.  Only the `xnor_*` functions of
the C ABI are exported: everything else is built with hidden visibility.
"""
import concurrent.futures
import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libxnor.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fvisibility=hidden", "-fvisibility-inlines-hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-Wall", "-Wno-unused-command-line-argument",
]
NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers_mtime():
    hs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return max(os.path.getmtime(h) for h in hs)


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if NOISE not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + err)
    return err


def build(verbose: bool = False, incremental: bool = False, extra_flags=(), lib: str = LIB, jobs: int = 8) -> str:
    """Compiles every source (incremental=True: only those older than their object) and links `lib`."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tag = "".join(c if c.isalnum() else "_" for c in " ".join(extra_flags))
    objdir = os.path.join(OBJ, tag or "default")
    os.makedirs(objdir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    hdr = _headers_mtime()
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = incremental and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), hdr)
        if not fresh:
            todo.append([hipcc] + HIPCC_FLAGS + list(extra_flags) + inc + ["-c", src, "-o", obj])
    with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        for cmd, err in zip(todo, ex.map(_run, todo)):
            if verbose:
                print(" ".join(cmd))
                if err.strip():
                    print(err)
    err = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument",
                "-Wl,--version-script=" + os.path.join(CSRC, "libxnor.map")] + objs + ["-o", lib])
    if verbose and err.strip():
        print(err)
    return lib


def build_host_ubsan(lib: str) -> str:
    """libxnor with the host code of csrc/api.hip (argument validation and dispatch of every entry point)
    instrumented by UndefinedBehaviorSanitizer, the other objects as built by build(): for the ABI tests that
    run on the CPU.  Device code is never instrumented."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(OBJ, "default")
    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in sources()]
    if not all(os.path.exists(o) for o in objs):
        build()
    # trap mode: a finding executes a trap instruction (the process dies with SIGILL) and no sanitizer runtime has
    # to be linked into the shared library
    san = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined"]
    api_obj = os.path.join(OBJ, "api_ubsan.o")
    _run([hipcc] + HIPCC_FLAGS + san + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
                                         os.path.join(CSRC, "api.hip"), "-o", api_obj])
    objs = [api_obj if os.path.basename(o) == "api.o" else o for o in objs]
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument",
          "-Wl,--version-script=" + os.path.join(CSRC, "libxnor.map")] + objs + ["-o", lib])
    return lib


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
