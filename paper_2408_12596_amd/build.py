"""Builds libpoplar.so in-tree with hipcc for gfx950.

    python -m paper_2408_12596_amd.build [--force]

Every source under csrc/ is compiled to an object (in parallel) and linked into
paper_2408_12596_amd/libpoplar.so.  Objects are rebuilt when their source or
any header is newer.
"""
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpoplar.so")

COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-munsafe-fp-atomics"]
# host numerics of the allocator must not be contracted into FMAs
HOST_ONLY = {"analysis.cpp": ["-ffp-contract=off"], "layout.cpp": []}


def _hipcc():
    for cand in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.isabs(cand) and os.path.exists(cand):
            return cand
    return "hipcc"


def _compile(src, force):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    deps = [src] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(HERE, "..", "include", "poplar.h"))
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj, None
    base = os.path.basename(src)
    cmd = [_hipcc()] + COMMON + HOST_ONLY.get(base, []) + ["-x", "hip", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {base}:\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    return obj, warn


def build(force=False, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))
    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        results = list(ex.map(lambda s: _compile(s, force), srcs))
    objs = [o for o, _ in results]
    if verbose:
        for _, w in results:
            if w:
                print(w)
    rebuilt = any(w is not None for _, w in results)
    if rebuilt or force or not os.path.exists(LIB):
        cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


HOST_ONLY_SOURCES = ["layout.cpp", "analysis.cpp"]
HOST_CHECK = os.path.join(OBJ, "host_check_san")


def build_host_sanitized():
    """The host-only part of the library (flat layout, shard arithmetic, speed curves, Algorithm 2, communication
    model) with its command-line driver csrc/host_check_main.cc, compiled for the host alone with AddressSanitizer and
    UndefinedBehaviorSanitizer (any finding aborts).  Returns the executable's path; tests/test_host_library.py runs it
    on the cases it gives the library and compares the outputs."""
    os.makedirs(OBJ, exist_ok=True)
    cmd = [_hipcc(), "-O1", "-g", "-std=c++17", "--offload-host-only", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
           "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all", "-ffp-contract=off", "-x", "hip"]
    cmd += [os.path.join(CSRC, f) for f in HOST_ONLY_SOURCES]
    cmd += ["-x", "c++", os.path.join(CSRC, "host_check_main.cc"), "-o", HOST_CHECK]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("sanitizer build of the host code failed:\n" + r.stderr)
    return HOST_CHECK


if __name__ == "__main__":
    if "--host-sanitize" in sys.argv:
        print(build_host_sanitized())
    else:
        print(build(force="--force" in sys.argv, verbose=True))
