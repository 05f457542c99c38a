"""Build libw2l.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_1812_07625_amd.build             # compile what changed, link
    python -m paper_1812_07625_amd.build --force     # recompile everything
    python -m paper_1812_07625_amd.build --sanitize  # libw2l_san.so: host code under ASan + UBSan
                                                     # (for the host-side tests; device code unchanged)
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libw2l.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-pass-failed",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _deps_mtime():
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hdrs.append(os.path.join(HERE, "..", "include", "w2l.h"))
    return max(os.path.getmtime(h) for h in hdrs)


# host-side sanitizers: each -fsanitize= directly after -Xarch_host, so the device pass never sees it
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
SAN_OBJDIR = os.path.join(HERE, "_build", "san")
SAN_LIB = os.path.join(HERE, "libw2l_san.so")


def _compile(src, force, sanitize=False):
    obj = os.path.join(SAN_OBJDIR if sanitize else OBJDIR, os.path.basename(src)[:-4] + ".o")
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) > max(os.path.getmtime(src), _deps_mtime())):
        return obj
    cmd = [HIPCC] + FLAGS + (SAN_FLAGS if sanitize else []) + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if "warning" in warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(force: bool = False, jobs: int = 8, sanitize: bool = False) -> str:
    os.makedirs(SAN_OBJDIR if sanitize else OBJDIR, exist_ok=True)
    lib = SAN_LIB if sanitize else LIB
    srcs = _sources()
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, sanitize), srcs))
    if force or not os.path.exists(lib) or any(os.path.getmtime(o) > os.path.getmtime(lib) for o in objs):
        tmp = lib + ".tmp.%d" % os.getpid()
        link = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] if sanitize else []
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + link + ["-o", tmp] + objs,
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        os.replace(tmp, lib)
    return lib


def asan_runtime() -> str:
    """The shared AddressSanitizer runtime of hipcc's clang: to be preloaded into the Python process
    that loads libw2l_san.so."""
    r = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    if r.returncode != 0 or not os.path.isabs(path):
        raise RuntimeError("cannot locate clang's ASan runtime: " + r.stderr)
    return path


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, sanitize="--sanitize" in sys.argv))
