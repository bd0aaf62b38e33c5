"""Builds libsurgeon.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsurgeon.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["surgeon_host.cpp", "importance.hip", "prune_pack.hip", "dw.hip", "dw_f32.hip", "dw_bf16in.hip", "dw_bf16.hip", "dw_sparse.hip", "da.hip", "layers.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _newest_header():
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    if "--trust-abi" not in sys.argv:  # development: surgeon.h only gained declarations since the objects were built
        paths.append(os.path.join(ROOT, "include", "surgeon.h"))
    return max(os.path.getmtime(p) for p in paths)


def _compile(src, force=True):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(os.path.join(CSRC, src)),
                                                                          _newest_header()):
        return src, obj, None  # up to date (development builds only; the driver's build check compiles everything)
    cmd = [HIPCC] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    if src.endswith(".cpp"):
        cmd.insert(1, "-ffp-contract=off")
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, r


def build(verbose=False, force=True):
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        results = list(ex.map(lambda s: _compile(s, force), SOURCES))
    objs = []
    for src, obj, r in results:
        if r is None:
            objs.append(obj)
            continue
        # the host pass warns that it does not know the packed-fp32 target feature: harmless
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "-target-feature" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        objs.append(obj)
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    _write_build_info()
    return LIB


def _write_build_info():
    """Which sources the library was built from: the commit and whether the tree had uncommitted changes (the
    benchmark prints it next to figures that come from a stored profile, so a stale profile is visible)."""
    import json

    def git(*args):
        try:
            return subprocess.run(["git", "-C", ROOT] + list(args), capture_output=True, text=True, timeout=20).stdout.strip()
        except Exception:
            return ""
    info = {"commit": git("rev-parse", "--short=12", "HEAD") or "unknown",
            "dirty": bool(git("status", "--porcelain", "--", "paper_2503_20354_amd/csrc", "include"))}
    with open(os.path.join(HERE, "build_info.json"), "w") as f:
        json.dump(info, f)


if __name__ == "__main__":
    print(build(verbose=True, force="--changed" not in sys.argv))
