"""Compile the HIP sources under csrc/ into paper_2603_12617_amd/liboco.so for gfx950."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liboco.so")
SOURCES = ["oco_api.hip", "dense_rounds.hip", "sparse_rounds.hip", "meta.hip", "specdec.hip",
           "comparator_gemm.hip", "dense_window.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def sources_newer_than_lib() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [
        os.path.join(HERE, "..", "include", h) for h in ("oco.h", "specdec.h")]
    return any(os.path.getmtime(f) > t for f in files)


def build(verbose: bool = False, extra_flags=(), lib: str = LIB, tag: str = "") -> str:
    """Compile and link.  `extra_flags`/`lib`/`tag` build a variant (e.g. other tile
    shapes via -DOCO_CFG64=...) next to the default library."""
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()

    def one(src):
        obj = os.path.join(OBJ, src.replace(".hip", tag + ".o"))
        cmd = [cc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0 or verbose:
            sys.stderr.write(res.stdout + res.stderr)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on " + src)
        return obj

    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(one, SOURCES))
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("link failed")
    return lib


PROBES = ["row_rate_probe.hip", "fetch_ahead_probe.hip"]


def build_probes() -> list:
    """Compile the stand-alone measurement probes under csrc/probes/ into _build/probes/ (executables
    that time memory access patterns on one GPU; the library does not use them)."""
    out_dir = os.path.join(OBJ, "probes")
    os.makedirs(out_dir, exist_ok=True)
    cc = _hipcc()
    outs = []
    for src in PROBES:
        exe = os.path.join(out_dir, src.replace(".hip", ""))
        cmd = [cc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(CSRC, "probes", src), "-o", exe]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError("hipcc failed on " + src)
        outs.append(exe)
    return outs


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
    if "--probes" in sys.argv:
        print(build_probes())
