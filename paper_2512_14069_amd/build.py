"""Builds the HIP library (libradar.so) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libradar.so")
SOURCES = ["radar_common.hip", "radar_expand.hip", "radar_accept.hip", "radar_attention.hip", "radar_policy.hip", "radar_accept_q.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed fp32 arithmetic is kept off for device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force=True, verbose=False):
    """Compile every kernel source and link paper_2512_14069_amd/libradar.so."""
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "radar.h"))
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    for src in SOURCES:
        sp = os.path.join(CSRC, src)
        if not os.path.exists(sp):
            raise RuntimeError(f"kernel source {sp} is missing")
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        if force or _stale(obj, [sp] + headers):
            cmd = [HIPCC] + FLAGS + ["-c", sp, "-o", obj]
            r = subprocess.run(cmd, capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed for {src}:\n{err}")
            if verbose and err.strip():
                print(err, file=sys.stderr)
        objs.append(obj)
    if force or _stale(LIB, objs):
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build_library(force="--force" in sys.argv, verbose=True))
