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
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the loads that write LDS directly are issued as assembly and name m0, a reserved register, as clobbered
         "-Wno-inline-asm"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


SAN_LIB = os.path.join(HERE, "libradar_san.so")
# host code only (the GPU side has no sanitizer here): each option directly after -Xarch_host
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def sanitizer_runtime():
    """Path of the address-sanitizer runtime the sanitized library needs preloaded."""
    r = subprocess.run([os.path.join(os.path.dirname(HIPCC), "..", "lib", "llvm", "bin", "clang"),
                        "--print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    return r.stdout.strip()


def build_library(force=True, verbose=False, sanitize=False):
    """Compile every kernel source and link paper_2512_14069_amd/libradar.so.  sanitize=True builds
    libradar_san.so instead: the same sources with the HOST code (argument checks, planning, launch
    paths) under AddressSanitizer and UndefinedBehaviorSanitizer; used by the CPU tests only."""
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "radar.h"))
    if sanitize:
        return _build(os.path.join(HERE, "_build", "san"), SAN_LIB, [f for f in FLAGS if f != "-O3"] + ["-O1"] + SAN_FLAGS,
                      ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"], headers, force, verbose)
    return _build(os.path.join(HERE, "_build"), LIB, FLAGS, [], headers, force, verbose)


def _build(objdir, lib, flags, link_flags, headers, force, verbose):
    os.makedirs(objdir, exist_ok=True)
    objs = []
    for src in SOURCES:
        sp = os.path.join(CSRC, src)
        if not os.path.exists(sp):
            raise RuntimeError(f"kernel source {sp} is missing")
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        if force or _stale(obj, [sp] + headers):
            cmd = [HIPCC] + flags + ["-c", sp, "-o", obj]
            r = subprocess.run(cmd, capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed for {src}:\n{err}")
            if verbose and err.strip():
                print(err, file=sys.stderr)
        objs.append(obj)
    if force or _stale(lib, objs):
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + link_flags + ["-o", lib] + objs,
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
    return lib


if __name__ == "__main__":
    print(build_library(force="--force" in sys.argv, verbose=True))
