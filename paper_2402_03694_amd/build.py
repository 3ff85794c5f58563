"""Builds the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libserveflow_hip.so")

# -ffp-contract=off: the feature statistics are defined with one rounding per operation.
# The packed-fp32 feature is switched off for device code (hipcc's host pass does not know
# the feature and says so; that warning is harmless).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every kernel file into one shared library; returns its path."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, *sources(), "-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


SAN_LIB = os.path.join(ROOT, "_build", "libserveflow_hip_hostsan.so")
CLANG_ASAN_RUNTIME = "/opt/rocm/llvm/lib/clang"


def build_host_sanitized() -> str:
    """A second copy of the library whose HOST code (argument checks, the threshold algorithms, workspace
    arithmetic) is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer; the device code is
    built as always.  For CPU-side tests only: load it with the sanitizer runtime preloaded
    (asan_runtime()) and SERVEFLOW_LIB pointing at it."""
    os.makedirs(os.path.dirname(SAN_LIB), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + [
        "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
        "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"]
    cmd = [hipcc, *flags, "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, *sources(), "-o", SAN_LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc (host sanitizers) failed:\n" + res.stdout)
    return SAN_LIB


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime that matches hipcc's host compiler."""
    hits = glob.glob(os.path.join(CLANG_ASAN_RUNTIME, "*", "lib", "linux", "libclang_rt.asan-x86_64.so"))
    if not hits:
        raise RuntimeError("no libclang_rt.asan-x86_64.so under " + CLANG_ASAN_RUNTIME)
    return sorted(hits)[-1]


if __name__ == "__main__":
    print(build(force=True, verbose=True))
