"""Build libtl.so (host packers + gfx950 HIP kernels + C ABI) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libtl.so")
OBJDIR = os.path.join(HERE, "_build")

SOURCES = ["tl_host.cpp", "tl_basic.hip", "tl_gemv.hip", "tl_gemv3.hip", "tl_mfma.hip", "tl_api.hip"]

# packed-fp32 VALU forms are switched off for every device translation unit.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", INCLUDE, "-I", CSRC,
]


def _newest_dep():
    t = 0.0
    for root in (CSRC, INCLUDE):
        for f in os.listdir(root):
            t = max(t, os.path.getmtime(os.path.join(root, f)))
    return t


# Host-side sanitizer build (AddressSanitizer + UBSan on the host pass only; the device code is
# compiled as usual): for running the CPU test suite over the packers, the ternariser and the
# argument checks.  See README, "Sanitizer pass".
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-g"]
SAN_LIB = os.path.join(HERE, "_build", "san", "libtl.so")


def build(force=True, verbose=False, extra_flags=(), sanitize=False):
    global OBJDIR, LIB
    if sanitize:
        objdir, lib = os.path.join(HERE, "_build", "san"), SAN_LIB
        saved = OBJDIR, LIB
        OBJDIR, LIB = objdir, lib
        try:
            return _build(True, verbose, tuple(extra_flags) + tuple(SAN_FLAGS),
                          ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"])
        finally:
            OBJDIR, LIB = saved
    return _build(force, verbose, extra_flags, [])


def _build(force, verbose, extra_flags, link_flags):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    dep_time = _newest_dep()
    objs = []
    procs = []
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        obj = os.path.join(OBJDIR, src + ".o")
        objs.append(obj)
        if not force and os.path.exists(obj) and os.path.getmtime(obj) >= dep_time:
            continue
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-x", "hip", "-c", path, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        text = "\n".join(l for l in text.splitlines()
                         if "packed-fp32-ops' is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] {src} failed:\n{text}\n")
        elif text.strip() and verbose:
            sys.stderr.write(text + "\n")
    if failed:
        raise RuntimeError("hipcc failed")
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *link_flags, "-o", LIB, *objs]
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True, sanitize="--sanitize" in sys.argv))
