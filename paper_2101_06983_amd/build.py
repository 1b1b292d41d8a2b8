"""Builds libgradcache.so (hipcc, gfx950 only) next to this file.

    python -m paper_2101_06983_amd.build [-f]

Objects go to _build/ at the repository root.  Nothing is built at import time:
tests, smoke() and bench.py load the library that is already there.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libgradcache.so")
SOURCES = ["api.hip", "loss_generic.hip", "loss_mfma.hip", "mlp.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the direct-to-LDS load statements name m0 in their clobber lists (they do write it); the backend notes for
    # each that m0 is one of its reserved registers, which is expected here
    "-Wno-inline-asm",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src, obj, extra):
    cmd = [HIPCC] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    return err


def build(force=True, extra_flags=(), verbose=False):
    bdir = os.path.join(ROOT, "_build")
    os.makedirs(bdir, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(ROOT, "include", "gradcache.h"))
    hdr_time = max(os.path.getmtime(h) for h in headers)
    jobs = []
    objs = []
    for s in SOURCES:
        obj = os.path.join(bdir, s.replace(".hip", ".o"))
        objs.append(obj)
        stale = force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(os.path.join(CSRC, s)), hdr_time)
        if stale:
            jobs.append((s, obj))
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        for msg in ex.map(lambda j: _compile(j[0], j[1], list(extra_flags)), jobs):
            if verbose and msg.strip():
                print(msg)
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", OUT] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return OUT


def build_host_checked(out, bdir):
    """A second library whose HOST code carries UndefinedBehaviorSanitizer checks that abort at the first finding
    (device code is unchanged: the sanitizer does not exist for it).  For the argument-check tests, which need no
    GPU.  api.hip, mlp.hip and loss_generic.hip are compiled again with the checks; the object of loss_mfma.hip,
    minutes of device compilation and no argument checks of its own, is taken from the ordinary build."""
    mfma = os.path.join(ROOT, "_build", "loss_mfma.o")
    if not os.path.exists(mfma):
        raise FileNotFoundError(mfma)
    san = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]
    srcs = [s for s in SOURCES if s != "loss_mfma.hip"]
    objs = [os.path.join(bdir, s.replace(".hip", "_ubsan.o")) for s in srcs]
    with ThreadPoolExecutor(max_workers=len(srcs)) as ex:
        list(ex.map(lambda j: _compile(j[0], j[1], san), zip(srcs, objs)))
    rt = subprocess.run([HIPCC, "-print-file-name=libclang_rt.ubsan_standalone-x86_64.so"], capture_output=True,
                        text=True).stdout.strip()
    if not os.path.isabs(rt):
        raise FileNotFoundError("the compiler's shared UBSan runtime")
    rt = os.path.dirname(os.path.realpath(rt))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-fsanitize=undefined",
                        "-shared-libsan", "-Wl,-rpath," + rt, "-Wno-option-ignored", "-o", out] + objs + [mfma],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return out


if __name__ == "__main__":
    print(build(force="-f" in sys.argv, verbose=True))
