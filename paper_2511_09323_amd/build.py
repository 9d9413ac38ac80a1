"""Builds the HIP library in-tree: paper_2511_09323_amd/libmoc_ffn.so (gfx950 only).

The entry points are spread over four translation units that are compiled side by side and
linked into one shared library.
"""
import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoc_ffn.so")
SOURCES = ["moc_api.hip", "moc_fwd.hip", "moc_bwd.hip", "moc_decode.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
] + os.environ.get("MOC_EXTRA_HIPCC_FLAGS", "").split()


def source_hash():
    """Content hash of the kernel sources (csrc/*.h, csrc/*.hip, include/moc.h).  The library carries the
    hash it was built from in moc_version(), so a measurement taken on one build can be told from a
    measurement taken on another."""
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hip")))
    files.append(os.path.join(os.path.dirname(HERE), "include", "moc.h"))
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    # The packed-fp32 feature is a device feature; hipcc also hands the flag to its host pass, which
    # answers with one "not a recognized feature for this target" line per use.  Those lines are
    # dropped so that any other diagnostic stands out.
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    for line in r.stderr.splitlines():
        if "packed-fp32-ops' is not a recognized feature for this target" in line:
            continue
        print(line, file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def build(verbose=True, only=None):
    """Compiles every source (or the ones named in `only`, reusing the other objects) and links."""
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    # moc_api.hip holds the version string with the source hash, so it is compiled every time
    todo = [(s, o) for s, o in zip(SOURCES, objs) if only is None or s in only or s == "moc_api.hip" or not os.path.exists(o)]
    define = ['-DMOC_SOURCE_HASH="%s"' % source_hash()]
    with ThreadPoolExecutor(max_workers=4) as pool:
        jobs = [pool.submit(_run, [HIPCC] + FLAGS + define + ["-c", os.path.join(CSRC, s), "-o", o], verbose) for s, o in todo]
        for j in jobs:
            j.result()
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build(only=sys.argv[1:] or None)
    print("built", LIB)
