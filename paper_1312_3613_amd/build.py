"""Compile the HIP library (csrc/) for gfx950 into paper_1312_3613_amd/libaugur_hip.so.

hipcc cross-compiles without a GPU.  Packed-fp32 instruction selection is switched off for
all device code.  Each source is compiled to an object of its own (in parallel) under
paper_1312_3613_amd/_build/ and the objects are linked; a digest of the sources is kept beside the
library so that a library older than its sources is noticed whatever the files' time stamps say.
"""
import hashlib
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libaugur_hip.so")
DIGEST = LIB + ".digest"
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["api.cpp", "lda.hip", "probe.hip", "gmm.hip", "mh.hip"]
HEADERS = ["common.hpp", "lda_device.hpp", "lda_sample_z.hpp", "lda_count.hpp", "lda_gamma.hpp",
           "lda_loglik.hpp", os.path.join("..", "..", "include", "augur.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def source_digest():
    h = hashlib.sha256()
    h.update(" ".join(FLAGS).encode())
    for path in sources() + [os.path.join(CSRC, x) for x in HEADERS]:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def stale():
    """True when the library is absent or was built from other sources than the ones present."""
    if not os.path.exists(LIB) or not os.path.exists(DIGEST):
        return True
    with open(DIGEST) as f:
        return f.read().strip() != source_digest()


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    digest = source_digest()

    def compile_one(src):
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        cmd = [HIPCC] + FLAGS + ["-x", "hip", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # the host pass does not know the packed-fp32 feature and says so once per function
        log = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{log}")
        if log.strip():
            print(log)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, sources()))
    if os.path.exists(DIGEST):
        os.remove(DIGEST)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], check=True)
    with open(DIGEST, "w") as f:
        f.write(digest + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
