"""Builds libmoeprefill.so (HIP, gfx950 only) in-tree with hipcc: every source is compiled to an
object of its own (in parallel), then linked.  The device ceilings probe (probe/ceilings.hip, used
by `bench.py --ceilings` only) becomes a small library of its own, libmoeceilings.so."""
from concurrent.futures import ThreadPoolExecutor
import glob
import hashlib
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoeprefill.so")
STAMP = LIB + ".srchash"
PROBE_SRC = os.path.join(HERE, "probe", "ceilings.hip")
PROBE_LIB = os.path.join(HERE, "libmoeceilings.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-inline-asm",
]
# the host pass does not know the gfx950 target feature above and says so once per function: noise
_NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if _NOISE not in l)
    if p.returncode != 0:
        sys.stderr.write(out + "\n")
        raise subprocess.CalledProcessError(p.returncode, cmd)
    if verbose and out.strip():
        print(out)


def build(verbose=False, extra=(), out=None, jobs=8, link_extra=()):
    """Compiles every source for gfx950 and links the shared library (always, also when one exists).
    `extra`: more hipcc flags (e.g. -D switches of an experiment, host sanitizers), `out`: another
    output path, `link_extra`: more flags for the link step."""
    out = out or LIB
    with tempfile.TemporaryDirectory(prefix="moe_build_") as tmp:
        objs = []
        cmds = []
        for src in sources():
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            objs.append(obj)
            cmds.append(["hipcc", *HIPCC_FLAGS, *extra, "-c", src, "-o", obj])
        with ThreadPoolExecutor(max(1, min(jobs, len(cmds)))) as ex:
            list(ex.map(lambda c: _run(c, verbose), cmds))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, "-o", out + ".tmp", *objs], verbose)
    os.replace(out + ".tmp", out)
    if out == LIB:
        build_probe(verbose)
    if out == LIB and not extra:
        with open(STAMP, "w") as f:
            f.write(source_hash() + "\n")
    elif out == LIB and os.path.exists(STAMP):
        os.remove(STAMP)             # an experiment's flags: never taken for the product build
    return out


def build_probe(verbose=False):
    """Compiles the ceilings probe into its own shared library."""
    _run(["hipcc", *HIPCC_FLAGS, "-shared", PROBE_SRC, "-o", PROBE_LIB + ".tmp"], verbose)
    os.replace(PROBE_LIB + ".tmp", PROBE_LIB)
    return PROBE_LIB


def source_hash():
    """Digest of everything the library is built from (sources, headers, flags)."""
    deps = sources() + sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h")))
    deps.append(PROBE_SRC)
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for p in deps:
        h.update(os.path.basename(p).encode())
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def needs_build():
    """True when the library is missing or was built from other sources than the tree holds now
    (the digest written beside it at build time differs; file times are not trusted: they do not
    survive every copy of the tree)."""
    if not os.path.exists(LIB) or not os.path.exists(PROBE_LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_hash()


def ensure_built():
    """What tests, smoke() and bench.py call before loading the library: builds it when it is
    missing or stale.  Must run before anything touches the GPU (the build starts hipcc children)."""
    if os.environ.get("MOE_PREFILL_LIB"):
        return os.environ["MOE_PREFILL_LIB"]       # an explicitly chosen build is taken as it is
    if needs_build():
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
