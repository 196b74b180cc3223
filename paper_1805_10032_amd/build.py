"""Build the HIP library for gfx950: one hipcc compile per source, one link.

    python -m paper_1805_10032_amd.build

The library lands in paper_1805_10032_amd/lib/libzeno_hip.so (in-tree)."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.environ.get("ZENO_BUILD_OUT") or os.path.join(LIB_DIR, "libzeno_hip.so")
OBJ_DIR = os.path.join(HERE, "_build")

# (source, object suffix, extra flags).  The streaming layer kernel's four instantiation files are compiled once per
# number of row blocks, longest first, so that twelve objects of similar size build in parallel.
LAYER_UNITS = ["zeno_layer_bf16_delta.hip", "zeno_layer_bf16_first.hip", "zeno_layer_f32_delta.hip", "zeno_layer_f32_first.hip"]
SOURCES = ([(u, f"_mb{mb}", [f"-DZENO_LAYER_MB={mb}"]) for mb in (4, 2, 1) for u in LAYER_UNITS] +
           [(s, "", []) for s in ("zeno_median.hip", "zeno_krum.hip", "zeno_capi.hip", "zeno_layer.hip", "zeno_loss.hip",
                                  "zeno_aggregate.hip", "zeno_median_select.hip", "zeno_conv.hip")])

# Packed-fp32 instruction selection is switched off for all device code.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


PER_FILE_FLAGS = {}


def _fresh(obj, src, stamp):
    """True if obj was built from the current source, headers and flags."""
    try:
        if open(obj + ".flags").read() != stamp:
            return False
        t = os.path.getmtime(obj)
        deps = [os.path.join(CSRC, src), os.path.join(CSRC, "zeno_internal.h"), os.path.join(ROOT, "include", "zeno.h")]
        if src.startswith("zeno_layer") or src in ("zeno_krum.hip", "zeno_conv.hip"):
            deps.append(os.path.join(CSRC, "zeno_layer_impl.h"))
        return all(os.path.getmtime(d) < t for d in deps)
    except OSError:
        return False


def _compile(unit, force=True):
    src, suffix, unit_flags = unit
    obj = os.path.join(OBJ_DIR, src.replace(".hip", suffix + ".o"))
    extra = [*unit_flags, *os.environ.get("ZENO_EXTRA_HIPCC_FLAGS", "").split()]
    stamp = " ".join([*HIPCC_FLAGS, *PER_FILE_FLAGS.get(src, []), *extra])
    if not force and _fresh(obj, src, stamp):
        return obj, ""
    cmd = [_hipcc(), *HIPCC_FLAGS, *PER_FILE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    with open(obj + ".flags", "w") as fh:
        fh.write(stamp)
    return obj, err


def build(verbose=True, force=True):
    """Compile and link.  force=False reuses objects whose source, headers and
    flags are unchanged (the 128-wide median network alone takes minutes)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(lambda s: _compile(s, force), SOURCES))
    for obj, err in results:
        if verbose and err.strip():
            print(err, file=sys.stderr)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *[o for o, _ in results]]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build(force="--force" in sys.argv)
