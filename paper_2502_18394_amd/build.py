"""Build the HIP library in-tree: ``python -m paper_2502_18394_amd.build [--incremental]``.

Cross-compiles for gfx950 with hipcc (no GPU needed): one object per source file, compiled in
parallel into ``_build/``, then one link.  Packed-fp32 instruction selection is switched off for
all device code.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libspectre_hip.so")
SOURCES = ["api.hip", "mix_pow2.hip", "mix_slab.hip", "mix_chirp.hip", "gate.hip", "prefix.hip", "project.hip",
           "wrm.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and out:
        print(out, flush=True)


def build(verbose=False, extra=(), incremental=False):
    """Compile every source (or, with incremental=True, those older than any source or header) and link."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(os.path.join(d, f))
                        for d in (CSRC, os.path.join(HERE, "..", "include"))
                        for f in os.listdir(d) if f.endswith(".h"))
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o"))
        stale = not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header)
        if stale or not incremental or extra:
            jobs.append([hipcc] + FLAGS + list(extra) + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    args = sys.argv[1:]
    inc = "--incremental" in args
    build(verbose=True, extra=[a for a in args if a != "--incremental"], incremental=inc)
    print("built", LIB)
