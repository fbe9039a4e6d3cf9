"""Build libhcache.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhcache.so")
SOURCES = ["api.cpp", "store.cpp", "saver.cpp", "restore_mode0.hip", "restore_mode1.hip",
           "restore_mode2.hip", "aux_kernels.hip", "static_restore.hip"]


def hipcc_path():
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


# Diagnostic builds: each name takes one companion of the matrix ops out of the restoration
# kernel's main loop (results are then wrong on purpose; timing only).  `--diag NAME[,NAME]`
# writes libhcache_diag_<names>.so next to the library; HCACHE_LIB=<path> makes the binding
# load it instead.
DIAG = {"no_sumsq": "-DHC_DIAG_NO_SUMSQ", "no_loads": "-DHC_DIAG_NO_LOADS",
        "no_ldsread": "-DHC_DIAG_NO_LDSREAD", "no_barrier": "-DHC_DIAG_NO_BARRIER",
        "no_epilogue": "-DHC_DIAG_NO_EPILOGUE", "no_rope_reads": "-DHC_DIAG_NO_ROPE_READS",
        "few_stores": "-DHC_DIAG_FEW_STORES", "same_tile": "-DHC_DIAG_SAME_TILE"}


def build(verbose=False, extra_flags=(), out=None, tag=""):
    """Compile every source for gfx950 (one hipcc process per file, in parallel) and link the
    shared library (`out`, default libhcache.so next to this file).  Always recompiles."""
    from concurrent.futures import ThreadPoolExecutor
    obj_dir = os.path.join(HERE, "_build" + tag)
    os.makedirs(obj_dir, exist_ok=True)
    common = [
        hipcc_path(), "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
        "-Wall", "-Wno-unused-result", "-pthread",
        # packed fp32 ALU forms are kept out of the generated code on purpose
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra_flags,
    ]

    def compile_one(src):
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        cmd = common + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        return obj, subprocess.run(cmd, capture_output=True, text=True)

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 16)) as pool:
        results = list(pool.map(compile_one, SOURCES))
    failed = [r for _, r in results if r.returncode != 0]
    if failed:
        for r in failed:
            sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed")
    if verbose:
        for _, r in results:
            sys.stderr.write(r.stderr)
    link = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread",
            *[o for o, _ in results], "-o", out or LIB]
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("link failed")
    return out or LIB


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--diag", default="", help="comma-separated diagnostic variants: " + ", ".join(DIAG))
    a = ap.parse_args()
    if a.diag:
        names = a.diag.split(",")
        print(build(verbose=True, extra_flags=tuple(DIAG[n] for n in names),
                    out=os.path.join(HERE, "libhcache_diag_" + "_".join(names) + ".so"),
                    tag="_diag_" + "_".join(names)))
    else:
        print(build(verbose=True))
