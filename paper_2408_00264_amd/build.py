"""Build libclover.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libclover.so")
SOURCES = ["kernels_generic.hip", "kernels_mfma.hip", "kernels_stream.hip", "kernels_panel.hip", "kernels_tile.hip", "kernels_attn.hip", "kernels_draft.hip", "kernels_dyn.hip", "clover_api.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-value", "-I", os.path.join(ROOT, "include")]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def build(verbose: bool = False, ablate: bool = False, out: str = "", defines=()) -> str:
    """Compile every source and link the library.  `ablate` adds -DCLOVER_ABLATE (kernel-tuning builds that read
    CLOVER_* environment switches; never the shipped library) and needs an explicit `out` path; `defines` are further
    NAME=VALUE macros of such a build (the compile-time ablation bits of a kernel, e.g. CLOVER_TILE_ABLATE=17)."""
    if (ablate or defines) and not out:
        raise ValueError("an ablation build must not overwrite the shipped library: pass out=<path>")
    if defines and not ablate:
        raise ValueError("macros are for ablation builds only")
    build_dir = BUILD + ("_ablate" if ablate else "")
    lib_path = out or LIB
    flags = FLAGS + (["-DCLOVER_ABLATE"] if ablate else []) + ["-D" + d for d in defines]
    os.makedirs(build_dir, exist_ok=True)
    hipcc = _hipcc()
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]

    def compile_one(src: str) -> str:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *flags, "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        lines = r.stderr.splitlines()
        # a kernel that keeps arrays or spills in scratch memory runs many times slower: say so loudly
        name = None
        for l in lines:
            if "Function Name:" in l:
                name = l.split("Function Name:")[1].split("[")[0].strip()
            elif "ScratchSize [bytes/lane]:" in l and name:
                n = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
                if n:
                    print(f"[build] WARNING: {src}: kernel {name} uses {n} bytes/lane of scratch", file=sys.stderr)
        err = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "-Rpass-analysis" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, srcs))
    r = subprocess.run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib_path, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return lib_path


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--ablate", action="store_true", help="tuning build that reads CLOVER_* switches (needs --out)")
    ap.add_argument("--out", default="")
    ap.add_argument("--define", action="append", default=[], metavar="NAME=VALUE",
                    help="macro for an ablation build, e.g. CLOVER_TILE_ABLATE=17 (repeatable)")
    a = ap.parse_args()
    print(build(verbose=True, ablate=a.ablate, out=a.out, defines=tuple(a.define)))
