"""Builds libgr.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libgr.so")
SOURCES = ["gr_api.hip", "gr_mask.hip", "gr_select.hip", "gr_attn.hip", "gr_reorder.hip", "gr_diag.hip"]
# packed-fp32 VALU forms are disabled on purpose (hipcc would otherwise form them from scalar code)
COMMON = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wno-inline-asm", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
PER_FILE = {"gr_select.hip": ["-ffp-contract=off"]}


def build_lib(verbose: bool = False) -> str:
    """Compile every HIP source and link libgr.so.  Always recompiles."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if pr.returncode != 0:
            failed = True
            print(f"--- {src} failed\n" + "\n".join(lines), file=sys.stderr)
        elif verbose and lines:
            print("\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL if not verbose else None, stderr=subprocess.STDOUT if not verbose else None)
    return LIB_PATH


if __name__ == "__main__":
    print(build_lib(verbose=True))
