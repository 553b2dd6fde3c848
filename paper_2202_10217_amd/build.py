"""Builds the HIP library (csrc/ -> lib/libtbs_syrk.so) for gfx950 with hipcc.

Run on the CPU-only build machine (hipcc cross-compiles); the GPU machine only loads the result.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT_DIR = os.path.join(HERE, "lib")
OUT = os.path.join(OUT_DIR, "libtbs_syrk.so")
SOURCES = ["syrk_kernels.hip", "potrf_kernels.hip", "tbs_planner.cpp", "tbs_api.cpp"]


def generate_loops() -> str:
    """Writes csrc/syrk_asm_loops.inc from csrc/gen_asm_loops.py (the main loops of the SYRK kernels)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("gen_asm_loops", os.path.join(CSRC, "gen_asm_loops.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod.main()


def build(verbose: bool = False) -> str:
    os.makedirs(OUT_DIR, exist_ok=True)
    generate_loops()
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           # no packed fp32 arithmetic: some forms have given wrong results on this hardware
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", OUT] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err:
        print(err)
    return OUT


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv))
