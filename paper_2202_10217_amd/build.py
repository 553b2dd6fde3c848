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


def generate_loops() -> str:
    """Writes csrc/syrk_asm_loops.inc from csrc/gen_asm_loops.py (the main loops of the SYRK kernels)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("gen_asm_loops", os.path.join(CSRC, "gen_asm_loops.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod.main()


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compiles the translation units in parallel (the SYRK kernels are compiled once per element type
    and kernel family: each takes a minute or two) and links them.  incremental=True (a developer's
    shortcut, `--incremental` on the command line) keeps an object file that is newer than every source
    and header; the default compiles everything."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OUT_DIR, exist_ok=True)
    obj_dir = os.path.join(OUT_DIR, "obj")
    os.makedirs(obj_dir, exist_ok=True)
    generate_loops()
    common = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
              # the assembly loops declare M0 clobbered; the compiler reports that it treats M0 as reserved
              # (it never keeps a value there across other code), once per loop instance
              "-Wno-inline-asm",
              # no packed fp32 arithmetic: some forms have given wrong results on this hardware
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    if verbose:
        common.insert(1, "-Rpass-analysis=kernel-resource-usage")
    syrk = os.path.join(CSRC, "syrk_kernels.hip")
    units = [("syrk_f64", syrk, ["-DTBS_UNIT_SYRK", "-DTBS_UNIT_TYPE=double"]),
             ("syrk_f32", syrk, ["-DTBS_UNIT_SYRK", "-DTBS_UNIT_TYPE=float"]),
             ("syrk_aug_f64", syrk, ["-DTBS_UNIT_SYRK_AUG", "-DTBS_UNIT_TYPE=double"]),
             ("syrk_aug_f32", syrk, ["-DTBS_UNIT_SYRK_AUG", "-DTBS_UNIT_TYPE=float"]),
             ("syr2k_f64", syrk, ["-DTBS_UNIT_SYR2K", "-DTBS_UNIT_TYPE=double"]),
             ("syr2k_f32", syrk, ["-DTBS_UNIT_SYR2K", "-DTBS_UNIT_TYPE=float"]),
             ("gemm_f64", syrk, ["-DTBS_UNIT_GEMM", "-DTBS_UNIT_TYPE=double"]),
             ("gemm_f32", syrk, ["-DTBS_UNIT_GEMM", "-DTBS_UNIT_TYPE=float"]),
             ("syrk_dispatch", syrk, ["-DTBS_UNIT_DISPATCH"]),
             ("potrf_kernels", os.path.join(CSRC, "potrf_kernels.hip"), []),
             ("tbs_planner", os.path.join(CSRC, "tbs_planner.cpp"), []),
             ("tbs_api", os.path.join(CSRC, "tbs_api.cpp"), [])]
    noise = "is not a recognized feature for this target"
    deps = [os.path.join(d, f) for d in (CSRC, os.path.join(ROOT, "include")) for f in os.listdir(d)
            if f.endswith((".h", ".inc", ".hip", ".cpp"))]

    def compile_unit(unit):
        name, src, defs = unit
        obj = os.path.join(obj_dir, name + ".o")
        if incremental and os.path.exists(obj):
            # (only tbs_api.cpp includes the public header)
            own = [src] + [f for f in deps if f.endswith((".h", ".inc")) and
                           (name == "tbs_api" or os.path.dirname(f) == CSRC)]
            if os.path.getmtime(obj) >= max(os.path.getmtime(f) for f in own):
                return obj, ""
        res = subprocess.run(common + defs + ["-c", src, "-o", obj], capture_output=True, text=True)
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on " + name + ":\n" + err)
        return obj, err

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        results = list(pool.map(compile_unit, units))
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + [o for o, _ in results],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed at the link step:\n" + res.stderr)
    if verbose:
        for _, err in results:
            if err:
                print(err)
    return OUT


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
