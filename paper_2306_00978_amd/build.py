"""Build libawq_mi355x.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libawq_mi355x.so")
# the same library with the planner constants open to environment overrides (experiments, and the
# test that runs the other kernel variants); the product is LIB, which reads no environment
LIB_KNOBS = os.path.join(HERE, "libawq_mi355x_knobs.so")
SOURCES = ["awq_api.hip", "awq_prep.hip", "awq_quantize.hip", "awq_gemv.hip", "awq_gemv_stream.hip", "awq_gemm.hip",
           "awq_linear.hip", "awq_search.hip", "awq_w3.hip", "awq_w2.hip", "awq_attention.hip"]

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # packed-FP32 instructions are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
]
# the quantizer decides integers: one rounding per operation, as on the CPU side
PER_FILE = {"awq_quantize.hip": ["-ffp-contract=off"], "awq_prep.hip": ["-ffp-contract=off"],
            "awq_w3.hip": ["-ffp-contract=off"], "awq_w2.hip": ["-ffp-contract=off"]}


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


# Host-side sanitizer build (validation layer, planners, marshalling): device code is compiled as
# always, the host pass with AddressSanitizer and UndefinedBehaviorSanitizer.  The result is loaded
# into a process that has the compiler's ASan runtime preloaded (sanitizer_runtime()).
SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]


def sanitizer_runtime() -> str:
    cc = hipcc()
    out = subprocess.run([cc, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = out.stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        import glob
        found = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
        if not found:
            raise RuntimeError("ASan runtime of the HIP compiler not found")
        path = found[-1]
    return path


def build(verbose: bool = False, save_temps: bool = False, sanitize_host_into: str | None = None,
          knobs: bool = False) -> str:
    """Compile every source and link the shared library. Always recompiles.
    sanitize_host_into: a directory; the library is then built there (not in-tree) with the host
    code under ASan + UBSan and its path returned.  knobs: build LIB_KNOBS (-DAWQ_TUNING_KNOBS)."""
    objdir = sanitize_host_into or os.path.join(HERE, "_build_knobs" if knobs else "_build")
    lib_path = os.path.join(objdir, "libawq_mi355x_san.so") if sanitize_host_into else (LIB_KNOBS if knobs else LIB)
    extra = SANITIZE if sanitize_host_into else (["-DAWQ_TUNING_KNOBS"] if knobs else [])
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [cc, "-c", os.path.join(CSRC, src), "-o", obj] + COMMON + PER_FILE.get(src, []) + extra
        if save_temps:
            cmd += ["-save-temps=obj"]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        try:
            out, _ = p.communicate(timeout=900)
        except subprocess.TimeoutExpired:
            p.kill()
            out, _ = p.communicate()
            out += "\n[build] compiler timed out after 900 s"
        out = "\n".join(l for l in out.splitlines()
                        if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    link = [cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib_path] + objs + \
           ["-Wl,-rpath,/opt/rocm/lib"] + (["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]
                                           if sanitize_host_into else [])
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return lib_path


def build_all(verbose: bool = False) -> str:
    """The product library and its tuning twin."""
    lib = build(verbose=verbose)
    build(verbose=verbose, knobs=True)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, save_temps="--save-temps" in sys.argv))
    if "--save-temps" not in sys.argv:
        print(build(verbose=True, knobs=True))
