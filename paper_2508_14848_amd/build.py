"""Build libgemm_mp.so (HIP, gfx950 only) in-tree with hipcc."""
import glob
import os
import shutil
import subprocess

from . import check_isa

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgemm_mp.so")
SOURCES = ["gemm_mp_host.hip", "kernels_scan_pack.hip", "kernels_gemm.hip",
           # the GEMM kernels: one template instance per file, compiled in parallel
           "gemm_owner_d.hip", "gemm_owner_d_mixed.hip", "gemm_owner_d_bf.hip", "gemm_owner_d_low.hip",
           "gemm_owner_f.hip", "gemm_owner_f_mixed.hip", "gemm_owner_f_bf.hip",
           "gemm_region_fp8.hip", "gemm_region_mxfp8.hip", "gemm_region_mxfp4.hip",
           "gemm_region_fp16.hip", "gemm_region_bf16.hip", "gemm_region_mxfp6.hip"]
# -ffp-contract=off: the only fused multiply-adds are the ones the code asks for.
# packed-fp32 instructions are switched off for this target.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]


def build_library(verbose=False, extra_flags=()):
    """Compile every source and link the shared library; always rebuilds."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    temps = os.path.join(CSRC, "_build")
    os.makedirs(temps, exist_ok=True)
    for src in SOURCES:
        # the 128 x 128 kernels keep their intermediate files: their assembly is checked below
        owner = src.startswith("gemm_owner_")
        obj = os.path.join(temps if owner else CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, *(["-save-temps=obj"] if owner else []), "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    for asm in sorted(glob.glob(os.path.join(temps, "gemm_owner_*-hip-amdgcn-amd-amdhsa-gfx950.s"))):
        n, bad = check_isa.violations(asm)
        if n == 0 or bad:
            raise RuntimeError("%s: %d basic blocks with inline-assembly matrix instructions, %d instructions that touch their "
                               "accumulators in mid-run (first: %s)" % (os.path.basename(asm), n, len(bad), bad[:1]))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    shutil.rmtree(temps, ignore_errors=True)            # tens of megabytes of intermediate files
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
