"""Build librtp.so (HIP kernels for gfx950 + the host scheduler) in-tree with hipcc."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librtp.so")
SOURCES = ["rtp_gemm_bf16.hip", "rtp_gemm_pp.hip", "rtp_gemm_pp_nt.hip", "rtp_gemm_pp_nn.hip", "rtp_gemm_pp_tn.hip",
           "rtp_gemm_pp_nt_f16.hip", "rtp_gemm_pp_nn_f16.hip", "rtp_gemm_pp_tn_f16.hip",
           "rtp_misc_kernels.hip", "rtp_host.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -packed-fp32-ops off: the compiler must not form packed fp32 arithmetic from scalar code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-x", "hip"]


def _newer(dst, srcs):
    return os.path.exists(dst) and all(os.path.getmtime(dst) >= os.path.getmtime(s) for s in srcs)


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    kernel_headers = [os.path.join(CSRC, h) for h in ("rtp_kernels.h", "rtp_gemm_epilogue.h", "rtp_gemm_pp.h")]
    host_headers = [os.path.join(CSRC, "rtp_kernels.h"), os.path.join(HERE, "..", "include", "rtp.h")]

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        headers = host_headers if src == "rtp_host.cpp" else kernel_headers
        if force or not _newer(o, [s] + headers):
            cmd = [HIPCC] + FLAGS + ["-c", s, "-o", o]
            tiled = src.startswith("rtp_gemm_pp_")
            if tiled:
                cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, check=True, stderr=subprocess.PIPE, text=True)
            if tiled:
                # the tiled GEMM must keep its accumulators in registers: a build that spills is a broken build
                spills = [ln for ln in res.stderr.splitlines() if "ScratchSize" in ln and not ln.rstrip().endswith(": 0 [-Rpass-analysis=kernel-resource-usage]")]
                if spills:
                    raise RuntimeError(f"{src}: the tiled GEMM kernel spills registers to scratch memory:\n" + "\n".join(spills))
                # ... and leave room for a wave of the staging copy kernel (96 registers) beside its own two waves on a
                # SIMD (512 registers): above 208 the copies only run where no GEMM wave sits, and the steps wait for them
                import re
                fat = [ln for ln in res.stderr.splitlines() if (m := re.search(r" VGPRs: (\d+)", ln)) and int(m.group(1)) > 208]
                if fat:
                    raise RuntimeError(f"{src}: the tiled GEMM kernel uses more than 208 vector registers:\n" + "\n".join(fat))
        return o

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    if force or not _newer(LIB, objs):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--force" in sys.argv, verbose=True))
