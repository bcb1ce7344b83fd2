"""Build libadacc.so (HIP, gfx950) in-tree.  `python -m paper_2508_00806_amd.build`."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libadacc.so")
CSRC = os.path.join(HERE, "csrc")
# one translation unit per group of kernel instantiations, so that the library builds in parallel
# Sources that touch the tensor's elements are compiled once per 16-bit format (bf16; binary16 with -DADACC_F16=1).
PER_FORMAT = (
    "adacc_k_none.hip", "adacc_k_abs.hip", "adacc_k_std.hip", "adacc_k_topk.hip",  # compress, per outlier mode
    "adacc_k_decompress.hip",
    "adacc_k_batch4.hip", "adacc_k_batch8.hip",
    "adacc_k_place.hip",      # placement of the outliers in the stream
    "adacc_k_tail.hip",       # the end of a tensor that the group sizes do not divide
    "adacc_k_generic.hip",    # fallback for group sizes that are no powers of two or exceed 4096
    "adacc_k_channel.hip",    # outlier channels by Z-score
    "adacc_k_channelwise.hip",  # channel-wise symmetric quantisation (Q / K / V)
)
ONCE = (
    "adacc.hip",              # host code, C ABI, utility kernels
    "adacc_k_mask.hip",       # dropout mask, byte <-> bit
)
# (source, object suffix, extra flags); the long ones first
SOURCES = ([(os.path.join(CSRC, f), "", ()) for f in PER_FORMAT] +
           [(os.path.join(CSRC, f), "_f16", ("-DADACC_F16=1",)) for f in PER_FORMAT] +
           [(os.path.join(CSRC, f), "", ()) for f in ONCE])
HEADERS = [os.path.join(CSRC, f) for f in ("adacc_common.hpp", "adacc_dtype.hpp", "adacc_compress.hpp",
                                           "adacc_decompress.hpp", "adacc_kernels.hpp", "adacc_fn.hpp",
                                           "adacc_channel.hpp", "adacc_tail.hpp", "adacc_generic.hpp")]
HEADERS.append(os.path.join(ROOT, "include", "adacc.h"))
OBJDIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",            # the order and rounding of every float operation is part of the format
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, extra=(), jobs: int = 8) -> str:
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJDIR, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    tag = os.path.splitext(os.path.basename(LIB))[0]

    def compile_one(item):
        src, suffix, defines = item
        obj = os.path.join(OBJDIR, tag + "_" + os.path.splitext(os.path.basename(src))[0] + suffix + ".o")
        cmd = [HIPCC, *FLAGS, *defines, *extra, *inc, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    print(LIB)
