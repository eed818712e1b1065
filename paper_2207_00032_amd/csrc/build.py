"""Build libsbi_gemm.so (gfx950 only) in-tree with hipcc.  Cross-compiles without a GPU."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
LIB = os.path.join(PKG, "libsbi_gemm.so")
SOURCES = ["sbi_abi.hip", "sbi_layout.hip", "sbi_mfma.hip", "sbi_stream.hip", "sbi_streamk.hip", "sbi_calib.hip", "sbi_i8.hip", "sbi_attn.hip"]
HEADERS = ["sbi_common.h", "sbi_block.h", "sbi_calib.h", os.path.join("..", "..", "include", "sbi_gemm.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         # keep the compiler from forming packed fp32 VALU instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


DEV_LIB = os.path.join(PKG, "libsbi_gemm_dev.so")
# The measurement build: the same sources with the development switches compiled in - per-block
# timestamps (SBI_TRACE: environment SBI_TRACE_PTR = device address of 8 x 64-bit words per block),
# parts of the kernel switched off (SBI_DEV: environment SBI_ABLATE = bit mask) and forced launch plans
# (SBI_DEV: SBI_PLAN_FORCE = "waves,depth,panels,T,lds_cap").  bench.py --timeline / --ablate load it.
DEV_FLAGS = ["-DSBI_DEV", "-DSBI_TRACE"]


def build(verbose: bool = False, extra_flags=(), lib: str = LIB, suffix: str = ".o") -> str:
    objs = []
    procs = []
    for s in SOURCES:
        obj = os.path.join(HERE, s.replace(".hip", suffix))
        cmd = ["hipcc", *FLAGS, *extra_flags, "-c", os.path.join(HERE, s), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.run(link, check=True)
    return lib


def build_dev(verbose: bool = False) -> str:
    return build(verbose, DEV_FLAGS, DEV_LIB, ".dev.o")


if __name__ == "__main__":
    if "--dev" in sys.argv[1:]:
        print(build_dev(verbose=True))
    else:
        print(build(verbose=True, extra_flags=sys.argv[1:]))
