"""Build the CPU emulation of the library: its host code and its MFMA / layout kernels compiled as
plain C++ for the host (hip/hip_runtime.h here stands in for the HIP runtime, one OS thread per
GPU thread, wave-wide operations through per-wave barriers) with AddressSanitizer, so that a
kernel's addressing can be checked against exact-size buffers without a GPU.  The kernel sources
are taken as they are; one sed-like substitution turns the dynamic LDS declaration into a
malloc'ed block whose overruns the sanitizer sees."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(ROOT, "paper_2207_00032_amd", "csrc")
CXX = "/opt/rocm/llvm/bin/clang++"
FLAGS = ["-std=c++17", "-O1", "-g", "-fPIC", "-pthread", "-fsanitize=address", "-fno-omit-frame-pointer",
         "-Wno-unused-value", "-Wno-ignored-attributes"]
LDS_DECL = "extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];"

STUBS = r'''
#include "sbi_common.h"
#include "sbi_gemm.h"
namespace sbi {
int launch_stream(const GemmParams&, int, int, size_t, hipStream_t) { return 1; }
int launch_streamk(const SkParams&, int, int, int, hipStream_t) { return 1; }
}
extern "C" {
sbi_status sbi_calib_read(const void*, size_t, void*, size_t, int32_t, int32_t, int32_t, int32_t, void*) { return SBI_ERR_HIP; }
sbi_status sbi_calib_copy(const void*, void*, size_t, void*) { return SBI_ERR_HIP; }
}
'''


def build(out_dir):
    gen = os.path.join(out_dir, "gen")
    os.makedirs(gen, exist_ok=True)
    for name in ("sbi_common.h", "sbi_block.h", "sbi_abi.hip", "sbi_mfma.hip", "sbi_layout.hip", "sbi_i8.hip", "sbi_attn.hip"):
        text = open(os.path.join(SRC, name)).read()
        text = text.replace(LDS_DECL, "unsigned char* smem_raw = emu::lds();")
        text = text.replace('"../../include/sbi_gemm.h"', '"sbi_gemm.h"')
        open(os.path.join(gen, name.replace(".hip", ".cpp")), "w").write(text)
    open(os.path.join(gen, "sbi_gemm.h"), "w").write(open(os.path.join(ROOT, "include", "sbi_gemm.h")).read())
    open(os.path.join(gen, "stubs.cpp"), "w").write(STUBS)
    inc = ["-I", HERE, "-I", gen]
    units = [os.path.join(gen, f) for f in ("sbi_abi.cpp", "sbi_mfma.cpp", "sbi_layout.cpp", "sbi_i8.cpp", "sbi_attn.cpp", "stubs.cpp")] + \
            [os.path.join(HERE, "emu.cpp")]
    procs = []
    objs = []
    for u in units:
        obj = os.path.join(out_dir, os.path.basename(u).replace(".cpp", ".o"))
        objs.append(obj)
        procs.append(subprocess.Popen([CXX, *FLAGS, *inc, "-c", u, "-o", obj], stdout=subprocess.PIPE,
                                      stderr=subprocess.STDOUT, text=True))
    for p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(out[-4000:])
    lib = os.path.join(out_dir, "libsbi_emu.so")
    subprocess.run([CXX, "-shared", "-fsanitize=address", "-pthread", "-o", lib, *objs], check=True)
    exes = []
    for drv in ("emu_gemm", "emu_layer", "emu_attn"):
        exe = os.path.join(out_dir, drv)
        subprocess.run([CXX, "-std=c++17", "-O1", "-g", "-fsanitize=address", *inc, os.path.join(HERE, drv + ".cpp"),
                        "-o", exe, "-L", out_dir, "-lsbi_emu", "-Wl,-rpath," + out_dir, "-pthread"], check=True)
        exes.append(exe)
    return exes


if __name__ == "__main__":
    print(build(sys.argv[1] if len(sys.argv) > 1 else os.path.join(HERE, "_build")))
