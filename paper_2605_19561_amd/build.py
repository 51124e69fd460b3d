"""Compile libtorq.so (HIP kernels + C ABI) for gfx950 with hipcc.

`python -m paper_2605_19561_amd.build` or `build()`.  The library is built in-tree
(paper_2605_19561_amd/libtorq.so) so that it travels with the source tree.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtorq.so")
SOURCES = ["api.hip", "quantize.hip", "rotate_quant.hip", "rotate_butterfly.hip", "mxfp4_gemm.hip", "mxfp4_gemm_skinny.hip", "block_gram.hip", "code_histogram.hip",
           "intra_calib.hip", "diag.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         # packed fp32 arithmetic is kept off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


# The rotate kernel post-processes its MFMA results with vector ALU code, so its accumulators are
# kept in ordinary VGPRs (no v_accvgpr_read traffic); the GEMM needs the AGPR half for its tile.
# rotate_quant.hip writes m0 in inline assembly (the LDS address of a buffer load into LDS) and says so in the
# clobber list; the compiler warns about every such statement, since it reserves m0 for itself -- nothing
# else in that kernel uses it.
EXTRA = {"rotate_quant.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-Wno-inline-asm"],
         "rotate_butterfly.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "mxfp4_gemm_skinny.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def device_asm(source: str, out_path: str) -> str:
    """Compile one source to gfx950 assembly text with the flags of the build (for the build test that
    counts the memory instructions of a hand-scheduled loop)."""
    cmd = [HIPCC, *FLAGS, *EXTRA.get(source, []), "--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", out_path]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return out_path


def build(verbose: bool = False) -> str:
    objs = []
    procs = []
    for s in SOURCES:
        obj = os.path.join(CSRC, s.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *EXTRA.get(s, []), "-c", os.path.join(CSRC, s), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
