"""Builds libwino.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

hipcc cross-compiles without a GPU.  Each translation unit is compiled to an
object in parallel and the objects are linked into
``paper_2002_10711_amd/libwino.so``.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libwino.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops off: the transforms must be built from scalar v_fma_f32 only.
# -ffp-contract=off: every fused multiply-add in the kernels is written explicitly;
# nothing else may be fused, or the int8 results would depend on the compiler.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wall",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


# Per-file additions.  The int8 fused forwards keep their MFMA results in VGPRs: the
# accumulators are consumed by VALU code right away, and the AGPR form costs an extra
# v_accvgpr_read / v_accvgpr_write per value.
EXTRA_FLAGS = {
    "fused_fwd_exact_m2.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "fused_fwd_exact_m4.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "fused_fwd_exact_m6.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "fused_fwd.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "wide16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "gemm_out_col.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "gemm_out_trow.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "conv_implicit.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
}


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)
                  if f.endswith((".hip", ".cpp")))


def _compile(src):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [HIPCC] + FLAGS + EXTRA_FLAGS.get(os.path.basename(src), []) + ["-x", "hip", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    return obj, r.stderr


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        res = list(ex.map(_compile, sources()))
    objs = [o for o, _ in res]
    if verbose:
        for _, err in res:
            if err.strip():
                print(err)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
