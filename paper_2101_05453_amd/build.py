"""Builds liblstm_int.so (HIP, gfx950) in-tree.  Run: python -m paper_2101_05453_amd.build"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblstm_int.so")
SOURCES = ["prepare.cpp", "kernels.hip", "persistent.hip", "in_gemm.hip", "rec_inst_8.hip", "rec_inst_20.hip",
           "rec_inst_32.hip", "rec_sparse_inst_8.hip", "rec_sparse_inst_20.hip", "rec_sparse_inst_32.hip", "rec16_inst.hip", "rec16_inst_4.hip", "rec16_inst_10.hip", "rec16_inst_16.hip", "stack.hip", "stack_inst_8.hip", "stack_inst_20.hip", "stack_inst_32.hip", "calibrate.hip", "ceiling.hip", "gru.hip", "sru.hip", "api.hip"]
HOSTMATH_LIB = os.path.join(HERE, "liblstm_int_hostmath.so")
HOSTMATH_SAN_LIB = os.path.join(HERE, "liblstm_int_hostmath_san.so")
SANITIZE_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]

# packed-fp32 instructions are disabled for all device code
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-function"]
# in_gemm.hip: MFMA results go to ordinary vector registers, where the requantization reads them without copies
EXTRA_FLAGS = {f: ["-mllvm", "-amdgpu-mfma-vgpr-form=1"] for f in ("in_gemm.hip", "rec_inst_8.hip", "rec_inst_20.hip", "rec_inst_32.hip", "rec_sparse_inst_8.hip", "rec_sparse_inst_20.hip", "rec_sparse_inst_32.hip", "rec16_inst_4.hip", "rec16_inst_10.hip", "rec16_inst_16.hip", "stack_inst_8.hip", "stack_inst_20.hip", "stack_inst_32.hip")}


def _compile(src, verbose):
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + HIP_FLAGS + EXTRA_FLAGS.get(src, [])
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 or verbose:
        print(" ".join(cmd))
        print(_filter(r.stderr))
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}")
    return obj


def build(verbose=False):
    """Compiles every source for gfx950 (translation units in parallel) and
    links the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(lambda s: _compile(s, verbose), SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    build_hostmath()
    return LIB


def build_hostmath(sanitize=False):
    """Host-only build of the device math header and of the offline phase, for CPU
    checks of them; sanitize=True builds a second copy under AddressSanitizer and
    UndefinedBehaviorSanitizer (signed overflow, shifts, bounds: the 64-bit
    headroom claims of the integer arithmetic trap instead of wrapping)."""
    out = HOSTMATH_SAN_LIB if sanitize else HOSTMATH_LIB
    cmd = ["g++", "-std=c++17", "-O1" if sanitize else "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-o", out,
           os.path.join(CSRC, "hostmath_shim.cpp"), os.path.join(CSRC, "prepare.cpp")] + (SANITIZE_FLAGS if sanitize else [])
    subprocess.run(cmd, check=True)
    return out


def _filter(text):
    return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)


if __name__ == "__main__":
    print(build(verbose=True))
