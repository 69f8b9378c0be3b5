"""Build the HIP library (libmi_gemm.so) in-tree with hipcc for gfx950.

Every source is compiled to an object file of its own, side by side (the kernel table is one translation
unit per data type), and the objects are linked into the shared library."""
import concurrent.futures
import os
import shutil
import subprocess
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libmi_gemm.so")
SOURCES = ["gemm_table_f32.hip", "gemm_table_f16.hip", "gemm_table_bf16.hip", "gemm_table_i8.hip", "gemm_table.hip",
           "gemm_static_ws.hip", "gemm_api.cpp"]
HEADERS = ["gemm_kernel.hpp", "gemm_kernel_dma.hpp", "gemm_kernel_ring.hpp", "gemm_kernel_dma32.hpp", "gemm_kernel_dma32t.hpp", "gemm_kernel_reg32.hpp",
           "gemm_kernel_reg16.hpp", "gemm_solo.hpp", "gemm_launchers.hpp", "gemm_table.h",
           os.path.join("..", "..", "include", "mi_gemm.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no packed-fp32 instructions from the auto-vectoriser
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(force=True, verbose=False):
    """Compile the library; with force=False only when a source is newer than it."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = tempfile.mkdtemp(prefix="mi_gemm_build_")
    tmp = LIB + ".tmp.%d" % os.getpid()
    try:
        objs = [os.path.join(objdir, os.path.splitext(f)[0] + ".o") for f in SOURCES]
        jobs = min(len(SOURCES), max(1, min(8, os.cpu_count() or 1)))
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda so: _run([hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose),
                          zip(SOURCES, objs)))
        _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-Wno-unused-command-line-argument"] + objs + ["-o", tmp],
             verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
        if os.path.exists(tmp):
            os.remove(tmp)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
