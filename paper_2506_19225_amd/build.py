"""Build libvxl.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2506_19225_amd.build`."""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libvxl.so")

SOURCES = ["vxl_api.hip", "vxl_simple.hip", "vxl_bilevel.hip", "vxl_prefill.hip", "vxl_decode.hip", "vxl_mass.hip", "vxl_prefill_pipe.hip", "vxl_store.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


# Kernels that keep their own count of outstanding vector-memory operations (direct global-to-LDS
# loads issued from inline assembly, waited for with hand-written vmcnt values): a register spill
# would add scratch loads and stores to that count behind the kernel's back, so the build refuses
# a compile in which one of them uses scratch memory.
NO_SCRATCH = {"vxl_prefill.hip": ("prefill_dma_kernel",), "vxl_decode.hip": ("decode_ring_kernel",),
              "vxl_prefill_pipe.hip": ("prefill_pipe_kernel",)}

# Per-file compiler options.  The software-pipelined pre-filling kernel runs one wave per SIMD with
# more than 256 registers; its score products must land in ordinary vector registers (the vector
# ALU reads them), its output accumulators are placed in the accumulation registers by hand.
EXTRA_FLAGS = {"vxl_prefill_pipe.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _check_no_scratch(src: str, remarks: str) -> None:
    name = None
    for ln in remarks.splitlines():
        if "remark: Function Name:" in ln:
            name = ln.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in ln and name and any(k in name for k in NO_SCRATCH[src]):
            size = int(ln.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size != 0:
                raise RuntimeError(f"{src}: kernel {name} spills ({size} bytes of scratch per lane); "
                                   "its hand-kept vmcnt bookkeeping needs a spill-free compile")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    extra = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SCRATCH else []
    extra += EXTRA_FLAGS.get(src, [])
    if os.environ.get("VXL_PIPE_ABL") and src == "vxl_prefill_pipe.hip":     # measurement builds only
        extra += ["-DVXL_PIPE_ABL=" + os.environ["VXL_PIPE_ABL"]]
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in r.stderr.splitlines() if noise not in ln)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if src in NO_SCRATCH:
        _check_no_scratch(src, err)
        keep, skip = [], 0                                   # drop the remarks (and their source echo)
        for ln in err.splitlines():
            if "[-Rpass-analysis=kernel-resource-usage]" in ln:
                skip = 2
            elif skip and (ln.lstrip().startswith("|") or "|" in ln[:8]):
                skip -= 1
            else:
                skip = 0
                keep.append(ln)
        err = "\n".join(keep)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_lib(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build_lib()
