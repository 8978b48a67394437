"""Build libvxl.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2506_19225_amd.build`."""
from __future__ import annotations

import concurrent.futures as cf
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libvxl.so")

SOURCES = ["vxl_api.hip", "vxl_simple.hip", "vxl_bilevel.hip", "vxl_prefill.hip", "vxl_decode.hip", "vxl_mass.hip", "vxl_store.hip", "vxl_debug.hip"]

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
NO_SCRATCH = {"vxl_prefill.hip": ("prefill_dma_kernel",),
              "vxl_decode.hip": ("decode_ring_kernel", "decode_wave_kernel"),
              "vxl_debug.hip": ("tile_loop_kernel",)}


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


def _check_no_compiler_m0(src: str) -> None:
    """The hand-issued direct loads of these kernels overwrite m0 inside inline assembly, behind
    the compiler's back; that is only sound while the compiler itself never reads or writes m0 in
    the same kernel.  Scan the device assembly (kept by --save-temps) outside the inline blocks."""
    stem = os.path.splitext(src)[0]
    asm = [f for f in os.listdir(OBJ) if f.startswith(stem + "-hip-amdgcn") and f.endswith(".s")]
    if not asm:
        raise RuntimeError(f"{src}: device assembly not found for the m0 check")
    name, in_asm = None, False
    hand, own = {}, {}            # per kernel: m0 written inside inline assembly / by the compiler
    for ln in open(os.path.join(OBJ, asm[0])):
        st = ln.strip()
        if st.startswith("_Z") and ":" in st and st.split(":")[0].isidentifier():
            name = st.split(":")[0]
        elif st.startswith(".Lfunc_end"):
            name = None
        elif st.startswith(";;#ASMSTART"):
            in_asm = True
        elif st.startswith(";;#ASMEND"):
            in_asm = False
        elif name and any(k in name for k in NO_SCRATCH[src]):
            code = st.split(";")[0]
            if re.search(r"\bm0\b", code):
                (hand if in_asm else own).setdefault(name, code.strip())
            if not in_asm and re.match(r"\s*scratch_(load|store)", code):
                raise RuntimeError(f"{src}: kernel {name} accesses scratch memory ({code.strip()}); its hand-kept "
                                   "vmcnt bookkeeping needs a compile without stack traffic")
    for name in hand:             # (an instance without hand-issued loads may use m0 as it likes)
        if name in own:
            raise RuntimeError(f"{src}: kernel {name} has a compiler-generated use of m0 ({own[name]}) "
                               "beside inline-assembly direct loads that overwrite m0")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    extra = ["-Rpass-analysis=kernel-resource-usage", "--save-temps=obj"] if src in NO_SCRATCH else []
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in r.stderr.splitlines() if noise not in ln)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if src in NO_SCRATCH:
        _check_no_scratch(src, err)
        _check_no_compiler_m0(src)
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
