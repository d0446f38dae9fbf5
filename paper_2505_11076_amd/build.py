"""Builds libdbf.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2505_11076_amd.build

hipcc cross-compiles without a GPU.  Every HIP source is compiled with packed fp32
instructions disabled (-packed-fp32-ops), as required on the target machines.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdbf.so")

SOURCES = [
    "dbf_layout.cpp",
    "dbf_api.hip",
    "dbf_gemv_valu.hip",
    "dbf_gemv_mfma.hip",
    "dbf_gemm_i8.hip",
    "dbf_gemm_static.hip",
    "dbf_probe.hip",
    "dbf_prune.hip",
    "dbf_svid.hip",
    "dbf_admm.hip",
]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    # kernel arguments arrive in scalar registers with the wavefront instead of being loaded by its first
    # instructions: one memory round trip less at the head of every kernel (0.25 us per launch of a lone layer)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


# Kernels that issue loads by inline assembly and wait for them by hand (the tile and operand rings).  The compiler
# does not know that such a load is still in flight: if it SPILLS the destination register right after the asm
# statement, it reuses the register -- for an address, say -- and the data that lands later overwrites it: a memory
# fault on the GPU, not a wrong number.  So these kernels must be built without a single spilled vector register;
# the build checks the compiler's own resource report and refuses the library otherwise.
NO_SPILL = {"dbf_gemv_mfma.hip": "dbf_items_mfma_kernel", "dbf_gemm_i8.hip": "dbf_gemm_i8_stage_kernel"}
REMARK = "-Rpass-analysis=kernel-resource-usage"


def _check_no_spills(src: str, stderr: str) -> None:
    name, bad = None, []
    for line in stderr.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "VGPRs Spill:" in line and name and NO_SPILL[src] in name:
            n = int(line.split("VGPRs Spill:")[1].split("[")[0].strip())
            if n:
                bad.append("%s: %d spilled vector registers" % (name, n))
    if bad:
        raise RuntimeError("%s: kernels with hand-issued loads must not spill registers (an in-flight load would land in "
                           "a register the compiler has reused):\n  %s" % (src, "\n  ".join(bad)))


# The second guard for the same kernels.  A ring slot must live in ONE set of registers for the whole kernel: if the
# compiler gives a slot two homes (it does as soon as a refill's destination is not the registers the consumed tile was in)
# it copies between them at loop ends -- registers whose load is still in flight, and the copy reads what was there before:
# wrong sums, no fault, and only on the paths that loop.  So the build compiles the file to assembly as well and counts, per
# kernel, the distinct destination register sets of the ring's loads: PF tile slots, plus PF per operand column group where
# the operand travels in the ring (SHARED >= 2).
RING_SRC = "dbf_gemv_mfma.hip"


def _ring_homes_report(code: str, pf: int, pf_f4: int):
    """(kernels seen, [complaints]) for the assembly text `code` of RING_SRC."""
    import re
    bad, seen = [], 0
    for m in re.finditer(r"^(_ZN\w*dbf_items_mfma_kernelILi(\d)ELb\dELi(\d)ELb\dELi\dELb(\d)E\w*):", code, re.M):
        body = code[m.end():code.index("s_endpgm", m.end())]
        homes = set(re.findall(r"buffer_load_dwordx4 (v\[\d+:\d+\])", body))
        ncg, shared, f4 = int(m.group(2)), int(m.group(3)), int(m.group(4))
        want = (pf_f4 if f4 else pf) * (1 + ncg if shared >= 2 else 1)
        seen += 1
        if len(homes) != want:
            bad.append("%s: %d register sets for %d ring slots" % (m.group(1), len(homes), want))
    return seen, bad


def _check_ring_homes() -> None:
    import re
    import tempfile
    text = open(os.path.join(CSRC, RING_SRC)).read()
    pf = int(re.search(r"#define DBF_PF (\d+)", text).group(1))
    pf_f4 = int(re.search(r"#define DBF_PF_F4 (\d+)", text).group(1))
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "ring.s")
        cmd = [_hipcc(), *[f for f in FLAGS if f != "-fPIC"], "--cuda-device-only", "-S", "-x", "hip",
               os.path.join(CSRC, RING_SRC), "-o", asm]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc -S failed for %s:\n%s" % (RING_SRC, res.stderr))
        code = open(asm).read()
    seen, bad = _ring_homes_report(code, pf, pf_f4)
    if not seen:
        raise RuntimeError("%s: no items kernel found in the assembly (has it been renamed?)" % RING_SRC)
    if bad:
        raise RuntimeError("%s: a ring slot has more than one register home (the compiler would copy registers whose load "
                           "is in flight):\n  %s" % (RING_SRC, "\n  ".join(bad)))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    extra = [REMARK] if src in NO_SPILL else []
    cmd = [_hipcc(), *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    if src in NO_SPILL:
        _check_no_spills(src, res.stderr)
    noise = "is not a recognized feature for this target"
    kept, skip = [], 0
    for l in res.stderr.splitlines():
        if REMARK in l:  # (a remark and the two lines of source context under it)
            skip = 2
        elif skip and ("|" in l[:12]):
            skip -= 1
        elif noise not in l and not l.endswith("remarks generated when compiling for gfx950."):
            kept.append(l)
    warn = "\n".join(kept).strip()
    if warn:
        print(warn, file=sys.stderr)
    return obj


def _compile_to(src_path: str, obj: str, extra) -> str:
    cmd = [_hipcc(), *FLAGS, *extra, "-x", "hip", "-c", src_path, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src_path, res.stdout, res.stderr))
    return obj


def build_sanitize_check(driver_cpp: str) -> str:
    """Links `driver_cpp` (a C++ program that calls the C ABI) with the library's sources into an executable
    whose HOST code is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer: the packer / tile
    layout and the file that holds the argument checks are compiled with the sanitizers, the kernel files are
    taken as already built (their host side is launch glue).  GPU code is never instrumented (each
    -fsanitize= sits behind -Xarch_host).  Returns the path of the executable."""
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    out_dir = os.path.join(OBJ, "sanitize")
    os.makedirs(out_dir, exist_ok=True)
    plain = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES
             if s not in ("dbf_layout.cpp", "dbf_api.hip")]
    if not all(os.path.exists(o) for o in plain):
        build(verbose=False)
    objs = [_compile_to(os.path.join(CSRC, "dbf_layout.cpp"), os.path.join(out_dir, "dbf_layout.o"), san),
            _compile_to(os.path.join(CSRC, "dbf_api.hip"), os.path.join(out_dir, "dbf_api.o"), san),
            _compile_to(driver_cpp, os.path.join(out_dir, "driver.o"), san)]
    exe = os.path.join(out_dir, "sanitize_host")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
           "-o", exe, *objs, *plain]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("sanitizer link failed:\n%s\n%s" % (res.stdout, res.stderr))
    return exe


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as pool:
        ring = pool.submit(_check_ring_homes)
        objs = list(pool.map(_compile, SOURCES))
        ring.result()
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
