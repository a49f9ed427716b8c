"""Builds libvocabtrim.so (the HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libvocabtrim.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


# The draft-step kernels issue their loads from inline assembly and wait for them by hand; the compiler
# does not know that such a register is still in flight, so a spill of one would save a value that
# has not arrived yet.  Their sources must therefore compile without any scratch memory.
NO_SCRATCH = ("vt_head_", "vt_row_select")
# For the same reason nothing may touch such a register between its load and the wait that covers it (a
# copy at the join of a branch, a split live range): the device assembly of these sources is checked
# path by path, see inflight_lint.py.
# The check recognises hand-issued loads by the markers the compiler puts around inline assembly and by their
# mnemonics; if a compiler update changed either it would find no loads and pass everything.  So the number of
# hand-issued loads it followed must reach a floor per source (well below today's counts -- vt_head_mfma.hip
# 1152, vt_head_gemv_np1/2/4/8.hip 344 / 344 / 300 / 72, vt_row_select.hip none, its loads are the compiler's own --
# and far above zero).  The model was validated against the assembly of AMD clang 20 (ROCm 7.2.0), -O3, gfx950.
MIN_HAND_LOADS = {"vt_head_mfma.hip": 600, "vt_head_gemv_np1.hip": 150, "vt_head_gemv_np2.hip": 150,
                  "vt_head_gemv_np4.hip": 150, "vt_head_gemv_np8.hip": 36}


def _scratch_users(remarks: str):
    """(kernel, bytes per lane) for every kernel the resource-usage remarks report with scratch memory."""
    out, name = [], None
    for line in remarks.splitlines():
        if "remark: Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and name is not None:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n != 0:
                out.append((name, n))
    return out


def _inflight_violations(src: str):
    """Compiles src to gfx950 assembly (same flags as the object) and runs the in-flight register check."""
    try:
        from . import inflight_lint
    except ImportError:      # run as a script
        import inflight_lint
    asm = os.path.join(OBJ, os.path.basename(src)[:-4] + ".s")
    r = subprocess.run([HIPCC] + FLAGS + ["--cuda-device-only", "-S", src, "-o", asm], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc -S failed on {src}:\n{r.stderr}")
    with open(asm) as f:
        bad, followed = inflight_lint.check_asm(f.read())
    os.remove(asm)
    floor = MIN_HAND_LOADS.get(os.path.basename(src), 0)
    if followed < floor:
        raise RuntimeError(f"{os.path.basename(src)}: the in-flight register check followed {followed} hand-issued "
                           f"loads, fewer than the {floor} this source is known to hold: it no longer recognises "
                           "them (compiler output changed?) and would pass anything")
    return bad


def _compile(src: str, force: bool) -> str:
    base = os.path.basename(src)
    obj = os.path.join(OBJ, base[:-4] + ".o")
    headers = glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(ROOT, "include", "*.h"))
    if force or _stale(obj, [src] + headers):
        check = base.startswith(NO_SCRATCH)
        extra = ["-Rpass-analysis=kernel-resource-usage"] if check else []
        r = subprocess.run([HIPCC] + FLAGS + extra + ["-c", src, "-o", obj], capture_output=True, text=True)
        if check:
            bad = _scratch_users(r.stderr)
            if bad:
                if os.path.exists(obj):
                    os.remove(obj)
                raise RuntimeError(f"{base}: kernels with hand-issued loads must not spill: {bad}")
            if r.returncode == 0:
                touched = _inflight_violations(src)
                if touched:
                    os.remove(obj)
                    raise RuntimeError(f"{base}: registers of hand-issued loads are touched before their wait "
                                       f"(kernel, line of the load, line and text of the instruction in the "
                                       f"device assembly): {touched[:5]}")
        lines = r.stderr.splitlines()
        if check and r.returncode == 0:
            lines = []      # the remarks (and their source excerpts) are not diagnostics
        err = "\n".join(l for l in lines if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def build_library(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = _sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    if force or _stale(LIB, objs):
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(force="--force" in sys.argv))
