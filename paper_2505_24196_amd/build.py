"""Compiles the HIP library (gfx950) in-tree: paper_2505_24196_amd/libclasp_hip.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libclasp_hip.so")
SOURCES = [os.path.join(CSRC, "clasp_api.hip")]
HEADERS = [os.path.join(CSRC, f) for f in ("clasp_common.h", "clasp_gemm.h", "clasp_attn.h", "clasp_misc.h", "clasp_sample.h", "clasp_prefill.h")] + [
    os.path.join(os.path.dirname(HERE), "include", "clasp.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """extra_flags / out: for tuning sweeps (e.g. -DCLASP_NW_DOWN=16 into another file); the product uses neither."""
    if not force and not is_stale():
        return LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 code generation
           "-Wno-unused-command-line-argument", "-o", out] + list(extra_flags) + SOURCES
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the GPU-only target feature and says so; that line is noise
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
