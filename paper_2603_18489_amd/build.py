"""Builds libec.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libec.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["ec_api.hip", "ec_rowstats.hip", "k_glue.hip", "k_gemm_f32.hip", "k_gemm_bf16.hip", "k_attn.hip", "k_attn_mfma.hip",
           "k_decide.hip"]
FLAGS = ["-O3", *os.environ.get("EC_EXTRA_FLAGS", "").split(), "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         # packed-fp32 code generation is switched off on purpose for the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


MFMA_SOURCES = ["k_gemm_bf16.hip", "k_attn_mfma.hip"]


def check_no_masked_mfma(hipcc: str) -> None:
    """MFMA instructions ignore the EXEC mask.  If the compiler if-converts a guarded MFMA into
    an EXEC-masked one (it does so for conditions it cannot prove wave-uniform), the MFMA runs
    anyway and corrupts the accumulator.  This scans the generated ISA and fails the build if an
    MFMA sits inside an EXEC-masked region that has no branch around it."""
    for src in MFMA_SOURCES:
        asm = os.path.join(OBJ_DIR, src.replace(".hip", ".s"))
        cmd = [hipcc, *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", asm]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src}:\n{r.stderr}")
        masked, kernel = False, "?"
        for line in open(asm):
            t = line.strip()
            if line.startswith("_ZN2ec") and ":" in line:
                kernel = line.split(":")[0]
            if t.startswith(("s_and_saveexec", "s_andn2_saveexec", "s_or_saveexec")):
                masked = True
            elif t.startswith(("s_cbranch_exec", "s_or_b64 exec", "s_mov_b64 exec")):
                masked = False
            elif t.startswith("v_mfma") and masked:
                raise RuntimeError(f"{src}: EXEC-masked MFMA in {kernel}: make its condition "
                                   "wave-uniform (readfirstlane) or remove the guard")


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    objs = []

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as pool:
        chk = pool.submit(check_no_masked_mfma, hipcc)
        objs = list(pool.map(compile_one, SOURCES))
        chk.result()
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
