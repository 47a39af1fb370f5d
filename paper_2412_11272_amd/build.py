"""Build libwf_encoder.so (gfx950) from csrc/*.hip with hipcc.  Usage: python -m paper_2412_11272_amd.build"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwf_encoder.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
         # packed-fp32 VALU forms are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results land in architectural VGPRs: the softmax and the epilogues consume them with VALU
         # instructions, and the AGPR form costs a v_accvgpr_read per value
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         # extra compiler flags for experiments (e.g. -D switches of compile-time variants)
         *os.environ.get("WF_HIPCC_EXTRA", "").split()]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


def build_sanitized_host_driver(driver_src: str, out_path: str) -> str:
    """Every source of the library with AddressSanitizer + UndefinedBehaviorSanitizer on the HOST side (device
    code is compiled as usual: GPU sanitizers are not used) and a driver program linked statically against those
    objects.  For tests of the host logic (planning, validation, round bookkeeping, beam pruning); no GPU needed."""
    obj_dir = os.path.join(OBJ_DIR, "asan")
    os.makedirs(obj_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1"] + san
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))

    def comp(src, lang=()):
        obj = os.path.join(obj_dir, os.path.basename(src) + ".o")
        r = subprocess.run([HIPCC, *lang, *flags, "-c", src, "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed on {src}:\n{r.stderr}")
        return obj

    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as ex:
        futs = [ex.submit(comp, s) for s in srcs] + [ex.submit(comp, driver_src, ("-x", "hip"))]
        objs = [f.result() for f in futs]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-rdc", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
                        "-o", out_path, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link (sanitized) failed:\n" + r.stderr)
    return out_path


if __name__ == "__main__":
    build()
