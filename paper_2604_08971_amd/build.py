"""Builds libsentryfuse.so (16-bit models in bfloat16) and libsentryfuse_f16.so (the same sources compiled with
-DSF_HALF_F16: 16-bit models in IEEE binary16) for gfx950, in-tree, with hipcc.
`python -m paper_2604_08971_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsentryfuse.so")
LIB_F16 = os.path.join(HERE, "libsentryfuse_f16.so")

SOURCES = ["api.hip", "masks.hip", "compact.hip", "gemm_bf16.hip", "gemm_bf16_fast.hip", "gemm_bf16_ws.hip", "gemm_f32.hip", "moe.hip", "gate.hip", "fp8_ffn.hip", "tokens.hip", "lazy_proj.hip", "fp8_proj.hip",
           "attention_common.hip", "attention_bf16.hip", "ceilings.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 VALU forms stay off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(job) -> str:
    src, half = job
    obj = os.path.join(OBJ, half, src.replace(".hip", ".o"))
    cmd = ["hipcc"] + FLAGS + (["-DSF_HALF_F16"] if half == "f16" else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src} ({half}):\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 7) -> str:
    for half in ("bf16", "f16"):
        os.makedirs(os.path.join(OBJ, half), exist_ok=True)
    work = [(s, h) for h in ("bf16", "f16") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, work))
    for half, lib in (("bf16", LIB), ("f16", LIB_F16)):
        mine = [o for o, (_, h) in zip(objs, work) if h == half]
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-Bsymbolic", "-o", lib] + mine
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
