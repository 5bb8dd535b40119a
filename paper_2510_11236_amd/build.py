"""Build libxq.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2510_11236_amd.build

The decode kernel is compiled once per (head_dim, group, key bits, value bits); the
objects are built in parallel and linked into paper_2510_11236_amd/libxq.so.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libxq.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _jobs():
    jobs = [("xq_host.o", "xq_host.cpp", ["-x", "hip", "-ffp-contract=off"]),
            ("xq_pack.o", "xq_pack.hip", ["-ffp-contract=off"]),
            ("xq_prefill.o", "xq_prefill.hip", ["-ffp-contract=off"]),
            ("xq_merge.o", "xq_merge.hip", [])]
    for D in (128, 64):
        for G in (32, 64):
            for bk in (1, 2):
                for bv in (1, 2):
                    jobs.append((f"xq_decode_{D}_{G}_{bk}{bv}.o", "xq_decode.hip",
                                 [f"-DXQ_D={D}", f"-DXQ_G={G}", f"-DXQ_BK={bk}", f"-DXQ_BV={bv}"]))
    for G in (32, 64):      # the kernels with the fp8 x fp4 key phase: head_dim 128, 2-bit keys
        for bv in (1, 2):
            jobs.append((f"xq_decode_kx_128_{G}_2{bv}.o", "xq_decode.hip",
                         ["-DXQ_KX_TU", "-DXQ_D=128", f"-DXQ_G={G}", "-DXQ_BK=2", f"-DXQ_BV={bv}",
                          # matrix results straight into ordinary registers (they are folded by vector
                          # instructions right away; the accumulator-register form costs a copy per value)
                          "-mllvm", "-amdgpu-mfma-vgpr-form=1"]))
    return jobs


def _compile(job):
    obj, src, extra = job
    cmd = [HIPCC] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ, obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{err}")
    return err


def build(workers: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = _jobs()
    with ThreadPoolExecutor(max_workers=workers) as ex:
        for err in ex.map(_compile, jobs):
            if err.strip():
                sys.stderr.write(err + "\n")
    objs = [os.path.join(OBJ, j[0]) for j in jobs]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
