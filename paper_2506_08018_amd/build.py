"""Compile the HIP sources under csrc/ into paper_2506_08018_amd/libkvmix.so for gfx950."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvmix.so")
OBJ_DIR = os.path.join(HERE, "_build")

COMMON = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# per-source extra flags: the quantizer's arithmetic is specified operation by operation
SOURCES = {
    "kvmix_quant.hip": ["-ffp-contract=off"],
    # tile claims are single-lane LDS atomics whose result is taken late; the wave-reduction rewrite of
    # uniform atomics would put a wait right behind them
    "kvmix_attn.hip": ["-mllvm", "-amdgpu-atomic-optimizer-strategy=None"],
    "kvmix_mixed.hip": ["-ffp-contract=off"],
    "kvmix_api.hip": [],
}


def _compile(item):
    src, extra = item
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    cmd = COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    return obj, err


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        results = list(ex.map(_compile, SOURCES.items()))
    if verbose:
        for obj, err in results:
            if err.strip():
                print(err)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for o, _ in results], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
