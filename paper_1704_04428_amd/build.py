"""Compile the HIP library for gfx950 into paper_1704_04428_amd/libconv_mcmk.so (in-tree).

Every .hip file under csrc/ is a translation unit; they are compiled in parallel and linked.
"""
import concurrent.futures
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libconv_mcmk.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",       # per-kernel register / LDS / spill report, kept beside the objects
    # the tile kernels are written as fully unrolled loops over (tap, position block); for 7 x 7 kernels the
    # body passes the default size limit for '#pragma unroll', and a loop left rolled turns the register
    # rings into scratch memory
    "-mllvm", "-pragma-unroll-threshold=200000",
]
JOBS = 8
TIMEOUT_S = 900      # per translation unit; a compile that takes longer is a bug, not patience


def units():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(name: str) -> str:
    obj = os.path.join(OBJ, name[:-4] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, name), "-o", obj]
    done = subprocess.run(cmd, check=True, timeout=TIMEOUT_S, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE)
    with open(os.path.join(OBJ, name[:-4] + ".usage.txt"), "wb") as f:
        f.write(done.stderr)
    return obj


def resource_usage() -> dict:
    """{mangled kernel name: {"VGPRs": n, "ScratchSize": n, "LDS": n, "Occupancy": n, ...}} from the last build."""
    import re
    out = {}
    if not os.path.isdir(OBJ):
        return out
    for fn in sorted(os.listdir(OBJ)):
        if not fn.endswith(".usage.txt"):
            continue
        name = None
        with open(os.path.join(OBJ, fn), errors="replace") as f:
            for line in f:
                m = re.search(r"remark: .*Function Name: (\S+)", line)
                if m:
                    name = m.group(1)
                    out[name] = {}
                    continue
                m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
                if m and name:
                    out[name][m.group(1).strip().replace(" ", "")] = int(m.group(2))
    return out


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    try:
        with concurrent.futures.ThreadPoolExecutor(max_workers=JOBS) as pool:
            objs = list(pool.map(_compile, units()))
    except subprocess.CalledProcessError as e:
        raise RuntimeError("hipcc failed:\n" + e.stderr.decode(errors="replace")[-4000:]) from None
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                   check=True, timeout=TIMEOUT_S)
    return LIB


if __name__ == "__main__":
    print(build())
