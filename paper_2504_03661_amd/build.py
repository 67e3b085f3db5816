"""Compile libpq_attn.so for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpq_attn.so")
SOURCES = ["pq12_codes.hip", "pq12_decode.hip", "pq12_decode_grouped.hip", "pq_api.hip", "pq_decode.hip", "pq_decode_grouped.hip", "pq_encode.hip", "pq_kmeans.hip", "pq_layout.hip"]
HEADERS = [os.path.join(CSRC, "pq_internal.h"), os.path.join(CSRC, "pq_device_utils.h"), os.path.join(CSRC, "pq_nearest_filter.h"), os.path.join(CSRC, "pq_filter_constants.h"),
           os.path.join(ROOT, "include", "pq_attn.h")]

# packed-fp32 instructions are switched off for all device code; -ffp-contract=off keeps
# the encode distances as separately rounded IEEE operations; matrix instructions write their
# results to ordinary vector registers (the kernels consume them with vector instructions at once:
# accumulation registers would cost one move per value).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-Wall", "-Wno-unused-result", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so: not an error
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if out.strip() and verbose:
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
