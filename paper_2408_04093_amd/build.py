"""Compile the HIP library for gfx950 into paper_2408_04093_amd/libtree_attn.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtree_attn.so")
SOURCES = ["ta_api.cpp", "decode_partial.hip", "decode_partial_mfma.hip", "tree_combine.hip"]
HEADERS = ["ta_internal.hpp", "wave_ops.hpp", "chunking.hpp", "mfma_tile.hpp", "balanced_index.hpp", "balanced_walk.hpp"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-x", "hip",
    # no packed-fp32 VALU instructions (v_pk_*_f32) in device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, h) for h in HEADERS] + \
        [os.path.join(HERE, "..", "include", "tree_attn.h")]
    return any(os.path.getmtime(d) > t for d in deps)


BENCH_DIR = os.path.join(HERE, "..", "bench")
PROBES = ("hbm_probe", "l2_read_probe")   # stand-alone measurement aids, not part of the library


def build_probe(verbose: bool = False) -> str:
    """The stand-alone probes under bench/ (HBM read/copy ceiling and counter calibration; reads of
    L2-resident data by access pattern).  Returns the path of the first."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for name in PROBES:
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", os.path.join(BENCH_DIR, name + ".hip"), "-o", os.path.join(BENCH_DIR, name)]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stderr)
    return os.path.join(BENCH_DIR, PROBES[0])


def build(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra) + sources() + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the AMDGPU feature name and says so; drop that line
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_probe(verbose=True))
