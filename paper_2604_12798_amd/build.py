"""Compile the HIP sources of this package into libvfa.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvfa.so")
SOURCES = ["vfa_fwd.hip", "vsa_pp.hip"]
# attn_vsa_pp_kernel sits at the register limit; with the scheduler's default register-pressure tracking the allocator
# spills an accumulator inside its steady loops, with this tracker it does not (checked on the generated code)
EXTRA_FLAGS = {"vsa_pp.hip": ["-mllvm", "-amdgpu-use-amdgpu-trackers=1"]}

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions must not be generated on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"),
]


PROBE_SRC = os.path.join(ROOT, "bench_probes.hip")   # bench.py's ceiling probes (MFMA only, HBM read only): a library of its own
PROBE_LIB = os.path.join(ROOT, "bench_probes.so")


def _run(cmd: list[str], verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err:
        print(err)


def build_lib(verbose: bool = False, extra: list[str] | None = None) -> str:
    """One object per source (some carry flags of their own), then one link."""
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="vfa_build_") as tmp:
        objs = []
        for src in SOURCES:
            obj = os.path.join(tmp, src + ".o")
            _run([hipcc] + compile_flags + EXTRA_FLAGS.get(src, []) + (extra or []) + ["-c", "-o", obj, os.path.join(CSRC, src)],
                 verbose)
            objs.append(obj)
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


def build_probe(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + HIPCC_FLAGS + ["-o", PROBE_LIB, PROBE_SRC], verbose)
    return PROBE_LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
    print(build_probe(verbose=True))
