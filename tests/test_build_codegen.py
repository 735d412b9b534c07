"""The VSA ping-pong kernel sits at the register limit: a spill inside one of its steady loops costs a factor, because
a scratch reload waits for vmcnt(0) and so drains the tile prefetches.  This test compiles vsa_pp.hip to assembly with
the flags build.py uses and checks that the fast loops hold no scratch access.  CPU only (hipcc cross-compiles)."""
import os
import re
import subprocess

import pytest

from paper_2604_12798_amd import build

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_vsa_fast_loops_have_no_scratch_access(tmp_path):
    out = tmp_path / "vsa_pp.s"
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")] + build.EXTRA_FLAGS["vsa_pp.hip"]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", "-o", str(out), os.path.join(build.CSRC, "vsa_pp.hip")],
                   check=True, capture_output=True)
    text = out.read_text()
    start = text.index("attn_vsa_pp_kernel")
    start = text.index(":\n", start)
    body = text[start:text.index(".Lfunc_end", start)].split("\n")
    labels = {m.group(1): n for n, l in enumerate(body) if (m := re.match(r"^(\.LBB\d+_\d+):", l))}
    # innermost loops = backward branches; a step pair of the pipeline holds 64 MFMAs
    loops = {}
    for n, l in enumerate(body):
        m = re.search(r"s_c?branch\w* (\.LBB\d+_\d+)", l)
        if m and m.group(1) in labels and labels[m.group(1)] < n:
            a = labels[m.group(1)]
            seg = body[a:n]
            if sum("v_mfma" in x for x in seg) == 64:
                loops[a] = min(loops.get(a, (1 << 30, 0)), (n - a, sum("scratch_" in x for x in seg)))
    assert len(loops) >= 4, "expected a fast and a general loop per group"
    # the fast loops are the two shortest ones (no masked / exact-max / ragged variants inside)
    fast = sorted(loops.values())[:2]
    assert all(length < 1300 for length, _ in fast), fast
    assert all(scratch == 0 for _, scratch in fast), f"scratch accesses in the VSA fast loops: {fast}"
