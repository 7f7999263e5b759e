"""Host-side guard for the kernels that load tiles from global memory straight into LDS.

Those loads are written as inline assembly that sets M0 (the LDS destination) itself and names M0 as clobbered.  That
is sound as long as the compiler has no use of M0 of its own in those kernels whose definition and use could straddle
one of the loads.  This test compiles the two source files to assembly (no GPU needed) and checks exactly that: every
direct load is immediately preceded by the instruction that sets M0 for it, and M0 appears nowhere else."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_15294_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.parametrize("source", ["attn_prefill_mfma.hip", "scores_prefill_mfma.hip"])
def test_m0_is_only_touched_by_the_direct_loads(tmp_path, source):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not found")
    out = tmp_path / (source + ".s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(CSRC, source)]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    code = [l.strip() for l in out.read_text().splitlines()]
    code = [l for l in code if l and not l.startswith((";", ".", "//")) and not l.endswith(":")]
    loads = [i for i, l in enumerate(code) if l.startswith("global_load_lds_dwordx4")]
    assert len(loads) >= 8, "the direct loads are gone from the generated code"
    setters = set()
    for i in loads:
        prev = code[i - 1]
        assert re.match(r"s_(mov_b32|add_i32|addk_i32|add_u32) m0,", prev), f"M0 is not set right before a direct load: {prev!r}"
        setters.add(i - 1)
    others = [l for i, l in enumerate(code) if re.search(r"\bm0\b", l) and i not in setters]
    assert not others, "M0 is used outside the direct loads:\n" + "\n".join(others[:10])
