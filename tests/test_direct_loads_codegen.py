"""Host-side guard for the kernels that load tiles from global memory straight into LDS.

Those loads are written as inline assembly that sets M0 (the LDS destination) itself and names M0 as clobbered.  That
is sound as long as the compiler has no use of M0 of its own in those kernels whose definition and use could straddle
one of the loads.  This test compiles the two source files to assembly (no GPU needed) and checks exactly that: every
direct load is preceded by the instruction that sets M0 for it and by the wait states the hardware leaves to software
(one after a scalar write of M0; five between a vector instruction's write of an SGPR and a vector-memory instruction
that reads it as its base, which the form with a uniform base covers by itself since the compiler does not look into
asm statements), and M0 appears nowhere else.  It also checks that no maximum is hidden in an asm statement."""
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
        # a scalar write of M0 needs one wait state before the instruction that reads it: write, s_nop, load
        nop = re.match(r"s_nop (\d+)$", code[i - 1])
        assert nop, f"no wait state between the write of M0 and a direct load: {code[i - 1]!r}"
        if re.search(r"\bs\[\d+:\d+\]", code[i]):  # uniform base in SGPRs: M0 write + s_nop 3 = five wait states
            assert int(nop.group(1)) >= 3, f"too few wait states before a direct load with a scalar base: {code[i - 1]!r}"
        prev = code[i - 2]
        assert re.match(r"s_(mov_b32|add_i32|addk_i32|add_u32) m0,", prev), f"M0 is not set right before a direct load: {prev!r}"
        setters.add(i - 2)
    others = [l for i, l in enumerate(code) if re.search(r"\bm0\b", l) and i not in setters]
    assert not others, "M0 is used outside the direct loads:\n" + "\n".join(others[:10])


def test_no_vector_arithmetic_hides_in_asm_statements():
    """The compiler inserts the wait states between a matrix-core product and a vector instruction that reads its
    result (and those in front of DPP and lane-swap instructions) only for instructions it can see.  A v_max_f32
    inside an asm statement once read logits of the previous tile that way.  The only asm statements the kernels may
    hold are the direct loads and empty ones (scheduling fences)."""
    bad = []
    for name in sorted(os.listdir(CSRC)):
        if not name.endswith((".hip", ".hpp")):
            continue
        text = open(os.path.join(CSRC, name)).read()
        for m in re.finditer(r"\basm\s*(volatile)?\s*\(\s*\"([^\"]*)\"", text):
            body = m.group(2)
            if body and "global_load_lds_dwordx4" not in body:
                bad.append(f"{name}: {body!r}")
    assert not bad, "asm statements with instructions the compiler cannot see:\n" + "\n".join(bad)
