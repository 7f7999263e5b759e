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


def _kernel_bodies(asm_text):
    """Mangled kernel name -> its instructions (comments, directives and labels dropped)."""
    bodies, name = {}, None
    for line in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name = m.group(1)
            bodies[name] = []
            continue
        l = line.strip()
        if l.startswith(".Lfunc_end"):
            name = None
        if name and l and not l.startswith((";", ".", "//")) and not l.endswith(":"):
            bodies[name].append(l)
    return bodies


def test_score_kernel_finds_its_chunk_by_scalar_loads(tmp_path):
    """The workgroups of the decode-shape score kernel start while their compute unit's vector memory queue is full of
    other workgroups' key tiles, so what tells a workgroup where its chunk lies must not come through that queue: the
    chunk descriptor, the rounds' lengths and the paged walk's block ids are read through the constant address space.
    If they turned into vector loads the results would stay right and the kernel would lose a tenth of its speed;
    this test looks at the generated code instead (no GPU needed)."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not found")
    out = tmp_path / "scores_mfma.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(CSRC, "scores_mfma.hip")]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    bodies = _kernel_bodies(out.read_text())
    kernels = {k: v for k, v in bodies.items() if "scores_mfma_kernel" in k}
    assert len(kernels) == 6, sorted(kernels)          # paged or not x table in LDS / descriptors / scalar table
    for name, code in kernels.items():
        mode = int(re.search(r"ELi(\d)E", name).group(1))
        paged = "ILb1E" in name
        narrow = [l for l in code if re.match(r"global_load_(dword|dwordx2|ushort|ubyte)\b", l)]
        wide = [l for l in code if l.startswith("global_load_dwordx4")]
        assert len(wide) >= 20, f"{name}: the key and query loads are gone"
        if mode == 0:
            assert narrow, f"{name}: the table in LDS is built from vector loads"
            continue
        # descriptors (1) and scalar table (2): every load that is not a key or query load is a scalar one
        assert not narrow, f"{name}: a table or block-table entry is read by a vector load: {narrow[:3]}"
        scalar = [l for l in code if l.startswith("s_load_dword")]
        assert len(scalar) >= (4 if mode == 1 else 32) + (4 if paged else 0), f"{name}: {len(scalar)} scalar loads"
        if mode == 1:
            assert any(l.startswith("s_load_dwordx4") for l in code), f"{name}: no 16-byte descriptor load"
