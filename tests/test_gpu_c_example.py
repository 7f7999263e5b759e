"""The C example (paper_2502_15294_amd/examples/decode_step.c, built by the package's build step with the host C
compiler) drives scores -> selection -> sparse decode attention through the C boundary alone, in a process of its
own without Python or PyTorch; its results are held to the same bars against the oracle."""
import os
import subprocess

import numpy as np
import pytest

import paper_2502_15294_amd as ra
from oracle import pipeline
from oracle import round_attention as ora
from synth import make_workload
from synth.layout import pack_layer
from synth.workloads import to_bf16_bits

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(ra.__file__), "ra_decode_step")


def test_c_program_runs_the_hot_path(tmp_path):
    assert os.path.exists(EXE), f"{EXE} is missing: build it with `python -m paper_2502_15294_amd.build`"
    w = make_workload("cfg2", B=3, R=9, length=("uniform", 5, 300))
    lam = 0.5
    p0, p1 = pack_layer(w, 0, with_v=False), pack_layer(w, 1)
    n_tok = p0.k.size // (w.Hkv * w.d)
    n_tok_v = p1.v.size // (w.Hkv * w.d)
    inp, outp = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        np.array([w.B, w.R_max, w.Hq, w.Hkv, w.d, int(lam * 1000), n_tok, n_tok_v], dtype=np.int32).tofile(f)
        np.array([p1.max_tokens], dtype=np.int64).tofile(f)
        p1.n_rounds.astype(np.int32).tofile(f)
        p1.seg_len.astype(np.int32).tofile(f)
        p1.seg_off.astype(np.int64).tofile(f)
        p1.seg_off_v.astype(np.int64).tofile(f)
        to_bf16_bits(w.q(0)[:, 0]).tofile(f)
        to_bf16_bits(w.q(1)[:, 0]).tofile(f)
        p0.k.tofile(f)
        p1.k.tofile(f)
        p1.v.tofile(f)
    r = subprocess.run([EXE, str(inp), str(outp)], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stderr
    raw = np.fromfile(outp, dtype=np.uint8)
    BR, rows = w.B * w.R_max, w.B * w.Hq
    o = 0
    S = raw[o:o + 4 * BR].view(np.float32).reshape(w.B, w.R_max); o += 4 * BR
    sel = raw[o:o + 4 * BR].view(np.int32).reshape(w.B, w.R_max); o += 4 * BR
    n_sel = raw[o:o + 4 * w.B].view(np.int32); o += 4 * w.B
    out = raw[o:o + 4 * rows * w.d].view(np.float32).reshape(w.B, w.Hq, w.d); o += 4 * rows * w.d
    lse = raw[o:o + 4 * rows].view(np.float32).reshape(w.B, w.Hq); o += 4 * rows
    assert o == raw.size
    ref = pipeline.run(w, select_params=dict(lam=lam))
    for b, rb in enumerate(ref):
        R = w.n_rounds(b)
        assert np.abs(S[b, :R] - rb.S).max() < 1e-5
        assert rb.info["margin"] > 1e-4
        assert sel[b, :n_sel[b]].tolist() == rb.sel and (sel[b, n_sel[b]:] == -1).all()
        assert ora.row_error(out[b][None], rb.out[1]) < 5e-5
        assert np.allclose(lse[b][None], rb.lse[1], rtol=0, atol=2e-5 * max(1.0, np.abs(rb.lse[1]).max()))
